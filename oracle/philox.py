"""Philox4x32-10 counter-based generator (oracle side; test infrastructure only).

The algorithm is the public one of Salmon, Moraes, Dror and Shaw, "Parallel
random numbers: as easy as 1, 2, 3" (SC'11): a 4x32-bit counter and a 2x32-bit
key go through ten rounds; each round multiplies two counter words by fixed
odd constants, mixes the high halves with the other two words and the key,
and the key is bumped by Weyl constants between rounds.

The paper's method needs "u ~ U[0,1]" (Alg. 1, step 1) and a draw from the
residual distribution (Alg. 1, last step); it does not say how the numbers are
produced beyond hashing of a token's global index (Sec. 4.3).  This build keys
every draw on (seed, sequence, position, iteration, stream, vocab id) so that
the CPU and the GPU draw the same numbers in any evaluation order.

Everything is NumPy uint64 arithmetic masked to 32 bits; arrays broadcast.
"""
import numpy as np

M0 = np.uint64(0xD2511F53)
M1 = np.uint64(0xCD9E8D57)
W0 = np.uint64(0x9E3779B9)
W1 = np.uint64(0xBB67AE85)
MASK = np.uint64(0xFFFFFFFF)
SH32 = np.uint64(32)

# stream ids (low byte of counter word 3)
STREAM_INIT = 0    # initial draft token of a never-evaluated position
STREAM_ACCEPT = 1  # the uniform of the accept test
STREAM_RESID = 2   # one uniform per vocab id for the residual race
STREAM_GUMBEL = 3  # one uniform per vocab id for the shared Gumbel noise of a position
STREAM_ALPHA = 4   # the Bernoulli(alpha) switch of the alpha-coupling
STREAM_INDEP = 5   # one uniform per vocab id for an independent draw from p


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox rounds.  All arguments broadcastable integer arrays holding
    32-bit values; returns four uint64 arrays with values < 2**32."""
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(
        *[np.asarray(a, dtype=np.uint64) & MASK for a in (c0, c1, c2, c3, k0, k1)])
    for _ in range(10):
        p0 = M0 * c0            # < 2**64, exact in uint64
        p1 = M1 * c2
        hi0, lo0 = p0 >> SH32, p0 & MASK
        hi1, lo1 = p1 >> SH32, p1 & MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def philox4x32_10_int(c0, c1, c2, c3, k0, k1):
    """The same ten rounds on plain Python integers (scalar draws)."""
    for _ in range(10):
        p0 = 0xD2511F53 * c0
        p1 = 0xCD9E8D57 * c2
        c0, c1, c2, c3 = (p1 >> 32) ^ c1 ^ k0, p1 & 0xFFFFFFFF, (p0 >> 32) ^ c3 ^ k1, p0 & 0xFFFFFFFF
        k0 = (k0 + 0x9E3779B9) & 0xFFFFFFFF
        k1 = (k1 + 0xBB67AE85) & 0xFFFFFFFF
    return c0, c1, c2, c3


def seed_key(seed):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return seed & 0xFFFFFFFF, seed >> 32


def counter_word3(b, stream):
    return (int(b) << 8) | int(stream)


def u01_from_bits(x):
    """Map 32 random bits to a uniform strictly inside (0,1) that is exactly
    representable in fp32: u = ((x >> 9) + 1/2) * 2**-23  (23 random bits).
    Returned as float64 (the value is identical in float32)."""
    x = np.asarray(x, dtype=np.uint64)
    return ((x >> np.uint64(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def uniform_scalar(seed, b, pos, it, stream):
    """One uniform for (sequence b, position pos, iteration it): lane 0 of the
    block with counter (0, pos, it, b<<8|stream)."""
    k0, k1 = seed_key(seed)
    r = philox4x32_10_int(0, int(pos), int(it), counter_word3(b, stream), k0, k1)
    return ((r[0] >> 9) + 0.5) * (2.0 ** -23)


def uniform_per_vocab(seed, b, pos, it, stream, n):
    """n uniforms, one per vocab offset v = 0..n-1: offset v takes lane v&3 of
    the block with counter (v>>2, pos, it, b<<8|stream)."""
    k0, k1 = seed_key(seed)
    nb = (n + 3) // 4
    r = philox4x32_10(np.arange(nb, dtype=np.uint64), pos, it,
                      counter_word3(b, stream), k0, k1)
    bits = np.stack(r, axis=1).reshape(-1)[:n]
    return u01_from_bits(bits)


def init_token(seed, b, pos, n_allowed):
    """Uniform draw from {0..n_allowed-1} for a never-evaluated position:
    floor(r * n_allowed / 2**64) with r the 64-bit word (lane0<<32 | lane1) of
    the block with counter (0, pos, 0, b<<8|INIT).  Bias <= n_allowed/2**64."""
    k0, k1 = seed_key(seed)
    r = philox4x32_10_int(0, int(pos), 0, counter_word3(b, STREAM_INIT), k0, k1)
    r64 = (r[0] << 32) | r[1]
    return (r64 * int(n_allowed)) >> 64
