"""Pins for the oracle's random-number layer (CPU only)."""
import os

import numpy as np
from scipy import stats

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        rows.append([int(x, 16) for x in line.split()])
    return rows


def test_known_answers_array_and_scalar():
    for row in _kat():
        c, k, want = row[:4], row[4:6], row[6:]
        got_a = [int(x) for x in philox.philox4x32_10(*c, *k)]
        got_s = list(philox.philox4x32_10_int(*c, *k))
        assert got_a == want
        assert got_s == want


def test_two_implementations_agree_on_random_inputs():
    g = np.random.default_rng(123)
    n = 20000
    args = [g.integers(0, 2 ** 32, n, dtype=np.uint64) for _ in range(6)]
    arr = np.stack(philox.philox4x32_10(*args), axis=1)
    for idx in g.integers(0, n, 300):
        got = philox.philox4x32_10_int(*[int(a[idx]) for a in args])
        assert [int(x) for x in arr[idx]] == list(got)


def test_uniform_mapping_is_open_interval_and_fp32_exact():
    bits = np.array([0, 1, 511, 512, 2 ** 31, 2 ** 32 - 1], dtype=np.uint64)
    u = philox.u01_from_bits(bits)
    assert u.min() == 2.0 ** -24 and u.max() == 1 - 2.0 ** -24
    assert np.all(u.astype(np.float32).astype(np.float64) == u)
    g = np.random.default_rng(5)
    u = philox.u01_from_bits(g.integers(0, 2 ** 32, 100000, dtype=np.uint64))
    assert np.all((u > 0) & (u < 1))
    assert np.all(u.astype(np.float32).astype(np.float64) == u)


def test_scalar_and_per_vocab_streams_use_the_documented_counters():
    seed, b, pos, it = 0x1234567890ABCDEF, 3, 77, 5
    k0, k1 = philox.seed_key(seed)
    assert (k0, k1) == (0x90ABCDEF, 0x12345678)
    r = philox.philox4x32_10_int(0, pos, it, (b << 8) | philox.STREAM_ACCEPT, k0, k1)
    assert philox.uniform_scalar(seed, b, pos, it, philox.STREAM_ACCEPT) == \
        ((r[0] >> 9) + 0.5) * 2.0 ** -23
    U = philox.uniform_per_vocab(seed, b, pos, it, philox.STREAM_RESID, 11)
    for v in range(11):
        r = philox.philox4x32_10_int(v >> 2, pos, it, (b << 8) | philox.STREAM_RESID, k0, k1)
        assert U[v] == ((r[v & 3] >> 9) + 0.5) * 2.0 ** -23


def test_uniformity_chi_square():
    U = philox.uniform_per_vocab(42, 0, 1, 2, philox.STREAM_RESID, 400000)
    counts, _ = np.histogram(U, bins=64, range=(0, 1))
    assert stats.chisquare(counts).pvalue > 1e-4
    # different positions / iterations / streams decorrelate
    a = philox.uniform_per_vocab(42, 0, 1, 2, philox.STREAM_RESID, 50000)
    for other in (philox.uniform_per_vocab(42, 0, 2, 2, philox.STREAM_RESID, 50000),
                  philox.uniform_per_vocab(42, 0, 1, 3, philox.STREAM_RESID, 50000),
                  philox.uniform_per_vocab(42, 1, 1, 2, philox.STREAM_RESID, 50000),
                  philox.uniform_per_vocab(43, 0, 1, 2, philox.STREAM_RESID, 50000)):
        assert abs(np.corrcoef(a, other)[0, 1]) < 0.02


def test_init_token_uniform_over_allowed():
    n = 7
    toks = [philox.init_token(9, 0, j, n) for j in range(21000)]
    assert min(toks) == 0 and max(toks) == n - 1
    assert stats.chisquare(np.bincount(toks, minlength=n)).pvalue > 1e-4
    # a power-of-two range reads the top bits of the 64-bit word
    k0, k1 = philox.seed_key(9)
    r = philox.philox4x32_10_int(0, 5, 0, philox.STREAM_INIT, k0, k1)
    assert philox.init_token(9, 0, 5, 1024) == r[0] >> 22
