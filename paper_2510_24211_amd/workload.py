"""Seeded synthetic inputs shaped like the paper's image and video settings.

This module only manufactures INPUT DATA (LM-head weights, hidden states,
toy logits) for the tests, the smoke run and the benchmark.  It contains none
of the decoding method's arithmetic and imports neither the HIP binding nor
the CPU oracle; both sides are handed the same arrays.

The settings mirror the paper's appendix "Experimental Details": Janus-Pro /
LlamaGen-like 24x24 token grids with top-k 1000, Lumina-mGPT-like 48x48 grids
with top-k 2000 and guidance scale 3, Cosmos-like multi-frame video
sequences.  The trained models and datasets are replaced by a drift model:
the hidden state of position i at its a-th evaluation is

    h_{i,a} = bf16( h*_i + amp * decay**a * n_{i,a} ),   a < age_cap
    h_{i,a} = bf16( h*_i ),                               a >= age_cap

with h*_i, n_{i,a} ~ N(0,1).  `a` (the "age") counts the earlier evaluations
of the position, i.e. the Jacobi iterations it has already spent in the
window, so that drafts converge left to right as they do under a real model.
The unconditional row of a CFG pair uses h*_u = 0.9 h*_c + 0.44 eps and its own
noise.  Video: h* of frame f is 0.9 h*_{f-1} + 0.44 eps at the same spatial
index.
"""
from dataclasses import dataclass, replace
import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    L: int
    N: int
    V: int
    d: int                  # 0 => logits are supplied directly (no LM head)
    v_lo: int = 0
    v_hi: int = -1
    top_k: int = 0
    temperature: float = 1.0
    cfg_lambda: float = 0.0
    seed: int = 0
    top_p: float = 0.0      # nucleus mass, 0 => off
    amp: float = 0.3
    decay: float = 0.6
    age_cap: int = 16
    frames: int = 1         # video: N = frames * tokens_per_frame
    w_std: float = 0.02
    logit_std: float = 2.0  # d == 0 only

    def __post_init__(self):
        if self.v_hi < 0:
            object.__setattr__(self, "v_hi", self.V)

    @property
    def C(self):
        return 2 if self.cfg_lambda != 0.0 else 1

    @property
    def n_allowed(self):
        return self.v_hi - self.v_lo

    @property
    def M(self):
        return self.B * self.C * self.L


WORKLOADS = {
    # Tiny toy problem, logits supplied, no LM head.
    "C0": Workload("C0", B=1, L=8, N=64, V=1024, d=0, seed=0, amp=1.0, decay=0.5, age_cap=32),
    # LlamaGen / Janus-shaped image: 24x24 grid, top-k 1000.
    "C1": Workload("C1", B=1, L=32, N=576, V=16384, d=1280, top_k=1000, seed=1),
    # Lumina-mGPT-shaped image: 48x48 grid, CFG 3.0, 8192 allowed image codes, top-k 2000.
    "C2": Workload("C2", B=1, L=32, N=2304, V=65536, d=4096, v_lo=4, v_hi=8196,
                   top_k=2000, cfg_lambda=3.0, seed=2),
    # Same shape with every one of the 65536 ids allowed (full-vocabulary stream).
    "C2-fullV": Workload("C2-fullV", B=1, L=32, N=2304, V=65536, d=4096,
                         top_k=2000, cfg_lambda=3.0, seed=2),
    # Batched image: 16 independent sequences.
    "C3": Workload("C3", B=16, L=32, N=2304, V=65536, d=4096, v_lo=4, v_hi=8196,
                   top_k=2000, cfg_lambda=3.0, seed=3),
    # Video-shaped: 8 frames x 40x40, L=64.
    "C4": Workload("C4", B=2, L=64, N=12800, V=64000, d=4096, top_k=2000,
                   cfg_lambda=3.0, seed=4, decay=0.7, age_cap=24, frames=8),
    # The same video shape with the nucleus filter p = 0.8 in place of top-k.
    "C4-topp": Workload("C4-topp", B=2, L=64, N=12800, V=64000, d=4096, top_p=0.8,
                        cfg_lambda=3.0, seed=4, decay=0.7, age_cap=24, frames=8),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller or otherwise modified copy of a workload (tests).  An id range
    that covered the whole vocabulary keeps covering it when V changes."""
    if "V" in kw and "v_hi" not in kw and w.v_lo == 0 and w.v_hi == w.V:
        kw["v_hi"] = kw["V"]
    return replace(w, **kw)


# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x):
    """Round-to-nearest-even conversion of fp32 values to bf16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def _rng(seed, *tags):
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), *map(int, tags)])))


def lm_head_weight(w: Workload):
    """W ~ N(0, w_std^2) as bf16 bit patterns, [V, d], generated in row blocks
    so that any prefix of rows is independent of V."""
    out = np.empty((w.V, w.d), dtype=np.uint16)
    blk = 4096
    for r0 in range(0, w.V, blk):
        r1 = min(w.V, r0 + blk)
        g = _rng(w.seed, 1, r0 // blk)
        x = g.standard_normal((blk, w.d), dtype=np.float32)[: r1 - r0] * np.float32(w.w_std)
        out[r0:r1] = f32_to_bf16_bits(x)
    return out


class HiddenTable:
    """Hidden states for every (sequence, cond/uncond, position, age).

    rows(b, p0, p1) -> uint16 [C, p1-p0, age_cap+1, d]; generated on demand in
    chunks of `chunk` spatial indices (all frames of a chunk together, because
    of the frame recursion) and cached."""

    chunk = 64

    def __init__(self, w: Workload):
        assert w.d > 0
        self.w = w
        self.per_frame = w.N // w.frames
        assert self.per_frame * w.frames == w.N
        self._cache = {}

    def _gen_chunk(self, b, ch):
        w = self.w
        s0 = ch * self.chunk
        s1 = min(self.per_frame, s0 + self.chunk)
        P, A, d = s1 - s0, w.age_cap, w.d
        g = _rng(w.seed, 2, b, ch)
        out = np.empty((w.C, w.frames, P, A + 1, d), dtype=np.uint16)
        hc_prev = None
        amps = (np.float32(w.amp) * np.float32(w.decay) ** np.arange(A, dtype=np.float32)
                ).astype(np.float32)
        for f in range(w.frames):
            eps = g.standard_normal((P, d), dtype=np.float32)
            hc = eps if f == 0 else np.float32(0.9) * hc_prev + np.float32(0.44) * eps
            hc_prev = hc
            stars = [hc]
            if w.C == 2:
                stars.append(np.float32(0.9) * hc
                             + np.float32(0.44) * g.standard_normal((P, d), dtype=np.float32))
            for c, hs in enumerate(stars):
                n = g.standard_normal((P, A, d), dtype=np.float32)
                out[c, f, :, :A] = f32_to_bf16_bits(hs[:, None, :] + amps[None, :, None] * n)
                out[c, f, :, A] = f32_to_bf16_bits(hs)
        return out

    def _chunk(self, b, ch):
        key = (b, ch)
        if key not in self._cache:
            self._cache[key] = self._gen_chunk(b, ch)
        return self._cache[key]

    def row(self, b, c, pos, age):
        f, s = divmod(pos, self.per_frame)
        ch, o = divmod(s, self.chunk)
        return self._chunk(b, ch)[c, f, o, min(age, self.w.age_cap)]

    def window(self, i_b, ages):
        """h bits [B, C, L, d] for windows starting at i_b[b]; ages[b][s] is the
        age of position i_b[b]+s.  Rows past the sequence end are zero."""
        w = self.w
        h = np.zeros((w.B, w.C, w.L, w.d), dtype=np.uint16)
        for b in range(w.B):
            for s in range(min(w.L, w.N - i_b[b])):
                for c in range(w.C):
                    h[b, c, s] = self.row(b, c, i_b[b] + s, int(ages[b][s]))
        return h

    def full(self, drop_cache=True):
        """The whole table as one array [B, C, N, age_cap+1, d] (benchmark:
        uploaded once, gathered on the device)."""
        w = self.w
        out = np.empty((w.B, w.C, w.N, w.age_cap + 1, w.d), dtype=np.uint16)
        nch = -(-self.per_frame // self.chunk)
        for b in range(w.B):
            for ch in range(nch):
                blk = self._gen_chunk(b, ch) if drop_cache else self._chunk(b, ch)
                s0 = ch * self.chunk
                P = blk.shape[2]
                for f in range(w.frames):
                    out[b, :, f * self.per_frame + s0: f * self.per_frame + s0 + P] = blk[:, f]
        return out


class ToyLogits:
    """d == 0 workloads: fp32 logits z_i + amp*decay**a * e_{i,a} per
    (sequence, position, age), z_i ~ N(0, logit_std^2), e ~ N(0,1)."""

    def __init__(self, w: Workload):
        assert w.d == 0
        self.w = w
        g = _rng(w.seed, 3)
        A, n = w.age_cap, w.n_allowed
        z = g.standard_normal((w.B, w.N, n), dtype=np.float32) * np.float32(w.logit_std)
        e = g.standard_normal((w.B, w.N, A, n), dtype=np.float32)
        amps = (np.float32(w.amp) * np.float32(w.decay) ** np.arange(A, dtype=np.float32)
                ).astype(np.float32)
        self.table = np.empty((w.B, w.N, A + 1, n), dtype=np.float32)
        self.table[:, :, :A] = z[:, :, None, :] + amps[None, None, :, None] * e
        self.table[:, :, A] = z

    def window(self, i_b, ages):
        """fp32 [B, L, |A|] logits for the windows (rows past the end zero)."""
        w = self.w
        z = np.zeros((w.B, w.L, w.n_allowed), dtype=np.float32)
        for b in range(w.B):
            for s in range(min(w.L, w.N - i_b[b])):
                z[b, s] = self.table[b, i_b[b] + s, min(int(ages[b][s]), w.age_cap)]
        return z
