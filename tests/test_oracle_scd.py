"""Pins for the oracle's SCD decode loop (CPU only).

  * L = 1 reduces to plain autoregressive sampling (one token per iteration,
    each drawn from p_i).
  * End-to-end losslessness (Thm 4.2): on a context-dependent toy model the
    joint law of the emitted sequence equals the autoregressive joint, for
    every window length -- this is the test that catches an off-by-one in the
    accept count, a mis-keyed draw or a stale draft distribution.
  * p == q gives full acceptance (ceil(N/L) iterations after the first).
  * The vectorised form and the sequential-with-break form emit identical
    tokens (Sec. 4.3).
  * The match rate of the coupled redraft against the previous draft equals
    1 - D_TV (Thm 4.3).
"""
import itertools

import numpy as np
from scipy import special, stats

from oracle import scd
from oracle.scd import ScdConfig
from paper_2510_24211_amd import workload as wl


# --------------------------------------------------------------------------
class ToyContextModel:
    """Logits of position j are a fixed random function of ALL earlier tokens."""

    def __init__(self, V, N, seed, scale=1.5):
        g = np.random.default_rng(seed)
        self.V, self.N = V, N
        self.tab = {}
        for j in range(N):
            for pre in itertools.product(range(V), repeat=j):
                self.tab[pre] = (g.standard_normal(V) * scale).astype(np.float32)

    def __call__(self, b, i, Lw, toks, t, age):
        return np.stack([self.tab[tuple(int(x) for x in toks[: i + s])] for s in range(Lw)])

    def ar_joint(self, top_k=0, top_p=0.0):
        J = {}
        for seq in itertools.product(range(self.V), repeat=self.N):
            pr = 1.0
            for j in range(self.N):
                z = self.tab[seq[:j]].astype(np.float64)
                if top_k:
                    thr = np.sort(z)[::-1][top_k - 1]
                    z = np.where(z >= thr, z, -np.inf)
                pz = special.softmax(z)
                if top_p:          # nucleus: most probable ids until their mass reaches top_p
                    order = np.argsort(-pz)
                    ncut = int(np.searchsorted(np.cumsum(pz[order]), top_p)) + 1
                    keep = np.zeros(self.V, dtype=bool)
                    keep[order[:ncut]] = True
                    pz = np.where(keep, pz, 0.0) / pz[keep].sum()
                pr *= pz[seq[j]]
            J[seq] = pr
        return J


def _joint_test(L, top_k, runs, seed0, top_p=0.0):
    V, N = 3, 3
    model = ToyContextModel(V, N, seed=7)
    want = model.ar_joint(top_k, top_p)
    counts = {k: 0 for k in want}
    nfe = 0
    for r in range(runs):
        cfg = ScdConfig(B=1, L=L, N=N, V=V, top_k=top_k, top_p=top_p, seed=seed0 + r)
        o = scd.decode(cfg, model)
        counts[tuple(int(x) for x in o.out[0])] += 1
        nfe += o.t[0]
    keys = [k for k in want if want[k] > 0]
    assert sum(counts[k] for k in want if want[k] == 0) == 0
    obs = np.array([counts[k] for k in keys], dtype=np.float64)
    exp = np.array([want[k] for k in keys])
    p = stats.chisquare(obs, exp / exp.sum() * obs.sum()).pvalue
    return p, nfe / runs


def test_L1_is_autoregressive_sampling():
    p, mean_nfe = _joint_test(L=1, top_k=0, runs=6000, seed0=1000)
    assert mean_nfe == 3.0            # one token per iteration, always
    assert p > 1e-4


def test_end_to_end_lossless_L2_L3():
    for L in (2, 3):
        p, mean_nfe = _joint_test(L=L, top_k=0, runs=12000, seed0=50000 * L)
        assert p > 1e-4, (L, p)
        assert mean_nfe < 3.0         # speculation does save iterations


def test_end_to_end_lossless_with_topk():
    p, _ = _joint_test(L=3, top_k=2, runs=8000, seed0=900000)
    assert p > 1e-4


def test_end_to_end_lossless_with_nucleus():
    """The nucleus filter changes the target distribution, nothing else: the decode samples
    the autoregressive model whose every conditional is cut to its most probable ids holding
    60 % of the mass (computed here with sort / cumsum / searchsorted)."""
    p, _ = _joint_test(L=3, top_k=0, runs=8000, seed0=1300000, top_p=0.6)
    assert p > 1e-4


# --------------------------------------------------------------------------
def _toy(name="C0", **kw):
    w = wl.scaled(wl.WORKLOADS[name], **kw)
    toy = wl.ToyLogits(w)
    cfg = ScdConfig(B=w.B, L=w.L, N=w.N, V=w.V, v_lo=w.v_lo, v_hi=w.v_hi, top_k=w.top_k,
                    top_p=w.top_p, temperature=w.temperature, cfg_lambda=0.0, seed=w.seed)

    def model(b, i, Lw, toks, t, age):
        return np.stack([toy.table[b, i + s, min(int(age[s]), w.age_cap)] for s in range(Lw)])
    return w, cfg, model


def test_identical_distributions_accept_everything():
    w, cfg, _ = _toy(N=40, L=8)
    toy = wl.ToyLogits(w)
    const = lambda b, i, Lw, toks, t, age: np.stack([toy.table[b, i + s, w.age_cap] for s in range(Lw)])
    o = scd.decode(cfg, const)
    # after a position's first evaluation p == q bit for bit => it is accepted for sure;
    # only a window's never-evaluated positions can reject.
    for b in range(cfg.B):
        assert sum(o.accept_hist[b]) == cfg.N
    # with a fully evaluated window (age >= 1 everywhere) acceptance is total:
    o2 = scd.ScdOracle(cfg)
    z = [np.stack([toy.table[0, s, w.age_cap] for s in range(8)])]
    plan = o2.evaluate(z)
    for s in range(8):                      # pretend these positions were evaluated before
        o2.q[0][s] = plan[0][s]["p"]
        o2.X[0, s] = int(np.argmax(plan[0][s]["p"]))
    res = o2.sample(plan)
    assert all(r["k"] == 1 for r in res[0])
    assert o2.commit(plan, res) == [8]


def test_vectorised_equals_sequential_on_C0_and_small_cases():
    cases = [_toy(), _toy(N=37, L=5, seed=3), _toy(N=20, L=1, seed=4), _toy(N=9, L=16, seed=5),
             _toy(N=30, L=8, seed=6, top_k=50), _toy(N=24, L=4, seed=8, B=3),
             _toy(N=30, L=8, seed=9, top_p=0.8), _toy(N=30, L=8, seed=10, top_k=50, top_p=0.5)]
    for w, cfg, model in cases:
        o = scd.decode(cfg, model)
        out, nfe, hist = scd.decode_sequential(cfg, model)
        assert np.array_equal(o.out, out)
        assert o.t == nfe
        assert o.accept_hist == hist
        assert (o.out >= cfg.v_lo).all() and (o.out < cfg.v_hi).all()
        for b in range(cfg.B):
            assert sum(hist[b]) == cfg.N and all(1 <= a <= cfg.L for a in hist[b])


def test_vectorised_equals_sequential_with_every_option_combined():
    """Top-k, nucleus, both couplings and the alpha switch together: the two forms of the
    decode reach each processor through different functions and must emit the same tokens."""
    for coupling, alpha, kw in [("gs", 1.0, dict(N=24, L=6, seed=51, top_k=40, top_p=0.7)),
                                ("mc", 0.4, dict(N=24, L=6, seed=52, top_p=0.9)),
                                ("gs", 0.6, dict(N=20, L=5, seed=53, top_k=30, top_p=0.5, B=2))]:
        w, cfg, model = _toy(**kw)
        cfg.coupling, cfg.alpha = coupling, alpha
        o = scd.decode(cfg, model)
        out, nfe, hist = scd.decode_sequential(cfg, model)
        assert np.array_equal(o.out, out) and o.t == nfe and o.accept_hist == hist


def test_C0_decodes_and_speculation_helps():
    w, cfg, model = _toy()
    o = scd.decode(cfg, model)
    assert o.done() and (o.out >= 0).all()
    assert o.t[0] < cfg.N            # fewer iterations than tokens
    assert o.positions_verified == sum(min(cfg.L, cfg.N - i) for i in
                                       np.cumsum([0] + o.accept_hist[0][:-1]))


def test_coupled_redraft_match_rate_is_one_minus_tv():
    """Thm 4.3 inside the decode loop: over the positions right of the first
    rejection the redraft equals the previous draft with probability 1 - TV."""
    w, cfg, model = _toy(N=64, L=8)
    hits, expect, var = 0.0, 0.0, 0.0
    for seed in range(60):
        cfg.seed = seed
        o = scd.ScdOracle(cfg)
        while not o.done():
            i, Lw = o.window(0)
            z = [model(0, i, Lw, None, o.t[0], o.age[0, i:i + Lw].copy())]
            plan = o.evaluate(z)
            res = o.sample(plan)
            for s in range(Lw):
                q = o.draft_row(0, i + s)
                tv = 0.5 * np.abs(plan[0][s]["p"] - q).sum()
                hits += res[0][s]["y"] == o.X[0, i + s]
                expect += 1 - tv
                var += tv * (1 - tv)
            o.commit(plan, res)
    assert abs(hits - expect) < 5 * np.sqrt(var)


def test_resume_from_saved_state_is_bit_identical():
    import copy
    w, cfg, model = _toy(N=48, L=8, seed=21)
    whole = scd.decode(cfg, model)
    o = scd.ScdOracle(cfg)
    for _ in range(5):
        i, Lw = o.window(0)
        o.step([model(0, i, Lw, None, o.t[0], o.age[0, i:i + Lw].copy())])
    o2 = copy.deepcopy(o)
    while not o2.done():
        i, Lw = o2.window(0)
        o2.step([model(0, i, Lw, None, o2.t[0], o2.age[0, i:i + Lw].copy())])
    assert np.array_equal(whole.out, o2.out) and whole.t == o2.t
