"""Pins for the oracle's per-position statistics (CPU only): closed forms,
inequalities the paper proves, and Monte-Carlo agreement with the oracle's own
samplers (which are pinned elsewhere)."""
import numpy as np

from oracle import diagnostics as dg
from oracle import mrs as omrs
from oracle import philox


def _rand_dist(g, n, sharp=1.0):
    z = g.standard_normal(n) * sharp
    e = np.exp(z - z.max())
    return e / e.sum()


def test_closed_forms():
    u4 = np.full(4, 0.25)
    assert dg.acceptance_rate(u4, u4) == 1.0
    assert abs(dg.renyi2_entropy(u4) - np.log(4)) < 1e-15            # uniform over k ids: H_2 = log k
    assert abs(dg.collision_probability(u4, u4) - 0.25) < 1e-15
    a = np.array([1.0, 0.0, 0.0])
    b = np.array([0.0, 1.0, 0.0])
    assert dg.acceptance_rate(a, b) == 0.0 and dg.collision_probability(a, b) == 0.0   # disjoint
    p = np.array([0.5, 0.3, 0.2])
    q = np.array([0.2, 0.3, 0.5])
    assert abs(dg.total_variation(p, q) - 0.3) < 1e-15               # by hand: (0.3 + 0 + 0.3) / 2
    assert abs(dg.acceptance_rate(p, q) - np.minimum(p, q).sum()) < 1e-15   # 1 - TV = sum min
    assert abs(dg.collision_probability(p, q) - (0.10 + 0.09 + 0.10)) < 1e-15
    assert dg.hamming([1, 2, 3, 4], [1, 5, 3, 0]) == 2 and dg.hamming([], []) == 0


def test_collision_bound_holds_and_is_tight_for_equal_distributions():
    g = np.random.default_rng(0)
    for _ in range(200):
        n = int(g.integers(2, 50))
        p, q = _rand_dist(g, n, 2.0), _rand_dist(g, n, 2.0)
        s = dg.row_statistics(p, q)
        assert s[1] <= dg.collision_bound(p, q) * (1 + 1e-12)        # Prop. SJD Collision Probability
        assert abs(dg.collision_bound(p, q) - np.sqrt(s[2] * s[3])) < 1e-12
        assert s[1] <= s[0] + 1e-15                                   # sum p q <= sum min(p, q)
        assert abs(dg.collision_probability(p, p) - dg.collision_bound(p, p)) < 1e-12   # equality at p = q


def test_acceptance_rate_is_the_accept_frequency_of_mrs():
    g = np.random.default_rng(1)
    n = 6
    p, q = _rand_dist(g, n), _rand_dist(g, n)
    want = dg.acceptance_rate(p, q)
    runs, acc = 20000, 0
    for r in range(runs):
        x = int(g.choice(n, p=q))
        u = philox.uniform_scalar(77, 0, r, 0, philox.STREAM_ACCEPT)
        acc += omrs.mrs(p, q, x, u, lambda r=r: philox.uniform_per_vocab(77, 0, r, 0, philox.STREAM_RESID, n))["k"]
    assert abs(acc / runs - want) < 4 * np.sqrt(want * (1 - want) / runs)


def test_collision_probability_is_the_match_frequency_of_independent_draws():
    g = np.random.default_rng(2)
    n = 5
    p, q = _rand_dist(g, n), _rand_dist(g, n)
    want = dg.collision_probability(p, q)
    runs = 40000
    hits = int((g.choice(n, size=runs, p=p) == g.choice(n, size=runs, p=q)).sum())
    assert abs(hits / runs - want) < 4 * np.sqrt(want * (1 - want) / runs)


def test_hamming_of_a_decode_follows_the_coupling():
    """Over a decode, the drafts that change per iteration are, in expectation, the surviving
    rows' 1 - beta under the maximal coupling (Thm. maximal coupling: match probability
    1 - D_TV) and 1 - C under independent redrafts (alpha = 0; Prop. SJD collision
    probability) -- and the first is far smaller (Sec. 5.3: the Hamming distance falls as alpha
    grows)."""
    from oracle import scd
    from paper_2510_24211_amd import workload as wl
    w = wl.scaled(wl.WORKLOADS["C0"], N=160, L=16, V=256, seed=41)
    toy = wl.ToyLogits(w)
    frac = {}
    for alpha in (1.0, 0.0):
        cfg = scd.ScdConfig(B=1, L=w.L, N=w.N, V=w.V, seed=w.seed, alpha=alpha)
        o = scd.ScdOracle(cfg)
        changed = surv = 0
        expect = var = 0.0
        while not o.done():
            i, Lw = o.window(0)
            z = np.stack([toy.table[0, i + s, min(int(o.age[0, i + s]), w.age_cap)] for s in range(Lw)])
            plan, res, acc = o.step([z])
            c, n_s = o.last_hamming[0]
            changed += c
            surv += n_s
            for s in range(acc[0], Lw):                 # survivors
                beta, coll = res[0][s]["stats"][:2]
                pm = beta if alpha == 1.0 else coll      # probability that the redraft equals the draft
                expect += 1 - pm
                var += pm * (1 - pm)
        assert surv > 300
        frac[alpha] = changed / surv
        assert abs(changed - expect) < 4.5 * np.sqrt(var) + 1, (alpha, changed, expect)
    assert frac[1.0] < 0.6 * frac[0.0]


def test_multi_step_hamming():
    """Hamm(t - n, t) over the positions common to both windows (Sec. 5.3 "Multi-Step
    Behavior").  n = 1 is the count of changed survivors (computed separately); with
    independent redrafts (alpha = 0) drafts n iterations apart are independent draws, so the
    changed fraction is about 1 - C for every n; under the maximal coupling changes accumulate:
    the fraction grows with n but stays below the independent one."""
    from oracle import scd
    from paper_2510_24211_amd import workload as wl
    w = wl.scaled(wl.WORKLOADS["C0"], N=600, L=32, V=64, seed=43, amp=2.0, decay=0.85, age_cap=24)
    toy = wl.ToyLogits(w)
    frac = {}
    for alpha in (1.0, 0.0):
        cfg = scd.ScdConfig(B=1, L=w.L, N=w.N, V=w.V, seed=w.seed, alpha=alpha)
        o = scd.ScdOracle(cfg)
        tot = np.zeros((3, 2))
        coll = []
        while not o.done():
            i, Lw = o.window(0)
            z = np.stack([toy.table[0, i + s, min(int(o.age[0, i + s]), w.age_cap)] for s in range(Lw)])
            plan, res, acc = o.step([z])
            assert o.last_hamming_multi[0][0] == o.last_hamming[0]
            tot += np.array(o.last_hamming_multi[0])
            coll += [res[0][s]["stats"][1] for s in range(acc[0], Lw) if o.age[0, i + s] > 1]
        frac[alpha] = tot[:, 0] / tot[:, 1]
        assert (tot[:, 1] > 400).all(), tot
        if alpha == 0.0:
            assert np.abs(frac[alpha] - (1 - np.mean(coll))).max() < 0.03
    assert frac[1.0][0] < frac[1.0][1] < frac[1.0][2] < frac[0.0].min()
