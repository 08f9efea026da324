"""Pins for the oracle's Gumbel-sharing coupling (CPU only).

What the paper and the mathematics fix:
  * Gumbel-max trick: X = argmax(log P + g) is distributed as P (chi-square).
  * GS(P, Q, G) is a coupling: X ~ P and Y ~ Q from one noise vector.
  * Exact diagonal of the joint law, appendix proof of the Gumbel-coupling theorem, Eq. 6:
    Pr[X = Y = k] = 1 / sum_j max(P_j / P_k, Q_j / Q_k); the draws must reproduce it.
  * The theorem's bound Pr[X = Y] >= (1 - TV) / (1 + TV), and Pr[X = Y] <= 1 - TV (no
    coupling beats the maximal one).
  * P = Q gives X = Y always.
  * The race form in which the draw is decided equals the printed argmax form.
  * In the decode loop: the vectorised and the sequential-with-break forms of SCD(pi_GS)
    emit identical tokens; the emitted sequence follows the autoregressive joint law
    (losslessness holds for any admissible drafter); the noise of a position does not
    depend on the iteration (same distribution twice => same draft).
"""
import numpy as np
from scipy import stats

from oracle import gs, philox, scd
from oracle.scd import ScdConfig
from test_oracle_scd import ToyContextModel, _toy


def _pq(V, seed, conc=0.7):
    r = np.random.default_rng(seed)
    return r.dirichlet(np.full(V, conc)), r.dirichlet(np.full(V, conc))


def test_gumbel_max_marginal_and_coupling_validity():
    P, Q = _pq(7, 1)
    n = 40000
    U = np.random.default_rng(2).random((n, 7))
    xy = np.array([gs.gs(P, Q, u) for u in U])
    for col, dist in ((0, P), (1, Q)):
        obs = np.bincount(xy[:, col], minlength=7)
        assert stats.chisquare(obs, dist * n).pvalue > 1e-4


def test_joint_diagonal_matches_eq6_and_bounds():
    for seed in (3, 4, 5):
        P, Q = _pq(6, seed)
        diag = gs.diagonal(P, Q)
        tv = 0.5 * np.abs(P - Q).sum()
        assert diag.sum() >= (1 - tv) / (1 + tv) - 1e-12
        assert diag.sum() <= 1 - tv + 1e-12
        n = 60000
        U = np.random.default_rng(10 + seed).random((n, 6))
        hits = np.zeros(6)
        for u in U:
            x, y = gs.gs(P, Q, u)
            if x == y:
                hits[x] += 1
        # cells: the six diagonal entries and "off the diagonal"
        obs = np.append(hits, n - hits.sum())
        exp = np.append(diag, 1 - diag.sum()) * n
        assert stats.chisquare(obs, exp).pvalue > 1e-4
    # closed form by hand on two ids: P = (a, 1-a), Q = (b, 1-b), a > b:
    # Pr[X=Y=0] = 1 / (1 + (1-b)/b) = b,  Pr[X=Y=1] = 1 / (a/(1-a) + 1) = 1 - a
    d = gs.diagonal([0.7, 0.3], [0.4, 0.6])
    assert np.allclose(d, [0.4, 0.3])


def test_equal_distributions_always_collide_and_zero_support_is_never_drawn():
    P, _ = _pq(9, 6)
    P[[2, 5]] = 0.0
    P /= P.sum()
    U = np.random.default_rng(7).random((3000, 9))
    for u in U:
        x, y = gs.gs(P, P, u)
        assert x == y and P[x] > 0


def test_race_form_equals_printed_argmax_form():
    r = np.random.default_rng(8)
    bad = 0
    for _ in range(4000):
        V = int(r.integers(2, 40))
        p = r.dirichlet(np.full(V, 0.5))
        u = philox.u01_from_bits(r.integers(0, 2 ** 32, size=V, dtype=np.uint64))
        w, score = gs.draw(p, u)
        if w != gs.draw_definition(p, u):
            assert gs.flag(p, u, w)          # only a numerically fragile draw may differ
            bad += 1
        # ties go to the lowest id
        assert w == int(np.flatnonzero(score == score.min())[0])
    assert bad <= 2


def test_flag_marks_close_races_only():
    p = np.array([0.5, 0.5])
    # E0/p0 vs E1/p1 with E = -ln U: equal uniforms => exact tie => fragile
    assert gs.flag(p, np.array([0.3, 0.3]), 0)
    assert not gs.flag(p, np.array([0.9, 0.1]), 0)


def test_vectorised_equals_sequential_gs():
    cases = [_toy(), _toy(N=37, L=5, seed=3), _toy(N=20, L=1, seed=4), _toy(N=9, L=16, seed=5),
             _toy(N=30, L=8, seed=6, top_k=50), _toy(N=24, L=4, seed=8, B=3)]
    for w, cfg, model in cases:
        cfg.coupling = "gs"
        o = scd.decode(cfg, model)
        out, nfe, hist = scd.decode_sequential(cfg, model)
        assert np.array_equal(o.out, out)
        assert o.t == nfe and o.accept_hist == hist
        for b in range(cfg.B):
            assert sum(hist[b]) == cfg.N and all(1 <= a <= cfg.L for a in hist[b])
    # and the two couplings are different samplers: same seed, different tokens somewhere
    w, cfg, model = _toy()
    mc = scd.decode(cfg, model).out
    cfg.coupling = "gs"
    assert not np.array_equal(mc, scd.decode(cfg, model).out)


def test_end_to_end_lossless_gs():
    V, N = 3, 3
    model = ToyContextModel(V, N, seed=7)
    want = model.ar_joint(0)
    for L in (2, 3):
        counts = {k: 0 for k in want}
        runs = 12000
        for r in range(runs):
            cfg = ScdConfig(B=1, L=L, N=N, V=V, seed=700000 * L + r, coupling="gs")
            counts[tuple(int(x) for x in scd.decode(cfg, model).out[0])] += 1
        keys = list(want)
        obs = np.array([counts[k] for k in keys], dtype=np.float64)
        exp = np.array([want[k] for k in keys]) * runs
        assert stats.chisquare(obs, exp).pvalue > 1e-4, L


def test_noise_depends_on_the_position_only():
    # the same distribution evaluated in two different iterations gives the same Gumbel draft
    w, cfg, model = _toy(N=24, L=6)
    cfg.coupling = "gs"
    o = scd.ScdOracle(cfg)
    z = [np.stack([wl_row for wl_row in model(0, 0, 6, None, 0, np.zeros(6, dtype=int))])]
    plan = o.evaluate(z)
    g0 = [r["g"] for r in o.sample(plan)[0]]
    o.t[0] = 5                                   # a later iteration, same positions
    g1 = [r["g"] for r in o.sample(plan)[0]]
    assert g0 == g1
    # while the MRS draws do depend on it (different accept uniforms)
    u0 = philox.uniform_scalar(cfg.seed, 0, 3, 0, philox.STREAM_ACCEPT)
    u5 = philox.uniform_scalar(cfg.seed, 0, 3, 5, philox.STREAM_ACCEPT)
    assert u0 != u5
    # match rate of consecutive Gumbel drafts inside a decode obeys the theorem's bound on average
    o = scd.ScdOracle(cfg)
    lhs = rhs = 0.0
    while not o.done():
        i, Lw = o.window(0)
        ages = o.age[0, i:i + Lw].copy()
        plan = o.evaluate([model(0, i, Lw, None, o.t[0], ages)])
        res = o.sample(plan)
        for s in range(Lw):
            if i + s in o.q[0]:                  # the position had a Gumbel draft from q before
                p, q = plan[0][s]["p"], o.q[0][i + s]
                tv = 0.5 * np.abs(p - q).sum()
                lhs += float(res[0][s]["g"] == o.X[0, i + s])
                rhs += (1 - tv) / (1 + tv)
        o.commit(plan, res)
    assert lhs >= rhs - 3.0 * np.sqrt(max(rhs, 1.0))


# ------------------------------------------------------------------ alpha-coupling
def test_alpha_one_is_scd_and_forms_agree_for_every_alpha():
    for coupling in ("mc", "gs"):
        w, cfg, model = _toy(N=40, L=8, seed=41)
        cfg.coupling = coupling
        base = scd.decode(cfg, model).out.copy()
        cfg.alpha = 1.0
        assert np.array_equal(scd.decode(cfg, model).out, base)
        for alpha in (0.0, 0.3, 0.8):
            cfg.alpha = alpha
            o = scd.decode(cfg, model)
            out, nfe, hist = scd.decode_sequential(cfg, model)
            assert np.array_equal(o.out, out) and o.t == nfe and o.accept_hist == hist
        cfg.alpha = 0.0
        assert not np.array_equal(scd.decode(cfg, model).out, base)


def test_alpha_mixture_collision_probability():
    # Sec. 5.3: pi^alpha = alpha pi_cpl + (1 - alpha) pi_ind, so the probability that a redraft
    # equals the previous draft is alpha * C_cpl + (1 - alpha) * sum_v p_v q_v.  Measured over a
    # decode on positions whose previous draft came from q (survivors of an earlier redraft).
    for alpha in (0.0, 0.5):
        lhs = rhs = 0.0
        var = 0.0
        for seed in range(40, 52):
            w, cfg, model = _toy(N=48, L=8, seed=seed, V=24)
            cfg.alpha = alpha
            o = scd.ScdOracle(cfg)
            while not o.done():
                i, Lw = o.window(0)
                plan = o.evaluate([model(0, i, Lw, None, o.t[0], o.age[0, i:i + Lw].copy())])
                res = o.sample(plan)
                for s in range(Lw):
                    if i + s in o.q[0]:
                        p, q = plan[0][s]["p"], o.q[0][i + s]
                        c_mc = 1 - 0.5 * np.abs(p - q).sum()          # maximal coupling: 1 - TV
                        pr = alpha * c_mc + (1 - alpha) * float((p * q).sum())
                        lhs += float(res[0][s]["next"] == o.X[0, i + s])
                        rhs += pr
                        var += pr * (1 - pr)
                o.commit(plan, res)
        assert abs(lhs - rhs) <= 4.0 * np.sqrt(var) + 1.0, (alpha, lhs, rhs)


def test_end_to_end_lossless_for_alpha_below_one():
    V, N = 3, 3
    model = ToyContextModel(V, N, seed=7)
    want = model.ar_joint(0)
    for alpha, coupling in ((0.0, "mc"), (0.5, "gs")):
        counts = {k: 0 for k in want}
        runs = 10000
        for r in range(runs):
            cfg = ScdConfig(B=1, L=3, N=N, V=V, seed=3100000 + r, coupling=coupling, alpha=alpha)
            counts[tuple(int(x) for x in scd.decode(cfg, model).out[0])] += 1
        keys = list(want)
        obs = np.array([counts[k] for k in keys], dtype=np.float64)
        exp = np.array([want[k] for k in keys]) * runs
        assert stats.chisquare(obs, exp).pvalue > 1e-4, (alpha, coupling)
