"""Pins for the oracle's Modified Rejection Sampling (CPU only).

Prop. 2.1: Y ~ P and Pr[accept] = sum_x min(p, q) = 1 - D_TV.
Thm 4.3 (proof): joint law f(x, y) = q(x) (a(x) delta_x(y) + (1 - a(x)) r(y)),
a(x) = min(1, p(x)/q(x)), r = norm(max(0, p - q)); Pr[X = Y] = 1 - D_TV.
"""
import numpy as np
from scipy import stats

from oracle import mrs, philox


def _dists(V, rng, disjoint=False, sparse=False):
    p = rng.gamma(0.7, size=V)
    q = rng.gamma(0.7, size=V)
    if disjoint:
        p[: V // 2] = 0
        q[V // 2:] = 0
    if sparse:
        p[rng.integers(0, V, V // 3)] = 0
    return p / p.sum(), q / q.sum()


def _run(p, q, n, seed):
    """n MRS calls with X ~ q by inverse CDF on an INIT-stream uniform."""
    V = p.size
    k0, k1 = philox.seed_key(seed)
    r = philox.philox4x32_10(0, np.arange(n), 0, philox.STREAM_INIT, k0, k1)
    ux = philox.u01_from_bits(r[0])
    X = np.minimum(np.searchsorted(np.cumsum(q), ux, side="right"), V - 1)
    # searchsorted may land on a zero-probability id at cumsum plateaus
    for i in np.nonzero(q[X] == 0)[0]:
        X[i] = np.nonzero(q > 0)[0][np.searchsorted(np.cumsum(q[q > 0]), ux[i], side="right")]
    r = philox.philox4x32_10(0, np.arange(n), 1, philox.STREAM_ACCEPT, k0, k1)
    ua = philox.u01_from_bits(r[0])
    Y = np.empty(n, dtype=np.int64)
    K = np.empty(n, dtype=np.int64)
    for i in range(n):
        out = mrs.mrs(p, q, int(X[i]), ua[i],
                      lambda i=i: philox.uniform_per_vocab(seed, 0, i, 1, philox.STREAM_RESID, V))
        Y[i], K[i] = out["y"], out["k"]
    return X, Y, K


def _closed_form_joint(p, q):
    V = p.size
    with np.errstate(divide="ignore", invalid="ignore"):
        a = np.where(q > 0, np.minimum(1.0, p / q), 0.0)
    r = np.maximum(0.0, p - q)
    r = r / r.sum() if r.sum() > 0 else r
    return q[:, None] * (a[:, None] * np.eye(V) + (1 - a)[:, None] * r[None, :])


def _chi2_p(counts, probs):
    m = probs > 0
    assert counts[~m].sum() == 0, "mass on an impossible outcome"
    return stats.chisquare(counts[m], probs[m] / probs[m].sum() * counts[m].sum()).pvalue


def test_marginal_accept_rate_and_joint():
    rng = np.random.default_rng(11)
    n = 40000
    for V, kw in [(4, {}), (8, {}), (16, dict(sparse=True)), (8, dict(disjoint=True))]:
        p, q = _dists(V, rng, **kw)
        X, Y, K = _run(p, q, n, seed=100 + V)
        tv = 0.5 * np.abs(p - q).sum()
        # marginal of Y is p (losslessness)
        assert _chi2_p(np.bincount(Y, minlength=V), p) > 1e-4
        # X was drawn from q (sanity of the driver)
        assert _chi2_p(np.bincount(X, minlength=V), q) > 1e-4
        # accept rate = 1 - TV, and accept <=> X == Y exactly (residual has no mass where p <= q)
        acc = K.mean()
        se = np.sqrt(max(tv * (1 - tv), 1e-9) / n)
        assert abs(acc - (1 - tv)) < 5 * se + 1e-9
        assert np.array_equal(K == 1, X == Y)
        # full joint against the closed form
        J = np.zeros((V, V))
        np.add.at(J, (X, Y), 1)
        assert _chi2_p(J.ravel(), _closed_form_joint(p, q).ravel()) > 1e-4


def test_identical_distributions_always_accept():
    rng = np.random.default_rng(3)
    p, _ = _dists(16, rng)
    X, Y, K = _run(p, p.copy(), 3000, seed=5)
    assert K.all() and np.array_equal(X, Y)


def test_disjoint_supports_always_reject_and_sample_p():
    rng = np.random.default_rng(4)
    p, q = _dists(8, rng, disjoint=True)
    X, Y, K = _run(p, q, 20000, seed=6)
    assert not K.any()
    assert _chi2_p(np.bincount(Y, minlength=8), p) > 1e-4


def test_accept_test_edges():
    assert mrs.accept_test(0.5, 0.5, 1 - 2.0 ** -24)       # p >= q always accepts
    assert mrs.accept_test(0.6, 0.3, 1 - 2.0 ** -24)
    assert not mrs.accept_test(0.0, 0.3, 2.0 ** -24)       # p = 0 always rejects
    assert mrs.accept_test(0.25, 0.5, 0.5)                 # boundary u = p/q accepts (<=)
    assert not mrs.accept_test(0.25, 0.5, 0.5 + 2.0 ** -23)
    assert mrs.accept_flag(0.25, 0.5, 0.5) and not mrs.accept_flag(0.25, 0.5, 0.6)


def test_residual_race_is_exponential_race_and_tie_rule():
    p = np.array([0.5, 0.3, 0.2, 0.0])
    q = np.array([0.1, 0.3, 0.1, 0.5])
    U = np.array([0.5, 0.5, 0.5, 0.5])
    w, score = mrs.residual_race(p, q, U)
    # support {0, 2}; same E, larger residual wins
    assert w == 0 and np.isinf(score[1]) and np.isinf(score[3])
    np.testing.assert_allclose(score[0], np.log(2) / 0.4, rtol=1e-6)
    # exact tie -> lowest id
    w, _ = mrs.residual_race(np.array([0.5, 0.5, 0.0]), np.array([0.25, 0.25, 0.5]),
                             np.array([0.25, 0.25, 0.9]))
    assert w == 0
    # empty residual
    w, _ = mrs.residual_race(p, p, U)
    assert w == -1
    # tiny U on a small-residual id can still win
    w, _ = mrs.residual_race(p, q, np.array([0.5, 0.5, 1 - 2.0 ** -24, 0.5]))
    assert w == 2


def test_residual_flag_marks_only_close_races():
    p = np.array([0.5, 0.3, 0.2])
    q = np.array([0.1, 0.3, 0.6])
    U = np.array([0.3, 0.5, 0.5])
    w, _ = mrs.residual_race(p, q, U)
    assert w == 0 and not mrs.residual_flag(p, q, U, w)
    # two ids with almost equal scores
    p = np.array([0.4, 0.4 + 1e-9, 0.2 - 1e-9])
    q = np.array([0.2, 0.2, 0.6])
    U = np.array([0.5, 0.5, 0.5])
    w, _ = mrs.residual_race(p, q, U)
    assert mrs.residual_flag(p, q, U, w)
    # massive cancellation p ~ q: a relative 1e-5 could move the support itself
    p = np.array([0.5 + 2e-7, 0.5 - 2e-7])
    q = np.array([0.5, 0.5])
    w, _ = mrs.residual_race(p, q, U[:2])
    assert w == 0 and mrs.residual_flag(p, q, U[:2], w)
    # a single-id support that no perturbation can change is never fragile
    p = np.array([0.9, 0.1])
    q = np.array([0.5, 0.5])
    w, _ = mrs.residual_race(p, q, U[:2])
    assert w == 0 and not mrs.residual_flag(p, q, U[:2], w)
