"""Pins for the oracle's LM head and logit processors (CPU only): brute force
on tiny inputs with exact rational arithmetic, library routines on the special
cases that reduce to them, and invariants."""
from fractions import Fraction

import numpy as np
from scipy import special

from oracle import logits as lg
from paper_2510_24211_amd.workload import f32_to_bf16_bits


def _bf16_fraction(bits):
    f = np.array([bits], dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return Fraction(float(f.view(np.float32)[0]))


def test_bf16_decode_matches_float_semantics():
    x = np.array([0.0, 1.0, -2.5, 0.02, 3.140625, -1e-3], dtype=np.float32)
    bits = f32_to_bf16_bits(x)
    back = lg.bf16_bits_to_f64(bits)
    # bf16 keeps 8 significant bits: relative error <= 2^-9, exact on short values
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -9)
    assert back[1] == 1.0 and back[2] == -2.5 and back[4] == 3.140625


def test_lm_head_brute_force_rational():
    g = np.random.default_rng(0)
    M, V, d = 3, 5, 16
    h = f32_to_bf16_bits(g.standard_normal((M, d)).astype(np.float32))
    W = f32_to_bf16_bits((g.standard_normal((V, d)) * 0.02).astype(np.float32))
    got = lg.lm_head(h, W)
    assert got.dtype == np.float32 and got.shape == (M, V)
    for m in range(M):
        for v in range(V):
            exact = sum(_bf16_fraction(h[m, k]) * _bf16_fraction(W[v, k]) for k in range(d))
            assert got[m, v] == np.float32(float(exact))   # transposed operand or wrong axis fails


def test_cfg_combine_roundings_and_closed_cases():
    c = np.array([1.0, 0.1, -3.3, 7.0], dtype=np.float32)
    u = np.array([1.0, 0.3, 2.2, -1.0], dtype=np.float32)
    # lambda = 0 returns c exactly; u == 0 gives (1+lambda) c
    assert np.array_equal(lg.cfg_combine(c, u, 0.0), c)
    assert np.array_equal(lg.cfg_combine(c, np.zeros_like(c), 3.0), np.float32(4.0) * c)
    # exact dyadic values: (1+3)*1 - 3*1 = 1 ; 4*7 - 3*(-1) = 31
    z = lg.cfg_combine(c, u, 3.0)
    assert z[0] == 1.0 and z[3] == 31.0
    # the three roundings, spelled with Fractions
    for ci, ui, zi in zip(c, u, z):
        a = np.float32(float(Fraction(float(ci)) * 4))
        b = np.float32(float(Fraction(float(ui)) * 3))
        assert zi == np.float32(float(Fraction(float(a)) - Fraction(float(b))))
    # guidance pushes away from u: sign convention (1+l)c - l u, not l c - (l-1) u
    assert lg.cfg_combine(np.float32([1.0]), np.float32([0.0]), 3.0)[0] == 4.0


def test_temperature():
    z = np.array([1.0, -2.0, 0.3], dtype=np.float32)
    assert np.array_equal(lg.apply_temperature(z, 1.0), z)
    assert np.array_equal(lg.apply_temperature(z, 2.0), z / np.float32(2.0))
    # sharper for tau < 1
    p_hot, _ = lg.softmax_kept(lg.apply_temperature(z, 0.5), -np.inf)
    p_one, _ = lg.softmax_kept(z, -np.inf)
    assert p_hot.max() > p_one.max()


def test_softmax_without_topk_is_library_softmax():
    g = np.random.default_rng(1)
    z = (g.standard_normal(1000) * 3).astype(np.float32)
    p, thr, lse = lg.distribution(z, 0)
    assert thr == -np.inf
    np.testing.assert_allclose(p, special.softmax(z.astype(np.float64)), rtol=1e-13)
    np.testing.assert_allclose(lse, special.logsumexp(z.astype(np.float64)), rtol=1e-14)
    # K = |A| keeps everything as well
    p2, thr2, _ = lg.distribution(z, z.size)
    assert thr2 == -np.inf
    np.testing.assert_allclose(p2, p, rtol=1e-13)


def test_topk_brute_force_and_ties():
    g = np.random.default_rng(2)
    for n, K in [(10, 3), (50, 1), (50, 49), (257, 100)]:
        z = g.standard_normal(n).astype(np.float32)
        thr = lg.topk_threshold(z, K)
        assert (z > thr).sum() == K - 1 and (z >= thr).sum() == K      # distinct values
        p, _ = lg.softmax_kept(z, thr)
        keep = np.argsort(-z)[:K]
        want = np.zeros(n)
        want[keep] = special.softmax(z[keep].astype(np.float64))
        np.testing.assert_allclose(p, want, rtol=1e-13, atol=0)
        assert abs(p.sum() - 1) < 1e-14 and (p > 0).sum() == K
    # ties at the threshold are all kept
    z = np.array([5, 3, 3, 3, 1, 0], dtype=np.float32)
    thr = lg.topk_threshold(z, 2)
    assert thr == 3.0
    p, _ = lg.softmax_kept(z, thr)
    assert (p > 0).sum() == 4
    # K larger than the row
    assert lg.topk_threshold(z, 100) == -np.inf and lg.topk_threshold(z, 6) == -np.inf
    assert lg.topk_threshold(z, 5) == 1.0


def test_lse_consistency():
    g = np.random.default_rng(3)
    z = (g.standard_normal(300) * 4).astype(np.float32)
    p, thr, lse = lg.distribution(z, 40)
    keep = z >= thr
    np.testing.assert_allclose(p[keep], np.exp(z[keep].astype(np.float64) - lse), rtol=1e-12)
    assert np.all(p[~keep] == 0)


# ---- nucleus (top-p) filter ---------------------------------------------------------
def _probs_to_logits(p):
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def test_nucleus_hand_worked_rows():
    # probabilities 0.5, 0.3, 0.15, 0.05 (any order of ids): cumulative 0.5, 0.8, 0.95, 1
    z = _probs_to_logits([0.15, 0.5, 0.05, 0.3])
    every = np.ones(4, dtype=bool)
    kept = lambda p: set(np.nonzero(z >= lg.nucleus_threshold(z, every, p))[0])
    assert kept(0.4) == {1}                 # the mode alone already holds 0.5
    assert kept(0.6) == {1, 3}
    assert kept(0.9) == {0, 1, 3}
    assert kept(0.96) == {0, 1, 2, 3}
    # off outside (0, 1)
    assert lg.nucleus_threshold(z, every, 0.0) == -np.inf
    assert lg.nucleus_threshold(z, every, 1.0) == -np.inf


def test_nucleus_brute_force_minimal_top_set():
    """Definition by exhaustion with rational arithmetic on small integer weights
    (probability = weight / total): over all sets that are closed upwards in probability
    (a kept id implies every more probable id and every id tied with it), the smallest one
    with mass >= p.  Targets closer than 1e-5 to a cumulative mass are skipped: the logits are
    ln(weight) rounded to fp32, so the row's probabilities are the weights only to ~1e-7."""
    g = np.random.default_rng(5)
    checked = 0
    for trial in range(200):
        n = int(g.integers(2, 8))
        w = g.integers(1, 9, size=n)                      # ties are frequent
        z = np.log(w.astype(np.float64)).astype(np.float32)
        total = Fraction(int(w.sum()))
        p = Fraction(int(g.integers(1, 64)), 64)
        levels = sorted(set(int(x) for x in w), reverse=True)
        masses = [Fraction(int(w[w >= lv].sum())) / total for lv in levels]
        if any(abs(float(m - p)) < 1e-5 for m in masses):
            continue
        best = next(set(np.nonzero(w >= lv)[0]) for lv, m in zip(levels, masses) if m >= p)
        thr = lg.nucleus_threshold(z, np.ones(n, dtype=bool), float(p))
        assert set(np.nonzero(z >= thr)[0]) == best
        checked += 1
    assert checked > 100


def test_nucleus_invariants_and_order_with_topk():
    g = np.random.default_rng(6)
    for _ in range(20):
        n = 200
        z = (g.standard_normal(n) * 2.5).astype(np.float32)
        top_p = float(g.uniform(0.05, 0.95))
        p_full = special.softmax(z.astype(np.float64))
        thr = lg.nucleus_threshold(z, np.ones(n, dtype=bool), top_p)
        kept = z >= thr
        assert p_full[kept].sum() >= top_p - 1e-12                       # enough mass
        weakest = p_full[kept].min()
        assert p_full[kept].sum() - weakest * (p_full[kept] == weakest).sum() < top_p + 1e-12   # minimal
        assert p_full[kept].min() >= p_full[~kept].max() if (~kept).any() else True   # most probable ids
        # against the library: sort, cumulative sum, searchsorted
        order = np.argsort(-p_full, kind="stable")
        cut = int(np.searchsorted(np.cumsum(p_full[order]), top_p, side="left"))
        assert kept.sum() == cut + 1                                     # no ties in this row
        # after top-k the nucleus is taken on the RENORMALISED top-k distribution
        K = 20
        pk, thr_k, _ = lg.distribution(z, K, 0.0)
        pkp, thr_kp, _ = lg.distribution(z, K, top_p)
        order_k = np.argsort(-pk, kind="stable")
        cut_k = int(np.searchsorted(np.cumsum(pk[order_k]), top_p, side="left"))
        assert (pkp > 0).sum() == cut_k + 1 and thr_kp >= thr_k
        assert abs(pkp.sum() - 1.0) < 1e-12
        np.testing.assert_allclose(pkp[pkp > 0], pk[pkp > 0] / pk[pkp > 0].sum(), rtol=1e-12)


def test_nucleus_ties_are_never_split():
    z = _probs_to_logits([0.4, 0.2, 0.2, 0.2])
    thr = lg.nucleus_threshold(z, np.ones(4, dtype=bool), 0.5)    # 0.4 + one of the 0.2s would do
    assert (z >= thr).sum() == 4
    thr = lg.nucleus_threshold(z, np.ones(4, dtype=bool), 0.3)
    assert (z >= thr).sum() == 1


def test_nucleus_is_monotone_and_nested_in_p():
    """A larger target mass never raises the threshold: the kept sets are nested, and their
    masses bracket the targets (property over random rows, ties included)."""
    g = np.random.default_rng(8)
    for trial in range(40):
        n = int(g.integers(3, 400))
        z = (g.standard_normal(n) * g.uniform(0.2, 4.0)).astype(np.float32)
        if trial % 4 == 0:
            z = (np.round(z * 2) / 2).astype(np.float32)          # many exact ties
        every = np.ones(n, dtype=bool)
        p_full = special.softmax(z.astype(np.float64))
        prev_thr, prev_kept = np.inf, 0
        for top_p in np.sort(g.uniform(0.01, 0.99, size=12)):
            thr = lg.nucleus_threshold(z, every, float(top_p))
            kept = z >= thr
            assert thr <= prev_thr and kept.sum() >= prev_kept
            assert p_full[kept].sum() >= top_p - 1e-12
            strictly_above = z > thr                               # without the last level: too little
            assert p_full[strictly_above].sum() < top_p + 1e-12
            prev_thr, prev_kept = thr, int(kept.sum())
