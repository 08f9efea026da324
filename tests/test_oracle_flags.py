"""Pins for the oracle's parity flags (CPU only): the helpers that decide on which
draws a second implementation may legitimately differ, and the override branches
through which the lock-step driver makes the oracle adopt such a decision.

The flags are not part of the method (Alg. 1, Alg. SCD(pi_MC)); they bound what the
GPU parity tests tolerate, so each is pinned on hand-made rows whose ambiguous set
is known by construction.  Every expected set is EXACT: a tolerance ten times wider
(or narrower) than stated changes it and fails the test.
"""
import numpy as np
import pytest

from oracle import mrs as omrs
from oracle import philox
from oracle import scd
from oracle.scd import ScdConfig, ScdOracle, _ambiguous_ids, _ambiguous_nucleus_ids


# ------------------------------------------------------------------ top-k boundary
def _row(vals):
    return np.asarray(vals, dtype=np.float32)


def test_topk_ambiguous_ids_exact_tie_at_the_kth_value():
    z = _row([5.0, 3.0, 3.0, 1.0, 0.0])          # K = 2: the 2nd and 3rd largest are equal
    thr = np.float32(3.0)
    assert list(_ambiguous_ids(z, thr, 2, 1e-4)) == [1, 2]
    # bit-identical logits on both sides: the tie is kept whole by both, nothing may differ
    assert _ambiguous_ids(z, thr, 2, 0.0).size == 0


def test_topk_ambiguous_ids_just_inside_and_just_outside_the_band():
    tol = 1e-3
    z = _row([5.0, 3.0, 3.0 - 0.9 * tol, 3.0 - 1.1 * tol, 3.0 + 1.1 * tol, 3.0 + 0.9 * tol, 0.0])
    thr = np.float32(3.0)                        # K = 4: 5, 3 + 1.1 tol, 3 + 0.9 tol, then 3.0 itself
    got = sorted(_ambiguous_ids(z, thr, 4, tol))
    assert got == [1, 2, 5]                      # the K-th itself, one below inside, one above inside
    # ten times wider: the two ids at 1.1 tol join; ten times narrower: only the K-th is left => empty
    assert sorted(_ambiguous_ids(z, thr, 4, 10 * tol)) == [1, 2, 3, 4, 5]
    assert _ambiguous_ids(z, thr, 4, tol / 10).size == 0


def test_topk_ambiguous_ids_single_id_gives_the_empty_set():
    z = _row([5.0, 3.0, 2.0, 1.0])
    assert _ambiguous_ids(z, np.float32(3.0), 2, 0.5).size == 0      # nearest other id is 1.0 away
    assert list(_ambiguous_ids(z, np.float32(3.0), 2, 1.0)) == [1, 2]  # band reaches it (<=)


def test_topk_ambiguous_ids_empty_when_nothing_is_filtered():
    z = _row([1.0, 1.0, 1.0])
    for k in (0, 3, 10):
        assert _ambiguous_ids(z, np.float32(-np.inf), k, 1.0).size == 0


# ------------------------------------------------------------------ nucleus boundary
def test_nucleus_ambiguous_ids_on_a_hand_made_row():
    p = np.array([0.5, 0.3, 0.15, 0.05])
    z = np.log(p).astype(np.float32)
    keep = np.ones(4, dtype=bool)
    # top_p = 0.8 is reached exactly by the first two ids; whether id 2 is needed depends on
    # which side of 0.8 a cumulative sum of 0.8 +- rounding falls: id 2 is the ambiguous one
    assert list(_ambiguous_nucleus_ids(z, keep, 0.8, 1e-3)) == [2]
    # top_p = 0.7: the boundary id 1 covers [0.5, 0.8); 0.7 +- 1e-3 stays inside => nothing ambiguous
    assert _ambiguous_nucleus_ids(z, keep, 0.7, 1e-3).size == 0
    # a band that reaches the next cumulative mass (0.7 + 0.11 > 0.8) flags id 2; one that
    # reaches the previous one (0.7 - 0.21 < 0.5) flags id 1 as well
    assert list(_ambiguous_nucleus_ids(z, keep, 0.7, 0.11)) == [2]
    assert list(_ambiguous_nucleus_ids(z, keep, 0.7, 0.21)) == [1, 2]
    # filter off
    assert _ambiguous_nucleus_ids(z, keep, 0.0, 0.5).size == 0
    assert _ambiguous_nucleus_ids(z, keep, 1.0, 0.5).size == 0


def test_nucleus_ambiguous_ids_respect_the_set_topk_left():
    p = np.array([0.4, 0.3, 0.2, 0.1])
    z = np.log(p).astype(np.float32)
    keep = np.array([True, True, True, False])     # top-k dropped id 3: masses renormalise to 4/9, 3/9, 2/9
    # cumulative 0.444, 0.778, 1: top_p = 0.778 sits on the boundary between ids 1 and 2
    assert list(_ambiguous_nucleus_ids(z, keep, 7.0 / 9.0, 1e-3)) == [2]
    assert 3 not in _ambiguous_nucleus_ids(z, keep, 0.99, 0.5)


# ------------------------------------------------------------------ evaluate(): flags and overrides
def _one_row_oracle(n, top_k, top_p=0.0, seed=5, lam=0.0):
    return ScdOracle(ScdConfig(B=1, L=1, N=1, V=n, top_k=top_k, top_p=top_p, seed=seed, cfg_lambda=lam))


def test_evaluate_flags_use_twice_the_logit_discrepancy():
    e = 1e-4
    z = _row([4.0, 2.0, 2.0 - 1.9 * e, 2.0 - 2.1 * e, 0.0, -1.0])
    o = _one_row_oracle(6, top_k=2)
    assert sorted(o.evaluate([[z]], logit_err=[[e]])[0][0]["ambiguous"]) == [1, 2]
    assert o.evaluate([[z]], logit_err=[[0.0]])[0][0]["ambiguous"].size == 0
    assert sorted(o.evaluate([[z]], logit_err=[[10 * e]])[0][0]["ambiguous"]) == [1, 2, 3]
    assert o.evaluate([[z]], logit_err=[[e / 10]])[0][0]["ambiguous"].size == 0
    # without a measured discrepancy: the a-priori band tol * (1 + 2 lambda) * max(1, |thr|)
    tol = o.tol * 2.0
    zb = _row([4.0, 2.0, 2.0 - 0.9 * tol, 2.0 - 1.1 * tol, 0.0, -1.0])
    assert sorted(o.evaluate([[zb]])[0][0]["ambiguous"]) == [1, 2]
    og = _one_row_oracle(6, top_k=2, lam=3.0)      # guidance amplifies an LM-head error 7 times
    assert sorted(og.evaluate([[zb]])[0][0]["ambiguous"]) == [1, 2, 3]


def test_evaluate_membership_override_on_ambiguous_ids_only():
    e = 1e-4
    z = _row([4.0, 2.0, 2.0 - 1.0 * e, 0.0, -1.0])
    o = _one_row_oracle(5, top_k=2)
    base = o.evaluate([[z]], logit_err=[[e]])[0][0]
    assert base["nkept"] == 2 and sorted(base["ambiguous"]) == [1, 2]
    assert base["p"][2] == 0.0 and abs(base["p"].sum() - 1.0) < 1e-15
    # the other implementation kept id 2 and dropped id 1
    sw = o.evaluate([[z]], {(0, 0): {1: False, 2: True}}, logit_err=[[e]])[0][0]
    assert sw["nkept"] == 2 and sw["p"][1] == 0.0 and sw["p"][2] > 0.0
    assert abs(sw["p"].sum() - 1.0) < 1e-15
    want = np.exp(np.float64(z[2]) - np.float64(z[0]))
    assert abs(sw["p"][2] / sw["p"][0] - want) < 1e-15
    # it kept both (a tie it did not split)
    both = o.evaluate([[z]], {(0, 0): {1: True, 2: True}}, logit_err=[[e]])[0][0]
    assert both["nkept"] == 3
    # an id outside the ambiguous set may not be overridden
    with pytest.raises(AssertionError):
        o.evaluate([[z]], {(0, 0): {3: True}}, logit_err=[[e]])
    with pytest.raises(AssertionError):          # nothing is ambiguous when the logits are bit-identical
        o.evaluate([[z]], {(0, 0): {2: True}}, logit_err=[[0.0]])


def test_evaluate_nucleus_override_and_mass_band():
    p = np.array([0.5, 0.3, 0.15, 0.05])
    z = np.log(p).astype(np.float32)
    o = _one_row_oracle(4, top_k=0, top_p=0.8)
    o.tol_mass = 1e-3
    base = o.evaluate([[z]], logit_err=[[0.0]])[0][0]
    assert list(base["ambiguous"]) == [2]
    nk = base["nkept"]
    flipped = o.evaluate([[z]], {(0, 0): {2: nk == 2}}, logit_err=[[0.0]])[0][0]
    assert flipped["nkept"] == (3 if nk == 2 else 2)
    assert flipped["thr"] == (z[2] if nk == 2 else z[1])
    with pytest.raises(AssertionError):
        o.evaluate([[z]], {(0, 0): {0: False}}, logit_err=[[0.0]])
    # a logit discrepancy widens the mass band by 2 e: top_p = 0.7 is 0.1 away from the boundary
    o7 = _one_row_oracle(4, top_k=0, top_p=0.7)
    assert o7.evaluate([[z]], logit_err=[[0.04]])[0][0]["ambiguous"].size == 0     # 2e-6 + 0.08 < 0.1
    assert list(o7.evaluate([[z]], logit_err=[[0.06]])[0][0]["ambiguous"]) == [2]   # 0.12 > 0.1


# ------------------------------------------------------------------ sample(): flags and overrides
SEED = next(s for s in range(100)
            if 0.3 < philox.uniform_scalar(s, 0, 0, 0, philox.STREAM_ACCEPT) < 0.7)


def _crafted_accept_case(delta, n=8, seed=SEED):
    """A one-position oracle whose single MRS call has p(x)/q(x) = u + delta: an accept
    (delta >= 0) or a rejection (delta < 0) that is |delta| away from the boundary.  The position
    was never evaluated, so q is uniform and x is its initial draft."""
    o = ScdOracle(ScdConfig(B=1, L=1, N=1, V=n, seed=seed))
    x = int(o.X[0, 0])
    u = philox.uniform_scalar(seed, 0, 0, 0, philox.STREAM_ACCEPT)
    px = (u + delta) / n
    p = np.full(n, (1.0 - px) / (n - 1))
    p[x] = px
    z = np.log(p).astype(np.float32)              # fp32 logits: p(x) is reproduced to ~1e-7 relative
    return o, z, x, u


def test_sample_accept_flag_band_and_override():
    # 3e-6 inside the accept side of the boundary: flagged under the stated 1e-5 rule
    o, z, x, u = _crafted_accept_case(+3e-6)
    plan = o.evaluate([[z]], logit_err=[[0.0]])
    r = o.sample(plan)[0][0]
    assert r["k"] == 1 and r["y"] == x and r["flag_accept"] and r["flag_accept_strict"]
    forced = o.sample(plan, accept_override={(0, 0): 0})[0][0]     # the other side rejected
    assert forced["k"] == 0 and forced["y"] != x                    # residual excludes x (p(x) < q(x))
    U = philox.uniform_per_vocab(SEED, 0, 0, 0, philox.STREAM_RESID, 8)
    assert forced["y"] == omrs.residual_race(plan[0][0]["p"], o.draft_row(0, 0), U)[0]
    # 1e-4 away: not flagged, and an override is refused
    o, z, x, u = _crafted_accept_case(-1e-4)
    plan = o.evaluate([[z]], logit_err=[[0.0]])
    r = o.sample(plan)[0][0]
    assert r["k"] == 0 and not r["flag_accept"] and not r["flag_accept_strict"]
    with pytest.raises(AssertionError):
        o.sample(plan, accept_override={(0, 0): 1})
    # the same draw when the logits of p were 1e-4 apart on the two sides: exp(z - lse) may be off
    # by a factor exp(2e-4) > 1 + 1e-4, so the band (1e-5 + 2e-4) covers it -- but not the strict flag
    plan = o.evaluate([[z]], logit_err=[[1e-4]])
    r = o.sample(plan)[0][0]
    assert r["flag_accept"] and not r["flag_accept_strict"] and abs(r["tol"] - (1e-5 + 2e-4)) < 1e-12
    assert o.sample(plan, accept_override={(0, 0): 1})[0][0]["k"] == 1
    # a discrepancy ten times smaller does not reach the draw
    plan = o.evaluate([[z]], logit_err=[[1e-5]])
    assert not o.sample(plan)[0][0]["flag_accept"]


def test_sample_residual_override_only_on_a_flagged_race():
    # a rejection whose residual race is not close: the token cannot be overridden
    o, z, x, u = _crafted_accept_case(-0.25)
    plan = o.evaluate([[z]], logit_err=[[0.0]])
    r = o.sample(plan)[0][0]
    assert r["k"] == 0
    other = (r["y"] + 1) % 8 if (r["y"] + 1) % 8 != x else (r["y"] + 2) % 8
    if not r["flag_resid"]:
        with pytest.raises(AssertionError):
            o.sample(plan, resid_override={(0, 0): other})
    # the flag itself on a hand-made race: two ids whose scores differ by 1e-6 relative
    p = np.array([0.5, 0.3, 0.2, 0.0])
    q = np.array([0.0, 0.0, 0.0, 1.0])
    U = np.array([np.exp(-0.5), np.exp(-0.3 * (1 + 1e-6)), 0.5, 0.5])   # scores 1, 1 + 1e-6, 3.47, -
    w, _ = omrs.residual_race(p, q, U)
    assert w in (0, 1)
    assert omrs.residual_flag(p, q, U, w, 1e-5)
    U2 = np.array([np.exp(-0.5), np.exp(-0.3 * 1.01), 0.5, 0.5])        # 1 % apart: safe at 1e-5 ...
    assert omrs.residual_race(p, q, U2)[0] == 0 and not omrs.residual_flag(p, q, U2, 0, 1e-5)
    assert omrs.residual_flag(p, q, U2, 0, 1e-2)                         # ... and flagged at 1e-2


def test_flags_do_not_change_what_is_decoded():
    # decode() with and without measured discrepancies emits the same tokens: flags only annotate
    from paper_2510_24211_amd import workload as wl
    w = wl.scaled(wl.WORKLOADS["C0"], name="t", N=24, L=4, V=64, top_k=16)
    toy = wl.ToyLogits(w)
    cfg = ScdConfig(B=1, L=4, N=24, V=64, top_k=16, seed=3)
    model = lambda b, i, Lw, toks, t, age: np.stack(
        [toy.table[b, i + k, min(int(age[k]), w.age_cap)] for k in range(Lw)])
    a = scd.decode(cfg, model)
    o = ScdOracle(cfg)
    while not o.done():
        i, Lw = o.window(0)
        z = model(0, i, Lw, None, o.t[0], o.age[0, i:i + Lw].copy())
        plan = o.evaluate([z], logit_err=[[1e-3] * Lw])
        o.commit(plan, o.sample(plan))
    assert np.array_equal(a.out, o.out) and a.t == o.t
