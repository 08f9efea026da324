"""Modified Rejection Sampling (Alg. 1) -- oracle side; test infrastructure only.

MRS(P, Q, X) with X ~ Q:
    u ~ U(0,1);  if u <= min(1, P(X)/Q(X)) return (X, 1)
    else return (Y ~ norm(max(0, P - Q)), 0)
Prop. 2.1: Y ~ P and Pr[accept] = 1 - D_TV(P, Q).  Thm 4.3: (X, Y) is a
maximal coupling of Q and P, so the same call is the paper's coupled sampler
pi_MC (Sec. 4.1).

Readings the paper leaves open, fixed here:
  * the accept test is evaluated without a division as  u*Q(X) <= P(X), in
    fp32 (one correctly rounded product, one comparison).  Q(X) > 0 because
    X ~ Q, u is strictly inside (0,1), so P(X) >= Q(X) always accepts and
    P(X) = 0 always rejects;
  * the residual draw is an exponential race: with one uniform U_v per vocab
    id, Y = argmin over {v : r_v > 0} of  -ln(U_v) / r_v,  r = max(0, P - Q).
    An exponential with rate r_v wins a race with probability r_v / sum(r), so
    Y ~ norm(r) without ever forming the normaliser.  Ties go to the lowest id.
    The decision is taken in fp32: r_v = fl(P_v - Q_v) on fp32-rounded
    probabilities, E_v = fl(-ln U_v), score = fl(E_v / r_v);
  * if no id has r_v > 0 (only reachable through rounding) the draw counts as
    an accept.

Each decision also returns a flag saying whether it is numerically fragile,
i.e. whether a relative perturbation of `tol` in the probabilities could flip
it.  A second implementation working in fp32 may legitimately differ on
flagged draws and on no others.
"""
import numpy as np

F32 = np.float32


def accept_test(px, qx, u):
    """Alg. 1 step 2 in fp32: fl(u * q(x)) <= p(x)."""
    return bool(F32(u) * F32(qx) <= F32(px))


def accept_flag(px, qx, u, tol=1e-5):
    """True when |u - p(x)/q(x)| < tol, written as |u*q - p| < tol*q."""
    return bool(abs(float(u) * float(qx) - float(px)) < tol * float(qx))


def residual_race(p, q, U):
    """Alg. 1 last step.  p, q: fp64 probability rows; U: one uniform per id.
    Returns (winner id or -1 if the residual is empty, score array fp32 with
    inf outside the support)."""
    p32 = np.asarray(p).astype(F32)
    q32 = np.asarray(q).astype(F32)
    r = p32 - q32                                    # fp32 subtraction
    sup = r > 0
    score = np.full(r.shape, np.inf, dtype=F32)
    if not sup.any():
        return -1, score
    E = (-np.log(np.asarray(U, dtype=np.float64))).astype(F32)
    score[sup] = E[sup] / r[sup]                     # fp32 division
    return int(np.argmin(score)), score              # first minimum = lowest id


def residual_flag(p, q, U, winner, tol=1e-5, tol_log=1e-6):
    """True when some other id could beat `winner` after perturbing every
    probability by a relative `tol` and every -ln U by a relative `tol_log`."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    E = -np.log(np.asarray(U, dtype=np.float64))
    r_hi = np.maximum(0.0, p * (1 + tol) - q * (1 - tol))
    r_lo = np.maximum(0.0, p * (1 - tol) - q * (1 + tol))
    with np.errstate(divide="ignore", invalid="ignore"):
        s_lo = np.where(r_hi > 0, E * (1 - tol_log) / r_hi, np.inf)
        s_hi_w = E[winner] * (1 + tol_log) / r_lo[winner] if r_lo[winner] > 0 else np.inf
    s_lo[winner] = np.inf
    return bool(s_lo.min() <= s_hi_w)


def mrs(p, q, x, u, U_fn, tol=1e-5):
    """One MRS call.  p, q fp64 rows, x the draft token (drawn from q), u the
    accept uniform, U_fn() -> per-id uniforms (called only on rejection).

    Returns dict(y, k, flag_accept, flag_resid, px, qx)."""
    px, qx = float(p[x]), float(q[x])
    out = dict(px=px, qx=qx, flag_accept=accept_flag(px, qx, u, tol), flag_resid=False)
    if accept_test(px, qx, u):
        out.update(y=int(x), k=1)
        return out
    U = U_fn()
    w, _ = residual_race(p, q, U)
    if w < 0:
        out.update(y=int(x), k=1)
        return out
    out.update(y=w, k=0, flag_resid=residual_flag(p, q, U, w, tol))
    return out
