"""Gumbel-sharing coupling (Alg. "GS(P, Q, G)") -- oracle side; test infrastructure only.

GS(P, Q, G):  X = argmax_i (log P_i + g_i),  Y = argmax_i (log Q_i + g_i)  with ONE
noise vector g_i ~ Gumbel(0, 1) for both.  By the Gumbel-max trick X ~ P and Y ~ Q
(Thm "Gumbel coupling", validity part); the appendix proof rewrites the same events as an
exponential race,  X = argmin_i E_i / P_i  with  E_i = exp(-g_i) ~ Exp(1),  and gives the
exact diagonal of the joint law (its Eq. 6):
    Pr[X = Y = k] = 1 / sum_j max(P_j / P_k, Q_j / Q_k),
hence  Pr[X = Y] >= (1 - D_TV) / (1 + D_TV).

In the decode loop (Alg. SCD(pi_GS)) the noise of window position j is a function of j
alone ("SampleGumbelNoiseUsingHash(j)"), so every iteration re-draws the draft of position j
from its newest distribution with the SAME noise.

Readings fixed here:
  * g_i = -ln(-ln U_i) with U_i the Philox uniform of (seed, sequence, position, vocab id)
    on its own stream; the iteration does not enter the key;
  * the draw is DECIDED in the race form and in fp32, as the residual draw of MRS is:
    E_i = fl(-ln U_i), score_i = fl(E_i / fl(P_i)), winner = lowest id among the minima,
    over the ids with P_i > 0.  `draw_definition` is the printed argmax form in fp64; the
    two agree except on draws that `flag` marks as numerically fragile.
"""
import numpy as np

F32 = np.float32


def gumbel(U):
    """g = -ln(-ln U), fp64."""
    U = np.asarray(U, dtype=np.float64)
    return -np.log(-np.log(U))


def draw_definition(p, U):
    """argmax_i (log p_i + g_i) over the support of p, fp64; first maximum = lowest id."""
    p = np.asarray(p, dtype=np.float64)
    with np.errstate(divide="ignore"):
        s = np.where(p > 0, np.log(p) + gumbel(U), -np.inf)
    return int(np.argmax(s))


def draw(p, U):
    """The same draw in race form, decided in fp32.  Returns (winner, scores)."""
    p32 = np.asarray(p).astype(F32)
    sup = p32 > 0
    score = np.full(p32.shape, np.inf, dtype=F32)
    E = (-np.log(np.asarray(U, dtype=np.float64))).astype(F32)
    score[sup] = E[sup] / p32[sup]
    return int(np.argmin(score)), score


def flag(p, U, winner, tol=1e-5, tol_log=1e-6):
    """True when another id could win after perturbing every probability by a relative
    `tol` and every -ln U by a relative `tol_log`."""
    p = np.asarray(p, dtype=np.float64)
    E = -np.log(np.asarray(U, dtype=np.float64))
    with np.errstate(divide="ignore", invalid="ignore"):
        s_lo = np.where(p > 0, E * (1 - tol_log) / (p * (1 + tol)), np.inf)
    s_hi_w = E[winner] * (1 + tol_log) / (p[winner] * (1 - tol))
    s_lo[winner] = np.inf
    return bool(s_lo.min() <= s_hi_w)


def gs(P, Q, U):
    """Alg. GS(P, Q, G) with G = gumbel(U): the coupled pair (X, Y)."""
    return draw(P, U)[0], draw(Q, U)[0]


def diagonal(P, Q):
    """Eq. 6 of the appendix: Pr[X = Y = k] for every k (0 where P_k Q_k = 0)."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    out = np.zeros_like(P)
    for k in range(P.size):
        if P[k] > 0 and Q[k] > 0:
            out[k] = 1.0 / np.maximum(P / P[k], Q / Q[k]).sum()
    return out
