"""LM head and logit post-processing (oracle side; test infrastructure only).

p^(t) is the distribution that remains once every logit processor (top-k,
guidance) has been applied (Sec. 4.3, last sentence).  The processors and
their parameters come from Sec. 5.1 "Effect on CFG" (mixed logit
(1+lambda)*c - lambda*u) and the appendix "Experimental Details" (temperature
tau = 1, top-k K = 2000 / 1000, nucleus p = 0.8 for video).  The order used here is
    LM head -> CFG combine -> allowed-id mask -> 1/tau -> top-k -> top-p -> softmax.

Precision: the LM head accumulates in fp64 over the exact bf16 input values and
rounds the logit once to fp32.  The three fp32 roundings of the CFG combine and
the fp32 division by tau are the method's stated arithmetic and are done in
fp32.  The top-k threshold is an exact order statistic of those fp32 values.
The softmax is evaluated in fp64.
"""
import numpy as np


def bf16_bits_to_f64(u16):
    """Exact value of bf16 bit patterns (uint16 array) as float64."""
    u16 = np.ascontiguousarray(u16, dtype=np.uint16)
    return (u16.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def lm_head(h_bits, w):
    """logit[m, v] = sum_k h[m, k] * W[v, k]  (the last linear layer of the
    target model; "Evaluate" step of Alg. 2 / Alg. 3).

    h_bits [M, d]: bf16 bit patterns.  w [V, d]: bf16 bit patterns (uint16), or
    the same matrix already decoded to float64 by bf16_bits_to_f64 (callers
    that evaluate many windows against one W decode it once).  fp64 accumulate,
    one rounding to fp32."""
    h = bf16_bits_to_f64(h_bits)
    w64 = w if w.dtype == np.float64 else bf16_bits_to_f64(w)
    return (h @ w64.T).astype(np.float32)


def cfg_combine(c, u, lam):
    """Classifier-free-guidance mix (1+lambda)*c - lambda*u (Sec. 5.1, "Effect
    on CFG"), evaluated in fp32 as fl(fl((1+lambda)*c) - fl(lambda*u)) with
    (1+lambda) itself rounded to fp32 first."""
    c = np.asarray(c, dtype=np.float32)
    u = np.asarray(u, dtype=np.float32)
    lam = np.float32(lam)
    one_plus = np.float32(np.float32(1.0) + lam)
    return (one_plus * c).astype(np.float32) - (lam * u).astype(np.float32)


def apply_temperature(z, tau):
    """z / tau in fp32."""
    return (np.asarray(z, dtype=np.float32) / np.float32(tau)).astype(np.float32)


def process_logits(c, u, lam, tau):
    """CFG (if u is given) then temperature.  c, u: fp32 [..., V_eff] already
    restricted to the allowed id range (the mask to -inf outside the range is
    realised by never forming those columns)."""
    z = np.asarray(c, dtype=np.float32) if u is None else cfg_combine(c, u, lam)
    return apply_temperature(z, tau)


def topk_threshold(z, top_k):
    """K-th largest value of the row; -inf when nothing is filtered (top-k off,
    i.e. top_k == 0, or K >= row length).  The kept set is
    {v : z_v >= threshold}: every value tied with the K-th is kept."""
    z = np.asarray(z, dtype=np.float32)
    n = z.shape[-1]
    if top_k <= 0 or top_k >= n:
        return np.float32(-np.inf)
    srt = np.sort(z)[::-1]
    return np.float32(srt[top_k - 1])


def nucleus_threshold(z, keep, top_p):
    """Nucleus (top-p) filter (appendix "Experimental Details", video generation:
    p = 0.8, applied to the distribution that the earlier processors leave):
    among the ids of `keep`, ordered by decreasing probability, the shortest
    prefix whose probabilities sum to at least top_p survives; ids tied with the
    last survivor survive too (the filter is a threshold on the logit, so equal
    logits are never split).  Returns that threshold as fp32 (the smallest
    surviving logit); -inf when the filter is off (top_p <= 0 or >= 1).  fp64."""
    if not (0.0 < top_p < 1.0):
        return np.float32(-np.inf)
    zs = np.sort(np.asarray(z, dtype=np.float32)[keep].astype(np.float64))[::-1]
    pr = np.exp(zs - zs[0])
    pr = pr / pr.sum()
    cum = np.cumsum(pr)
    reach = np.nonzero(cum >= top_p)[0]
    last = reach[0] if reach.size else zs.size - 1     # rounding may leave cum[-1] just below 1
    return np.float32(zs[last])


def softmax_kept(z, thr):
    """Probability row p_v = [z_v >= thr] * exp(z_v - m) / sum_kept exp(z_w - m),
    fp64.  Also returns the log normaliser lse = m + log(sum)."""
    z64 = np.asarray(z, dtype=np.float32).astype(np.float64)
    keep = z64 >= np.float64(thr)
    m = z64[keep].max()
    e = np.where(keep, np.exp(z64 - m), 0.0)
    s = e.sum()
    return e / s, m + np.log(s)


def distribution(z, top_k, top_p=0.0):
    """(p fp64 row, thr fp32, lse fp64) for a processed-logit row: top-k first,
    then the nucleus filter on what top-k left."""
    z = np.asarray(z, dtype=np.float32)
    thr = topk_threshold(z, top_k)
    thr = max(thr, nucleus_threshold(z, z >= thr, top_p))
    p, lse = softmax_kept(z, thr)
    return p, np.float32(thr), lse
