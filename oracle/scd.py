"""Speculative Coupled Decoding (oracle side; test infrastructure only): the
maximal-coupling variant pi_MC and, with ScdConfig.coupling = "gs", the
Gumbel-sharing variant pi_GS.

Two forms of the same decode loop are written out:

  * ScdOracle / decode(): the "efficient" form (appendix "Algorithms",
    Alg. SCD(pi_MC)): after the target model has been evaluated on the window,
    ONE Modified-Rejection-Sampling call per window position, without break;
    the index of the first rejection decides how many tokens are emitted.  Left
    of it the calls are the speculative verification, at it the call is the
    residual resample, right of it the calls are the coupled redraft of the
    next iteration's draft tokens.
  * decode_sequential(): the pedagogical form (Sec. 4.1, Alg. "Pseudo code for
    our SCD"): a Drafting phase that re-couples every not-yet-verified draft
    with MRS, an Evaluate phase, and a sequential Verify phase that breaks at
    the first rejection.  Sec. 4.3 states that the two are the same operation;
    with draws keyed on (position, iteration) they emit identical tokens.

Readings fixed here (the paper's loops are ambiguous about them):
  * the window is exactly L positions [i, i+L) clipped to the sequence end
    (Lw = min(L, N-i)); a rejection at window offset r emits r+1 tokens
    (r accepted drafts + the resampled token), no rejection emits Lw tokens;
  * a position that has never been evaluated carries the draft distribution
    Uniform(allowed ids) and a draft token drawn from it ("p <- Random(),
    X ~ p" in the algorithms' initialisation);
  * the iteration index in the key of a draw is the iteration whose Evaluate
    produced the target distribution P of that MRS call;
  * tokens are handled as offsets 0..|A|-1 into the allowed id range
    [v_lo, v_hi); emitted tokens are v_lo + offset.

pi_GS (Alg. SCD(pi_GS) of the appendix "Algorithms"): the verification is the
same sequence of MRS calls up to the first rejection; what changes is the
redraft of the positions right of it, which is the shared-noise Gumbel-max draw
from the position's newest distribution, X_j = argmax_v(log p_j(v) + G_j(v)),
with G_j a function of the position only.  Further readings for it:
  * a never-evaluated position gets its first draft exactly as under pi_MC (one
    uniform draw from its own stream): its "Random()" distribution is uniform,
    any draw from it is admissible, and this one costs one random number instead
    of one per vocabulary id;
  * the vectorised form evaluates the MRS call of every window position (the
    calls right of the first rejection are discarded) and the Gumbel draw of
    every window position (the draws left of it are discarded).

alpha-coupling (Sec. 5.3 "Coupling Strength", appendix Alg. "alpha-Coupling
Implementation"): pi^alpha = alpha * pi_cpl + (1 - alpha) * pi_ind.  Per redraft one
uniform u; if u <= alpha the coupled redraft above is taken, otherwise an
independent draw X ~ p (here: a Gumbel-max / exponential-race draw with noise
keyed by position AND iteration, i.e. fresh every time).  alpha = 1 is SCD,
alpha = 0 is vanilla SJD.  Only the redraft changes; verification does not.
"""
from dataclasses import dataclass, field
import numpy as np

from . import philox
from . import logits as lg
from . import mrs as mrs_mod
from . import gs as gs_mod
from . import diagnostics as dg


@dataclass
class ScdConfig:
    B: int = 1
    L: int = 8
    N: int = 64
    V: int = 1024
    v_lo: int = 0
    v_hi: int = -1           # -1 => V
    top_k: int = 0           # 0 => off
    top_p: float = 0.0       # nucleus mass; 0 (or >= 1) => off
    temperature: float = 1.0
    cfg_lambda: float = 0.0  # 0 => no CFG
    seed: int = 0
    coupling: str = "mc"     # "mc": maximal coupling (MRS redraft); "gs": Gumbel sharing
    alpha: float = 1.0       # coupling strength: probability of the coupled redraft

    def __post_init__(self):
        if self.v_hi < 0:
            self.v_hi = self.V
        assert self.coupling in ("mc", "gs")
        assert 0.0 <= self.alpha <= 1.0

    @property
    def n_allowed(self):
        return self.v_hi - self.v_lo


def _ambiguous_ids(z, thr, top_k, tol_z):
    """Ids whose membership in the top-k set could differ in an implementation
    whose logits are within tol_z / 2 of z (sup norm): every id within tol_z of
    the threshold, the K-th itself included (an exact tie here may be split
    there), provided there is more than one such id.  Why tol_z = 2 * error is
    exact: an order statistic moves by at most the sup-norm error e, and so does
    every logit, so z_v >= thr can change only where |z_v - thr| <= 2 e.
    tol_z <= 0 (bit-identical logits): nothing is ambiguous."""
    if top_k <= 0 or top_k >= z.shape[-1] or not tol_z > 0.0:
        return np.zeros(0, dtype=np.int64)
    d = np.abs(z.astype(np.float64) - np.float64(thr))
    ids = np.nonzero(d <= tol_z)[0]
    return ids if ids.size > 1 else np.zeros(0, dtype=np.int64)


def _ambiguous_nucleus_ids(z, keep, top_p, tol_mass):
    """Ids whose membership in the nucleus could flip if the cumulative masses
    were off by tol_mass (relative to the total): those between the thresholds
    for top_p + tol_mass and top_p - tol_mass."""
    if not (0.0 < top_p < 1.0):
        return np.zeros(0, dtype=np.int64)
    t_in = lg.nucleus_threshold(z, keep, max(top_p - tol_mass, np.finfo(np.float64).tiny))
    t_out = lg.nucleus_threshold(z, keep, min(top_p + tol_mass, 1.0 - 1e-16))
    return np.nonzero(keep & (z >= t_out) & (z < t_in))[0]


class ScdOracle:
    """State machine of the vectorised form.  One step = evaluate() (turn the
    processed-logit rows of the window into distributions), sample() (one MRS
    per window position) and commit() (emit, slide, re-initialise)."""

    def __init__(self, cfg: ScdConfig, tol=1e-5, tol_mass=2e-6):
        self.cfg = cfg
        self.tol = tol
        self.tol_mass = tol_mass              # nucleus boundary: relative error of a cumulative mass
        B, L, N = cfg.B, cfg.L, cfg.N
        self.i = [0] * B                      # accepted-prefix pointer
        self.t = [0] * B                      # iterations done (= NFE)
        self.X = np.full((B, N + L), -1, dtype=np.int64)      # current draft per position
        self.age = np.zeros((B, N + L), dtype=np.int64)       # evaluations so far
        self.q = [dict() for _ in range(B)]   # pos -> fp64 row of the draft distribution
        self.qerr = [dict() for _ in range(B)]  # pos -> logit discrepancy bound that row was flagged with
        self.out = np.full((B, N), -1, dtype=np.int64)
        self.accept_hist = [[] for _ in range(B)]
        self.last_hamming = [(0, 0)] * B      # (changed drafts, surviving positions) of the last step
        # Hamm(t + 1 - n, t + 1), n = 1..3 (Sec. 5.3 "Multi-Step Behavior"): drafts of the window
        # after the last step against the drafts n iterations earlier, over the positions that
        # sit in both windows; (differing, compared) per n
        self.last_hamming_multi = [[(0, 0)] * 3 for _ in range(B)]
        self._draft_hist = [[] for _ in range(B)]     # newest first: (window start, drafts by position)
        self.positions_verified = 0
        for b in range(B):
            for j in range(min(L, N)):
                self._init_position(b, j)

    # -- helpers -----------------------------------------------------------
    def _init_position(self, b, j):
        self.X[b, j] = philox.init_token(self.cfg.seed, b, j, self.cfg.n_allowed)
        self.age[b, j] = 0
        self.q[b].pop(j, None)
        self.qerr[b].pop(j, None)

    def window(self, b):
        i = self.i[b]
        return i, max(0, min(self.cfg.L, self.cfg.N - i))

    def done(self):
        return all(i >= self.cfg.N for i in self.i)

    def draft_row(self, b, j):
        """Draft distribution of position j: stored p of its last evaluation,
        or uniform over the allowed ids if never evaluated."""
        if j in self.q[b]:
            return self.q[b][j]
        n = self.cfg.n_allowed
        # fp32(1/n) is what an fp32 implementation holds; keep that value.
        return np.full(n, np.float64(np.float32(1.0) / np.float32(n)))

    # -- phase 1: distributions ---------------------------------------------
    def evaluate(self, z_rows, keep_override=None, logit_err=None):
        """z_rows[b]: fp32 [Lw_b, |A|] processed logits of the window
        (after CFG, mask, temperature).  Returns plan[b][s] =
        dict(p, thr, lse, nkept, ambiguous, err).  thr is the smallest kept logit when a
        filter removed something, else -inf.  keep_override[(b, position)] = {id: kept}
        forces the membership of ids listed as ambiguous (top-k stage, then nucleus stage).

        Flags (what a second implementation may legitimately decide differently):
        logit_err[b][s] = sup-norm distance between this row's logits and the other
        implementation's (0 for bit-identical logits).  Ids within 2 * logit_err of a
        filter threshold are ambiguous (see _ambiguous_ids); a cumulative nucleus mass
        may be off by tol_mass + 2 * logit_err (every normalised probability moves by a
        factor within exp(+-2 e)).  Without logit_err an a-priori band is used:
        tol * (1 + 2 lambda) * max(1, |thr|) per logit (the guidance mix amplifies an
        LM-head error by 1 + 2 lambda), tol_mass per mass."""
        cfg = self.cfg
        plan = []
        for b in range(cfg.B):
            i, Lw = self.window(b)
            rows = []
            for s in range(Lw):
                z = np.asarray(z_rows[b][s], dtype=np.float32)
                thr = lg.topk_threshold(z, cfg.top_k)
                if logit_err is not None:
                    err = float(logit_err[b][s])
                    tol_z = 2.0 * err
                    tol_mass = self.tol_mass + 2.0 * err
                else:
                    err = None
                    tol_z = self.tol * max(1.0, abs(float(thr))) * (1.0 + 2.0 * cfg.cfg_lambda) \
                        if np.isfinite(thr) else 0.0
                    tol_mass = self.tol_mass
                amb = _ambiguous_ids(z, thr, cfg.top_k, tol_z)
                keep = z >= thr
                ov = (keep_override or {}).get((b, i + s))
                if ov:
                    for v, kv in ov.items():
                        if v in amb:
                            keep[v] = kv
                if 0.0 < cfg.top_p < 1.0:
                    thr_p = lg.nucleus_threshold(z, keep, cfg.top_p)
                    amb_p = _ambiguous_nucleus_ids(z, keep, cfg.top_p, tol_mass)
                    # ids tied with the last kept logit to within the logit tolerance: another
                    # rounding of the LM head may split the tie (same rule as at the top-k boundary)
                    tol_zp = tol_z if err is not None else \
                        self.tol * max(1.0, abs(float(thr_p))) * (1.0 + 2.0 * cfg.cfg_lambda)
                    near = np.nonzero(keep & (np.abs(z.astype(np.float64) - np.float64(thr_p)) <= tol_zp))[0]
                    if near.size > 1 and tol_zp > 0.0:
                        amb_p = np.union1d(amb_p, near)
                    keep = keep & (z >= thr_p)
                    if ov:
                        for v, kv in ov.items():
                            if v in amb_p:
                                keep[v] = kv
                    thr = np.float32(z[keep].min())
                    amb = np.union1d(amb, amb_p)
                if ov:
                    assert all(v in amb for v in ov), "membership override outside the ambiguous set"
                z64 = z.astype(np.float64)
                m = z64[keep].max()
                e = np.where(keep, np.exp(z64 - m), 0.0)
                ssum = e.sum()
                rows.append(dict(p=e / ssum, thr=thr, lse=m + np.log(ssum),
                                 nkept=int(keep.sum()), ambiguous=amb, err=err or 0.0))
            plan.append(rows)
        return plan

    # -- phase 2: one MRS per window position ------------------------------
    def sample(self, plan, accept_override=None, resid_override=None, gs_override=None):
        """Vectorised MRS (Alg. SCD(pi_MC), the parallel-for over the window); under
        pi_GS also the Gumbel draw g of every window position (Alg. SCD(pi_GS),
        "fixed noise sampling").  Overrides force a decision and are legal only on
        flagged draws.  A draw is flagged when a relative perturbation of its
        probabilities by tol + 2 (e_p + e_q) could flip it: tol covers the other side's fp32
        evaluation of exp and of the normaliser, e_p / e_q are the logit discrepancies
        the rows of p and q were evaluated with (p_v = exp(z_v - lse) moves by a factor
        within exp(+-2 e) when every logit moves by at most e).  flag_accept_strict is the
        same test at tol alone (the |u - p/q| < 1e-5 rule as stated)."""
        cfg = self.cfg
        res = []
        for b in range(cfg.B):
            i, Lw = self.window(b)
            t = self.t[b]
            rows = []
            for s in range(Lw):
                j = i + s
                p = plan[b][s]["p"]
                q = self.draft_row(b, j)
                x = int(self.X[b, j])
                u = philox.uniform_scalar(cfg.seed, b, j, t, philox.STREAM_ACCEPT)
                U_fn = lambda b=b, j=j, t=t: philox.uniform_per_vocab(
                    cfg.seed, b, j, t, philox.STREAM_RESID, cfg.n_allowed)
                tol = self.tol + 2.0 * (plan[b][s]["err"] + self.qerr[b].get(j, 0.0))
                r = mrs_mod.mrs(p, q, x, u, U_fn, tol)
                r["flag_accept_strict"] = mrs_mod.accept_flag(r["px"], r["qx"], u, self.tol)
                r["tol"] = tol
                r["u"] = u
                r["stats"] = dg.row_statistics(p, q)     # (beta, collision, sum p^2, sum q^2)
                key = (b, j)
                if accept_override and key in accept_override and accept_override[key] != r["k"]:
                    assert r["flag_accept"], "accept override on an unflagged draw"
                    forced = accept_override[key]
                    if forced:
                        r.update(y=x, k=1, flag_resid=False)
                    else:
                        U = U_fn()
                        w, _ = mrs_mod.residual_race(p, q, U)
                        r.update(y=w, k=0, flag_resid=mrs_mod.residual_flag(p, q, U, w, tol))
                if resid_override and key in resid_override and r["k"] == 0 \
                        and resid_override[key] != r["y"]:
                    assert r["flag_resid"], "residual override on an unflagged draw"
                    r["y"] = int(resid_override[key])
                # what a surviving position drafts next
                indep = False
                if cfg.alpha < 1.0:
                    # u <= alpha, decided in fp32 like every other threshold test of the path
                    ua = philox.uniform_scalar(cfg.seed, b, j, t, philox.STREAM_ALPHA)
                    indep = not (np.float32(ua) <= np.float32(cfg.alpha))
                r["indep"] = indep
                Ug = None
                if indep:          # fresh noise: keyed by the iteration too
                    Ug = philox.uniform_per_vocab(cfg.seed, b, j, t, philox.STREAM_INDEP,
                                                  cfg.n_allowed)
                elif cfg.coupling == "gs":   # shared noise: keyed by the position only
                    Ug = philox.uniform_per_vocab(cfg.seed, b, j, 0, philox.STREAM_GUMBEL,
                                                  cfg.n_allowed)
                if Ug is not None:
                    g, _ = gs_mod.draw(p, Ug)
                    r["flag_gs"] = gs_mod.flag(p, Ug, g, self.tol + 2.0 * plan[b][s]["err"])
                    if gs_override and key in gs_override and gs_override[key] != g:
                        assert r["flag_gs"], "Gumbel override on an unflagged draw"
                        g = int(gs_override[key])
                    r["g"] = g
                r["next"] = r["g"] if Ug is not None else r["y"]
                rows.append(r)
            res.append(rows)
        return res

    # -- phase 3: first rejection, emit, slide -----------------------------
    def commit(self, plan, res):
        cfg = self.cfg
        accept_len = []
        for b in range(cfg.B):
            i, Lw = self.window(b)
            if Lw == 0:
                accept_len.append(0)
                continue
            first_rej = Lw
            for s in range(Lw):
                if res[b][s]["k"] == 0:
                    first_rej = s
                    break
            a = min(first_rej + 1, Lw)
            for s in range(a):
                self.out[b, i + s] = cfg.v_lo + res[b][s]["y"]
            self._draft_hist[b] = ([(i, self.X[b].copy())] + self._draft_hist[b])[:3]
            survivors = list(range(i + a, i + Lw))
            self.last_hamming[b] = (dg.hamming(self.X[b, survivors],
                                               [res[b][j - i]["next"] for j in survivors]), len(survivors))
            for s in range(a, Lw):                    # survivors: coupled redraft
                j = i + s
                self.X[b, j] = res[b][s]["next"]
                self.q[b][j] = plan[b][s]["p"]
                self.qerr[b][j] = plan[b][s]["err"]
                self.age[b, j] += 1
            for s in range(a):                        # retired positions
                self.q[b].pop(i + s, None)
                self.qerr[b].pop(i + s, None)
            for j in range(i + Lw, min(i + a + cfg.L, cfg.N)):   # entering positions
                self._init_position(b, j)
            multi = []
            for n_back in range(3):
                if n_back < len(self._draft_hist[b]):
                    start, drafts = self._draft_hist[b][n_back]
                    both = range(i + a, min(start + cfg.L, cfg.N))       # in the new and in that window
                    multi.append((dg.hamming(drafts[both], self.X[b][both]), len(both)))
                else:
                    multi.append((0, 0))
            self.last_hamming_multi[b] = multi
            self.positions_verified += Lw
            self.i[b] = i + a
            self.t[b] += 1
            self.accept_hist[b].append(a)
            accept_len.append(a)
        return accept_len

    def step(self, z_rows):
        plan = self.evaluate(z_rows)
        res = self.sample(plan)
        return plan, res, self.commit(plan, res)


def decode(cfg: ScdConfig, model, tol=1e-5):
    """Run the vectorised form to the end.  model(b, i, Lw, tokens, t, age) ->
    fp32 [Lw, |A|] processed logits for positions i..i+Lw-1, where tokens[j] is
    the emitted token offset for j < i and the current draft for i <= j < i+Lw
    (row s may depend on tokens[:i+s] only), and age[s] counts the earlier
    evaluations of position i+s."""
    o = ScdOracle(cfg, tol)
    while not o.done():
        z_rows = []
        for b in range(cfg.B):
            i, Lw = o.window(b)
            if Lw == 0:
                z_rows.append(None)
                continue
            toks = np.concatenate([o.out[b, :i] - cfg.v_lo, o.X[b, i:i + Lw]])
            z_rows.append(model(b, i, Lw, toks, o.t[b], o.age[b, i:i + Lw].copy()))
        o.step(z_rows)
    return o


def decode_sequential(cfg: ScdConfig, model, tol=1e-5):
    """Pedagogical form (Sec. 4.1): Drafting / Evaluate / Verify-with-break.
    Returns (out [B, N], nfe [B], accept lengths per sequence)."""
    B, L, N, n = cfg.B, cfg.L, cfg.N, cfg.n_allowed
    uniform = np.full(n, np.float64(np.float32(1.0) / np.float32(n)))
    out = np.full((B, N), -1, dtype=np.int64)
    nfe, hist = [], []
    for b in range(B):
        X = {}          # draft token per position
        p_new = {}      # p^{t}   : newest evaluated distribution per position
        p_old = {}      # p^{t-1} : the one before (uniform if none)
        t_new = {}      # iteration whose Evaluate produced p_new
        age = {}
        for j in range(min(L, N)):
            X[j] = philox.init_token(cfg.seed, b, j, n)
        i, t, h = 0, 0, []
        while i < N:
            Lw = min(L, N - i)
            # Drafting: re-couple drafts whose newest distribution has not
            # been used on them yet (positions right of the last rejection).
            for j in range(i, i + Lw):
                if j in p_new:
                    ua = philox.uniform_scalar(cfg.seed, b, j, t_new[j], philox.STREAM_ALPHA)
                    if cfg.alpha < 1.0 and not (np.float32(ua) <= np.float32(cfg.alpha)):
                        Ui = philox.uniform_per_vocab(cfg.seed, b, j, t_new[j], philox.STREAM_INDEP, n)
                        X[j] = gs_mod.draw(p_new[j], Ui)[0]
                    elif cfg.coupling == "gs":
                        Ug = philox.uniform_per_vocab(cfg.seed, b, j, 0, philox.STREAM_GUMBEL, n)
                        X[j] = gs_mod.draw(p_new[j], Ug)[0]
                    else:
                        u = philox.uniform_scalar(cfg.seed, b, j, t_new[j], philox.STREAM_ACCEPT)
                        U_fn = lambda j=j: philox.uniform_per_vocab(
                            cfg.seed, b, j, t_new[j], philox.STREAM_RESID, n)
                        r = mrs_mod.mrs(p_new[j], p_old.get(j, uniform), X[j], u, U_fn, tol)
                        X[j] = r["y"]
                    p_old[j] = p_new.pop(j)
            # Evaluate
            toks = np.array([out[b, j] - cfg.v_lo for j in range(i)] +
                            [X[j] for j in range(i, i + Lw)], dtype=np.int64)
            ages = np.array([age.get(j, 0) for j in range(i, i + Lw)])
            z = model(b, i, Lw, toks, t, ages)
            for s in range(Lw):
                j = i + s
                p_new[j], _, _ = lg.distribution(z[s], cfg.top_k, cfg.top_p)
                t_new[j] = t
                age[j] = age.get(j, 0) + 1
            # Verify, sequentially, break at the first rejection
            j = i
            while j < i + Lw:
                u = philox.uniform_scalar(cfg.seed, b, j, t, philox.STREAM_ACCEPT)
                U_fn = lambda j=j: philox.uniform_per_vocab(
                    cfg.seed, b, j, t, philox.STREAM_RESID, n)
                r = mrs_mod.mrs(p_new[j], p_old.get(j, uniform), X[j], u, U_fn, tol)
                out[b, j] = cfg.v_lo + r["y"]
                for dct in (p_new, p_old, X):
                    dct.pop(j, None)
                j += 1
                if r["k"] == 0:
                    break
            a = j - i
            for jn in range(i + Lw, min(i + a + L, N)):
                X[jn] = philox.init_token(cfg.seed, b, jn, n)
            i, t = j, t + 1
            h.append(a)
        nfe.append(t)
        hist.append(h)
    return out, nfe, hist
