"""Lock-step driver for the GPU parity tests: runs the HIP path (through the C
ABI) and the CPU oracle side by side on the same seeded inputs, one decode
iteration at a time, and compares everything the iteration produces.

Integer results (tokens, accept bits, accept lengths, positions, ages,
thresholds' kept-set sizes) must be identical, except on draws the oracle flags
as numerically fragile.  Every flag is derived from ONE measured number per row,
e = max_v |z_gpu[v] - z_oracle[v]| (0 when the logits are supplied):
  * top-k / nucleus membership: ids within 2 e of the threshold (an order statistic
    and every logit move by at most e), cumulative masses within 2e-6 + 2 e;
  * accept draws with |u - p(x)/q(x)| < 1e-5 + 2 (e_p + e_q), residual and Gumbel races
    that a relative perturbation of that size in the probabilities could flip
    (1e-5 = the stated rule, covering the fp32 exp / normaliser; the rest is how far
    exp(z - lse) moves when every logit moves by e).  Draws inside the stated 1e-5
    band alone are counted separately (flag_accept_strict).
On a flagged draw that differs the oracle adopts the GPU's decision, the event is
counted, and both continue from the same state.  Any unflagged difference fails.

Floating-point results: processed logits within 2e-3 relative (the stated bf16-GEMM
bar) AND within `logit_cap` absolute, a bound derived from fp32 accumulation
(4 * 2^-24 * sqrt(d) * (1 + 2 lambda) / tau * max(1, rms of the raw logits), about 3x the
largest error observed); kept-set thresholds within e (exact for supplied logits);
log normalisers within e + 1e-6 relative; p(x), q(x) within 2 e + 4e-6 relative.
"""
import numpy as np
import torch

from oracle import logits as lg
from oracle import scd as oscd
from paper_2510_24211_amd import binding as B
from paper_2510_24211_amd import workload as wl


def bf16_tensor(bits_np, device):
    return torch.from_numpy(bits_np.view(np.int16)).to(device).view(torch.bfloat16)


_W_CACHE = {}      # the last LM-head weight: (bf16 on the device, allowed rows as fp64 on the host)


def _weights(w, device):
    key = (w.seed, w.V, w.d, w.w_std, w.v_lo, w.v_hi, str(device))
    if key not in _W_CACHE:
        _W_CACHE.clear()
        W = wl.lm_head_weight(w)
        _W_CACHE[key] = (bf16_tensor(W, device), lg.bf16_bits_to_f64(W[w.v_lo:w.v_hi]))
    return _W_CACHE[key]


class LockStep:
    def __init__(self, w: wl.Workload, device="cuda:0", coupling="mc", sjd_mix=0.0, diagnostics=False):
        self.w = w
        self.device = device
        self.coupling = coupling
        self.cfg_c = B.config_from_workload(w)
        self.cfg_c.coupling = B.COUPLING_GS if coupling == "gs" else B.COUPLING_MC
        self.cfg_c.sjd_mix = sjd_mix
        self.cfg_c.diagnostics = int(diagnostics)
        self.diagnostics = diagnostics
        # the library's alpha is fl32(1 - sjd_mix); the oracle gets exactly that number
        alpha = float(np.float32(1.0) - np.float32(self.cfg_c.sjd_mix))
        self.has_g = coupling == "gs" or sjd_mix > 0
        self.gpu = B.Scd(self.cfg_c, device)
        self.state = self.gpu.alloc_state()
        self.gpu.reset(self.state)
        self.ocfg = oscd.ScdConfig(B=w.B, L=w.L, N=w.N, V=w.V, v_lo=w.v_lo, v_hi=w.v_hi,
                                   top_k=w.top_k, top_p=w.top_p, temperature=w.temperature,
                                   cfg_lambda=w.cfg_lambda, seed=w.seed, coupling=coupling,
                                   alpha=alpha)
        self.oracle = oscd.ScdOracle(self.ocfg)
        self.n = w.n_allowed
        if w.d > 0:
            self.W_gpu, self.W64 = _weights(w, device)
            self.table = wl.HiddenTable(w)
        else:
            self.toy = wl.ToyLogits(w)
        f = self.gpu.state_field
        self.v = {name: f(self.state, fid) for name, fid in [
            ("pos", B.F_POS), ("iter", B.F_ITER), ("X", B.F_X), ("age", B.F_AGE), ("out", B.F_OUT),
            ("acc", B.F_ACCEPT), ("y", B.F_Y), ("k", B.F_K), ("px", B.F_PX), ("qx", B.F_QX),
            ("thr", B.F_THR), ("lse", B.F_LSE), ("nkept", B.F_NKEPT), ("z", B.F_Z),
            ("verified", B.F_VERIFIED), ("g", B.F_G), ("diag", B.F_DIAG), ("hamm", B.F_HAMM)]}
        self.stats = dict(steps=0, draws=0, flag_accept=0, flag_accept_strict=0, flag_resid=0,
                          flag_topk=0, flag_gs=0,
                          adopt_accept=0, adopt_accept_strict=0, adopt_resid=0, adopt_topk=0, adopt_gs=0,
                          max_logit_abs=0.0, max_logit_rel=0.0, max_lse_abs=0.0, max_prob_rel=0.0,
                          max_logit_abs_over_cap=0.0)
        self.check_initial_state()

    # ------------------------------------------------------------------
    def check_initial_state(self):
        w, o = self.w, self.oracle
        X = self.v["X"].cpu().numpy().reshape(w.B, w.L)
        for b in range(w.B):
            for j in range(min(w.L, w.N)):
                assert X[b, j] == o.X[b, j], "initial draft differs"
        assert (self.v["out"].cpu().numpy() == -1).all()

    def _windows(self):
        o, w = self.oracle, self.w
        ages = [[int(o.age[b, o.i[b] + s]) if o.i[b] + s < w.N else 0 for s in range(w.L)]
                for b in range(w.B)]
        return list(o.i), ages

    def step(self):
        w, o, st, v = self.w, self.oracle, self.stats, self.v
        Bn, L, n = w.B, w.L, self.n
        i_b, ages = self._windows()
        t_b = list(o.t)
        lives = [o.window(b)[1] for b in range(Bn)]
        # ---- the same input bytes to both sides -----------------------------
        if w.d > 0:
            h = self.table.window(i_b, ages)                       # [B, C, L, d] bf16 bits
            self.gpu.step(bf16_tensor(h, self.device), self.W_gpu, self.state)
            z_rows, c_rows, u_rows = [], [], []
            for b in range(Bn):
                Lw = lives[b]
                if Lw == 0:
                    z_rows.append(None)
                    c_rows.append(None)
                    u_rows.append(None)
                    continue
                c = lg.lm_head(h[b, 0, :Lw], self.W64)
                u = lg.lm_head(h[b, 1, :Lw], self.W64) if w.C == 2 else None
                c_rows.append(c)
                u_rows.append(u)
                z_rows.append(lg.process_logits(c, u, w.cfg_lambda, w.temperature))
        else:
            z = self.toy.window(i_b, ages)                         # [B, L, n] fp32
            self.gpu.step_logits(torch.from_numpy(z).to(self.device), self.state)
            # scd_step_logits takes logits that are already processed: no guidance mix, no 1/tau
            z_rows = [lg.process_logits(z[b, :lives[b]], None, 0.0, 1.0)
                      if lives[b] else None for b in range(Bn)]
        rc, flags = self.gpu.status(self.state)
        assert rc == B.SCD_OK, (rc, flags)

        # ---- download what the step produced --------------------------------
        g = {k: v[k].cpu().numpy() for k in ("pos", "iter", "X", "age", "acc", "y", "k", "px",
                                             "qx", "thr", "lse", "nkept", "verified", "g", "diag",
                                             "hamm")}
        g["thr"] = g["thr"].reshape(2, Bn, L)
        g["lse"] = g["lse"].reshape(2, Bn, L)
        g["nkept"] = g["nkept"].reshape(2, Bn, L)
        zg = v["z"].view(2, Bn, L, n)

        # ---- distributions: logits, threshold, normaliser --------------------
        # e[b][s]: sup-norm distance between the two sides' logits of the row -- the one
        # number every flag and every floating-point tolerance below is derived from
        errs = []
        for b in range(Bn):
            par = t_b[b] & 1
            eb = []
            if lives[b]:
                zgb = zg[par, b].cpu().numpy()                     # [L, n] by ring slot
                if w.d > 0:
                    raw = [c_rows[b]] + ([u_rows[b]] if u_rows[b] is not None else [])
            for s in range(lives[b]):
                slot = (i_b[b] + s) % L
                zo = z_rows[b][s]
                zgr = zgb[slot]
                if w.d == 0:
                    assert np.array_equal(zgr, zo), "supplied logits must be stored bit-exactly"
                    eb.append(0.0)
                    continue
                diff = np.abs(zgr.astype(np.float64) - zo)
                e = float(diff.max())
                assert np.isfinite(e), "non-finite logit"
                st["max_logit_abs"] = max(st["max_logit_abs"], e)
                scale = np.maximum(np.abs(zo), float(np.sqrt(np.mean(zo.astype(np.float64) ** 2))))
                rel = float((diff / scale).max())
                st["max_logit_rel"] = max(st["max_logit_rel"], rel)
                assert rel <= 2e-3, f"logit relative error {rel}"
                rms = max(1.0, max(float(np.sqrt(np.mean(r_[s].astype(np.float64) ** 2))) for r_ in raw))
                cap = 4 * 2.0 ** -24 * np.sqrt(w.d) * (1 + 2 * abs(w.cfg_lambda)) * rms / w.temperature
                st["max_logit_abs_over_cap"] = max(st["max_logit_abs_over_cap"], e / cap)
                assert e <= cap, f"logit abs error {e} above the fp32-accumulation bound {cap}"
                eb.append(e)
            errs.append(eb)
        keep_override = {}
        plan = o.evaluate(z_rows, logit_err=errs)
        for b in range(Bn):
            par = t_b[b] & 1
            for s in range(lives[b]):
                slot = (i_b[b] + s) % L
                row = plan[b][s]
                zo = z_rows[b][s]
                amb = row["ambiguous"]
                if len(amb):
                    st["flag_topk"] += 1
                    zamb = zg[par, b, slot][torch.from_numpy(amb).to(self.device)].cpu().numpy()
                    gmem = zamb >= g["thr"][par, b, slot]
                    omem = zo[amb] >= row["thr"]
                    if not np.array_equal(gmem, omem):
                        keep_override[(b, i_b[b] + s)] = {int(vv): bool(m) for vv, m in zip(amb, gmem)}
        if keep_override:
            st["adopt_topk"] += len(keep_override)
            plan = o.evaluate(z_rows, keep_override, logit_err=errs)
        for b in range(Bn):
            par = t_b[b] & 1
            for s in range(lives[b]):
                slot = (i_b[b] + s) % L
                row = plan[b][s]
                e = errs[b][s]
                assert g["nkept"][par, b, slot] == row["nkept"], \
                    f"kept-set size b={b} s={s}: gpu {g['nkept'][par, b, slot]} oracle {row['nkept']}"
                thr_g, thr_o = g["thr"][par, b, slot], row["thr"]
                if e == 0.0 or not np.isfinite(thr_o):
                    assert thr_g == thr_o, f"threshold differs: {thr_g} vs {thr_o}"
                else:     # the smallest logit of the same kept set on either side
                    assert abs(float(thr_g) - float(thr_o)) <= e, f"threshold differs: {thr_g} vs {thr_o} (e = {e})"
                dl = abs(float(g["lse"][par, b, slot]) - row["lse"])
                st["max_lse_abs"] = max(st["max_lse_abs"], dl)
                assert dl <= e + 1e-6 * max(1.0, abs(row["lse"])), f"lse differs by {dl} (e = {e})"

        # ---- one MRS per window position -----------------------------------
        res = o.sample(plan)
        acc_ov, res_ov, gs_ov = {}, {}, {}
        gg = g["g"].reshape(Bn, L)
        gk = g["k"].reshape(Bn, L)
        gy = g["y"].reshape(Bn, L)
        gpx = g["px"].reshape(Bn, L)
        gqx = g["qx"].reshape(Bn, L)
        for b in range(Bn):
            for s in range(lives[b]):
                r = res[b][s]
                key = (b, i_b[b] + s)
                st["draws"] += 1
                st["flag_accept"] += r["flag_accept"]
                st["flag_accept_strict"] += r["flag_accept_strict"]
                st["flag_resid"] += r["flag_resid"]
                e_p, e_q = errs[b][s], o.qerr[b].get(i_b[b] + s, 0.0)
                for gval, oval, e in ((gpx[b, s], r["px"], e_p), (gqx[b, s], r["qx"], e_q)):
                    err = abs(float(gval) - oval)
                    rel = err / max(oval, 1e-30) if oval > 0 else (0.0 if gval == 0 else np.inf)
                    if oval > 1e-30:
                        st["max_prob_rel"] = max(st["max_prob_rel"], rel)
                    assert rel <= 2 * e + 4e-6 or err <= 1e-12, \
                        f"p(x)/q(x) differs: gpu {gval} oracle {oval} (e = {e})"
                if int(gk[b, s]) != r["k"]:
                    assert r["flag_accept"], \
                        f"accept bit differs on an unflagged draw b={b} s={s}: u={r['u']} px={r['px']} qx={r['qx']}"
                    acc_ov[key] = int(gk[b, s])
                    st["adopt_accept_strict"] += r["flag_accept_strict"]
                elif r["k"] == 0 and int(gy[b, s]) != r["y"]:
                    assert r["flag_resid"], f"residual token differs on an unflagged draw b={b} s={s}"
                    res_ov[key] = int(gy[b, s])
                if "g" in r:
                    st["flag_gs"] += r["flag_gs"]
                    if int(gg[b, s]) != r["g"]:
                        assert r["flag_gs"], f"Gumbel draw differs on an unflagged draw b={b} s={s}"
                        gs_ov[key] = int(gg[b, s])
        if acc_ov or res_ov or gs_ov:
            st["adopt_accept"] += len(acc_ov)
            st["adopt_gs"] += len(gs_ov)
            res = o.sample(plan, acc_ov, res_ov, gs_ov)
            for (b, j), kk in acc_ov.items():     # a forced rejection resamples: token may be flagged too
                s = j - i_b[b]
                if kk == 0 and res[b][s]["y"] != int(gy[b, s]):
                    assert res[b][s]["flag_resid"]
                    res_ov[(b, j)] = int(gy[b, s])
            st["adopt_resid"] += len(res_ov)
            if res_ov:
                res = o.sample(plan, acc_ov, res_ov, gs_ov)
        for b in range(Bn):
            for s in range(L):
                if s < lives[b]:
                    assert int(gk[b, s]) == res[b][s]["k"] and int(gy[b, s]) == res[b][s]["y"]
                    if self.has_g:      # -1 where the row made no Gumbel-max draw
                        assert int(gg[b, s]) == res[b][s].get("g", -1)
                else:
                    assert int(gk[b, s]) == 1 and int(gy[b, s]) == -1
                    if self.has_g:
                        assert int(gg[b, s]) == -1

        # ---- per-position statistics ---------------------------------------
        if self.diagnostics:
            gd = g["diag"].reshape(Bn, L, 4)
            for b in range(Bn):
                for s in range(L):
                    if s >= lives[b]:
                        assert not gd[b, s].any()
                        continue
                    e2 = errs[b][s] + o.qerr[b].get(i_b[b] + s, 0.0)
                    for got, want in zip(gd[b, s], res[b][s]["stats"]):
                        err = abs(float(got) - want)
                        st["max_stat_rel"] = max(st.get("max_stat_rel", 0.0), err / max(want, 1e-30))
                        assert err <= 4 * (2 * e2 + 4e-6) * want + 1e-9, \
                            f"statistic differs b={b} s={s}: gpu {gd[b, s]} oracle {res[b][s]['stats']}"

        # ---- commit --------------------------------------------------------
        acc = o.commit(plan, res)
        if self.diagnostics:
            gh = g["hamm"].reshape(Bn, 3, 2)
            for b in range(Bn):
                if lives[b]:
                    want = [tuple(x) for x in o.last_hamming_multi[b]]
                    got = [tuple(int(x) for x in pair) for pair in gh[b]]
                    assert got == want, f"changed drafts differ: gpu {got} oracle {want}"
                    assert got[0] == o.last_hamming[b]
                else:
                    assert not gh[b].any()
        assert list(g["acc"]) == acc, f"accept lengths differ: {list(g['acc'])} vs {acc}"
        assert list(g["pos"]) == list(o.i) and list(g["iter"]) == list(o.t)
        assert int(g["verified"].sum()) == o.positions_verified
        gX = g["X"].reshape(Bn, L)
        gage = g["age"].reshape(Bn, L)
        for b in range(Bn):
            i, Lw = o.window(b)
            for s in range(Lw):
                slot = (i + s) % L
                assert gX[b, slot] == o.X[b, i + s], "draft token differs after the slide"
                assert gage[b, slot] == o.age[b, i + s], "age differs after the slide"
        st["steps"] += 1
        return acc

    def run(self, max_steps=None):
        import os, time
        # a long decode reports where it is twice a minute (a file a watcher can see grow)
        root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
        os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
        last = time.monotonic()
        while not self.oracle.done() and (max_steps is None or self.stats["steps"] < max_steps):
            self.step()
            if time.monotonic() - last > 30.0:
                last = time.monotonic()
                with open(os.path.join(root, "gpurun_out", "lockstep_progress.log"), "a") as f:
                    f.write(f"{self.w.name}: {self.stats['steps']} iterations, positions {list(self.oracle.i)}\n")
        out_g = self.v["out"].cpu().numpy().reshape(self.w.B, self.w.N)
        assert np.array_equal(out_g, self.oracle.out), "emitted tokens differ"
        if self.oracle.done():
            rc, flags = self.gpu.status(self.state)
            assert flags[1] == 1 and flags[2] == max(self.oracle.t)
        return self.stats
