#!/usr/bin/env python3
"""Benchmark of the SCD draft-and-verify step on one MI355X.

A "step" is one whole decode iteration (scd_step: LM-head GEMM + CFG +
temperature, top-k select + softmax normaliser, vectorised MRS, first
rejection / emit / window slide) over the synthetic workload's current Jacobi
windows.  The windows' hidden states (which depend on the decode state) are
assembled for every step by an untimed recording decode, so all inputs are
resident in HBM before the timed region starts; nothing crosses PCIe inside it.

Prints ONE JSON line.  The top level is the full-vocabulary workload (C2-fullV: every one of
the V = 65536 ids allowed, the stream the ">= 70 % of HBM" target is stated on): `value` =
window positions verified per second, `tokens_per_s` = emitted tokens per second, both from the
MEDIAN of `repeats` timed passes of exactly `steps` steps each (the passes continue one decode
after `warmup` untimed steps; `ms_per_step_min` / `_max` give the spread).  `roofline` describes
the dominant kernel (the LM-head stream over W), timed with HIP events attached to the LM-head
dispatch inside scd_step (they take the kernel's own start and stop time on the stream it runs
on) in one more identical pass (a step launched that way is about a microsecond slower, so
`value` never comes from it); `roofline.step_frac` is the whole step against the same peak:
algorithmic step bytes / median step time / 8 TB/s.  `companions` holds the same measurement of
the other workloads (C2 as specified = 8192 allowed ids, C1, C3, C4) with the same --steps /
--warmup / --repeats.  `cpu_baseline` is the NumPy oracle timed on the host cores on a bounded
sample of the top-level workload, with the number of draws it flags as numerically fragile.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps; 0 = one whole decode")
    ap.add_argument("--warmup", type=int, default=0, help="untimed steps; 0 = one whole decode")
    ap.add_argument("--workload", default=None,
                    help="C1 | C2 | C2-fullV | C3 | C4 | C4-topp (see paper_2510_24211_amd/workload.py): "
                         "measure this workload alone.  Default: C2-fullV at the top level and "
                         "C2, C1, C3, C4 as `companions`")
    ap.add_argument("--repeats", type=int, default=5,
                    help="timed passes of --steps steps each; value = their median (default 5)")
    ap.add_argument("--no-companions", action="store_true",
                    help="default run only: skip the companion workloads")
    ap.add_argument("--diagnostics", action="store_true",
                    help="also compute the per-position statistics in every step (config.diagnostics) "
                         "and report their means over the recorded decode")
    ap.add_argument("--coupling", default="mc", choices=["mc", "gs"],
                    help="mc: maximal coupling (the paper's pi_MC, default); gs: Gumbel sharing (pi_GS)")
    ap.add_argument("--sjd-mix", type=float, default=0.0,
                    help="1 - alpha of the alpha-coupling: probability that a redraft is an independent "
                         "draw (0 = SCD, default; 1 = vanilla SJD)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--quick", action="store_true",
                    help="profiling aid: skip the whole-decode warm-up, run --warmup then --steps "
                         "iterations from a fresh state (both must be given and fit in one decode)")
    ap.add_argument("--no-events", action="store_true",
                    help="do not record the per-step LM-head events (no roofline object)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="profiling aid: run 20 launches of the library's plain copy kernel over MIB "
                         "MiB and exit (scales a profiler's HBM byte counters)")
    return ap.parse_args()


class HipEvents:
    """hipEvent_t pairs created through the HIP runtime (ctypes)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.ev = []
        for _ in range(2 * n):
            e = ctypes.c_void_p()
            # hipEventDisableSystemFence: such an event does not flush the caches to system scope
            # (nothing is read by the host at these points: the stream is synchronised before
            # any result is read).
            assert self.hip.hipEventCreateWithFlags(ctypes.byref(e), 0x20000000) == 0
            self.ev.append(e)

    def pair(self, i):
        return self.ev[2 * i].value, self.ev[2 * i + 1].value

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.ev[2 * i], self.ev[2 * i + 1])
        assert rc == 0, rc
        return ms.value

    def destroy(self):
        for e in self.ev:
            self.hip.hipEventDestroy(e)


def cpu_baseline(w, seconds, coupling="mc", sjd_mix=0.0):
    """The oracle as it stands, on the host cores, for about `seconds` (whole decodes are
    repeated until the time is up; the last one may be cut short).  Also counts the draws the
    oracle flags as numerically fragile on that sample (its a-priori bands: |u - p/q| < 1e-5, a
    residual race that a 1e-5 relative perturbation could flip, a top-k boundary with another
    logit within 1e-5 (1 + 2 lambda) max(1, |thr|)): the draws on which a second implementation
    is allowed to decide differently."""
    import numpy as np
    from oracle import logits as lg
    from oracle import scd as oscd
    from paper_2510_24211_amd import workload as wl
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    W = wl.lm_head_weight(w)
    W64 = lg.bf16_bits_to_f64(W[w.v_lo:w.v_hi])
    del W
    tab = wl.HiddenTable(w)
    cfg = oscd.ScdConfig(B=w.B, L=w.L, N=w.N, V=w.V, v_lo=w.v_lo, v_hi=w.v_hi, top_k=w.top_k,
                         top_p=w.top_p, temperature=w.temperature, cfg_lambda=w.cfg_lambda, seed=w.seed,
                         coupling=coupling, alpha=float(np.float32(1.0) - np.float32(sjd_mix)))
    o = oscd.ScdOracle(cfg)
    tab.window(list(o.i), [[0] * w.L for _ in range(w.B)])      # warm the generator caches
    t_in = 0.0
    steps = positions = tokens = decodes = 0
    flagged = dict(draws=0, accept=0, residual=0)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 - t_in < seconds:
        if o.done():
            positions += o.positions_verified
            tokens += int(sum(o.i))
            decodes += 1
            o = oscd.ScdOracle(cfg)
        ti = time.perf_counter()
        ages = [[int(o.age[b, o.i[b] + s]) if o.i[b] + s < w.N else 0 for s in range(w.L)]
                for b in range(w.B)]
        h = tab.window(list(o.i), ages)
        t_in += time.perf_counter() - ti          # input generation is not the method
        z_rows = []
        for b in range(w.B):
            Lw = o.window(b)[1]
            if Lw == 0:
                z_rows.append(None)
                continue
            c = lg.lm_head(h[b, 0, :Lw], W64)
            u = lg.lm_head(h[b, 1, :Lw], W64) if w.C == 2 else None
            z_rows.append(lg.process_logits(c, u, w.cfg_lambda, w.temperature))
        plan, res, _ = o.step(z_rows)
        ti = time.perf_counter()                  # reading the flags off is not the method either
        for rows_p, rows_r in zip(plan, res):
            for rp, rr in zip(rows_p, rows_r):
                flagged["draws"] += 1
                flagged["accept"] += int(rr["flag_accept_strict"])
                flagged["residual"] += int(rr["flag_resid"])
        t_in += time.perf_counter() - ti
        steps += 1
    T = time.perf_counter() - t0 - t_in
    positions += o.positions_verified
    tokens += int(sum(o.i))
    return {"value": positions / T, "unit": "positions/s", "cores": int(threads),
            "kind": "oracle", "tokens_per_s": float(tokens) / T,
            "sample": f"{steps} iterations of {w.name} ({decodes} whole decodes and the start of the "
                      f"next; {positions} window positions, {tokens} tokens) in {T:.1f} s, NumPy fp64",
            # draws of this oracle-only sample within 1e-5 of a tie (accept test: |u q - p| < 1e-5 q;
            # residual race: a relative perturbation of 1e-5 could change the winner); what the
            # GPU parity runs flagged and adopted is under "parity_flags"
            "flagged_draws": flagged}


COMPANIONS = ("C2", "C1", "C3", "C4")
# what a companion object keeps of a workload's result
COMPANION_KEYS = ("value", "unit", "tokens_per_s", "steps", "warmup", "repeats", "ms_per_step",
                  "ms_per_step_min", "ms_per_step_max", "config", "roofline", "parity_flags")


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures ONE MI355X; --gpus must be 1 "
              "(no multi-GPU path exists in this repository)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2510_24211_amd import binding as B
    from paper_2510_24211_amd import workload as wl

    if a.copy_calibration > 0:
        assert torch.cuda.is_available(), "bench.py needs the GPU"
        nbytes = a.copy_calibration << 20
        src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(20):
            B.device_copy(src, dst)
        torch.cuda.synchronize()
        assert bool((dst[-4:] == 1).all())
        print(json.dumps({"copy_kernel_launches": 20, "bytes_read_per_launch": nbytes,
                          "bytes_written_per_launch": nbytes}))
        return

    top = a.workload or "C2-fullV"
    out, w = measure(a, top, inputs := {})
    if a.workload is None and not a.quick and not a.no_companions:
        out["companions"] = {}
        for name in COMPANIONS:
            print(f"bench.py: companion workload {name}", file=sys.stderr, flush=True)
            r, _ = measure(a, name, inputs)
            out["companions"][name] = {k: r[k] for k in COMPANION_KEYS}
    inputs.clear()
    if not a.no_cpu_baseline:
        print("bench.py: CPU oracle baseline", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(w, a.cpu_seconds, a.coupling, a.sjd_mix)
    print(json.dumps(out))


def measure(a, name, inputs):
    """Runs workload `name` on cuda:0 and returns (its result dict, the Workload)."""
    import numpy as np
    import torch
    from paper_2510_24211_amd import binding as B
    from paper_2510_24211_amd import workload as wl

    w = wl.WORKLOADS[name]
    assert w.d > 0, "the benchmark runs the LM-head path"
    dev = "cuda:0"
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    torch.cuda.set_device(0)

    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    t_setup = time.perf_counter()
    # W and the hidden-state table depend on the shape and the seed only, not on the allowed ids
    key = (w.V, w.d, w.B, w.C, w.N, w.age_cap, w.seed, w.decay, w.frames)
    if inputs.get("key") != key:
        inputs.clear()
        torch.cuda.empty_cache()
        inputs.update(key=key, W=to_dev(wl.lm_head_weight(w)), table=to_dev(wl.HiddenTable(w).full()))
    W, table = inputs["W"], inputs["table"]
    cfg = B.config_from_workload(w)
    cfg.coupling = B.COUPLING_GS if a.coupling == "gs" else B.COUPLING_MC
    cfg.sjd_mix = a.sjd_mix
    cfg.diagnostics = int(a.diagnostics)
    s = B.Scd(cfg, dev)
    st = s.alloc_state()
    t_setup = time.perf_counter() - t_setup

    # ---- recording pass (untimed; also the warm-up of the caches) -------------------------
    # The hidden states of a step depend on the decode state (window start and ages), which
    # lives on the device.  One untimed decode assembles every step's [B, C, L, d] input with
    # the device-side gather and keeps it, so that the timed steps below find their inputs
    # resident in HBM and consist of scd_step alone.  The trajectory is deterministic (same
    # seed, same kernels), which the comparison of the window starts after every timed pass
    # confirms.  Per recorded step it also keeps the running totals of verified positions and
    # emitted tokens, from which the work of any range of steps follows.
    CH = 64
    chunks = []

    def h_of(i):
        while i // CH >= len(chunks):
            chunks.append(torch.empty((CH, w.B, w.C, w.L, w.d), dtype=torch.bfloat16, device=dev))
        return chunks[i // CH][i % CH]

    diag_sum = torch.zeros(4, dtype=torch.float64, device=dev)     # beta, C, bound, live rows
    hamm_sum = torch.zeros(6, dtype=torch.int64, device=dev)       # (differing, compared) for 1, 2, 3 iterations apart
    totals = []                                                    # per step: [verified, tokens] so far (device)
    pos_after = []                                                 # per step: window starts after it (device)

    def record(limit):
        """Decode from a fresh state, at most `limit` steps; returns the iteration count."""
        s.reset(st)
        i = 0
        while i < limit:
            for _ in range(min(16, limit - i)):
                hi = h_of(i)
                s.gather_hidden(table, w.age_cap, st, hi)
                s.step(hi, W, st)
                pos = s.state_field(st, B.F_POS)
                totals.append(torch.stack([s.state_field(st, B.F_VERIFIED).sum(), pos.sum()]))
                pos_after.append(pos.clone())
                if a.diagnostics:                 # rows that are not live hold zeros
                    d = s.state_field(st, B.F_DIAG).view(-1, 4).double()
                    diag_sum[0] += d[:, 0].sum()
                    diag_sum[1] += d[:, 1].sum()
                    diag_sum[2] += (d[:, 2] * d[:, 3]).sqrt().sum()
                    diag_sum[3] += (d[:, 2] > 0).sum()
                    hamm_sum.add_(s.state_field(st, B.F_HAMM).view(-1, 6).sum(0))
                i += 1
            rc, flags = s.status(st)
            assert rc == B.SCD_OK, (rc, flags)
            if flags[1]:
                return flags[2]
        return i

    R = max(1, a.repeats)
    if a.quick:
        assert a.steps > 0 and a.warmup > 0, "--quick needs --steps and --warmup"
        nfe = record(a.warmup + (R + 1) * a.steps)   # the decode may end earlier: then steps wrap
    else:
        nfe = record(1 << 30)                     # whole decode
    tot = torch.stack(totals[:nfe]).cpu().numpy().astype(np.int64)       # [nfe, 2] cumulative
    per_step = np.diff(np.concatenate([np.zeros((1, 2), dtype=np.int64), tot]), axis=0)
    whole = not a.quick
    K = a.steps if a.steps > 0 else nfe
    Wm = a.warmup
    hs = [h_of(i) for i in range(nfe)]            # views, made outside the timed loops

    cursor = [0]                                  # next recorded step

    def run_steps(count, with_events=None):
        """Enqueues `count` steps that continue the decode (a finished decode is followed by a
        fresh one); returns the recorded indices of the steps."""
        idx = []
        for i in range(count):
            if cursor[0] == nfe:
                s.reset(st)
                cursor[0] = 0
            if with_events is not None:
                s.set_lm_head_events(*with_events.pair(i))
            s.step(hs[cursor[0]], W, st)
            idx.append(cursor[0])
            cursor[0] += 1
        return idx

    def check_reproduced():
        got = s.state_field(st, B.F_POS)
        assert torch.equal(got, pos_after[cursor[0] - 1]), "decode is not reproducible"

    def timed_pass(ev=None):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        idx = run_steps(K, ev)
        t_enq = time.perf_counter() - t0
        torch.cuda.synchronize()
        T = time.perf_counter() - t0
        if ev is not None:
            s.set_lm_head_events(None, None)
        check_reproduced()
        work = per_step[idx].sum(axis=0)
        return dict(T=T, verified=int(work[0]), tokens=int(work[1]), enqueue_us=t_enq / K * 1e6,
                    first_step=int(idx[0]))

    # The passes are spread evenly over the decode (untimed steps between them): its first
    # iterations, where every draft is a fresh uniform draw and nearly every row rejects, are a
    # transient of a few percent of the decode and would otherwise be all that K << nfe steps see.
    gap = max(0, (nfe - Wm - R * K) // R) if whole else 0
    s.reset(st)
    if Wm > 0:
        run_steps(Wm)
    passes = []
    for r in range(R):
        passes.append(timed_pass())
        if gap and r + 1 < R:
            run_steps(gap)
    # A step whose LM head carries the events is about a microsecond slower (the dispatch then
    # reports its timestamps), so the throughput comes from the passes without them and the
    # LM-head timing from one more identical pass with them.
    use_events = not a.no_events
    lm_ms = T_ev = None
    if use_events:
        ev = HipEvents(K)
        T_ev = timed_pass(ev)["T"]
        lm_ms = float(np.mean([ev.elapsed_ms(i) for i in range(K)]))
        ev.destroy()
    rc, flags = s.status(st)
    assert rc == B.SCD_OK

    order = sorted(range(R), key=lambda r: passes[r]["T"])
    med = passes[order[(R - 1) // 2]]             # the median pass (lower median for an even count)
    T = med["T"]

    n = w.n_allowed
    w_bytes = 2 * w.d * n
    h_bytes = 2 * w.M * w.d
    alg_bytes = w_bytes + h_bytes               # per LM-head launch (W slice once + hidden rows)
    step_bytes = alg_bytes + 2 * w.B * w.L * min(n, w.top_k or n) * 8   # + the sparse q-state, read and written
    flops = 2.0 * w.M * w.d * n
    resident = w_bytes <= 192 * 1024 * 1024      # the library's own rule for keeping W in the caches
    mfma_bound = w.M > 310                       # GEMM intensity M FLOP/B against the ridge 2.5 PF / 8 TB/s
    roof = None
    if lm_ms:
        gbs = alg_bytes / (lm_ms * 1e-3) / 1e9
        tfl = flops / (lm_ms * 1e-3) / 1e12
        extra = {}
        for tag in ("traffic", "mfma_util"):
            tpath = os.path.join(ROOT, "profiles", f"{tag}_{w.name}.json")
            extra[tag] = json.load(open(tpath)) if os.path.exists(tpath) else None
        roof = {"bound": "mfma" if mfma_bound else "hbm",
                "achieved": tfl if mfma_bound else gbs,
                "peak": MFMA_BF16_PEAK_TFLOPS if mfma_bound else HBM_PEAK_GBS,
                "unit": "TFLOP/s" if mfma_bound else "GB/s",
                "frac": tfl / MFMA_BF16_PEAK_TFLOPS if mfma_bound else gbs / HBM_PEAK_GBS,
                "traffic": (extra["traffic"] or {}).get("hbm_bytes_per_launch"),
                "kernel": s.lm_head_kernel_name(),
                "avg_launch_us": lm_ms * 1e3, "algorithmic_bytes_per_launch": alg_bytes,
                "hbm_gbs": gbs, "hbm_frac": gbs / HBM_PEAK_GBS,
                "mfma_tflops": tfl, "mfma_frac_by_time": tfl / MFMA_BF16_PEAK_TFLOPS,
                "mfma_counters": extra["mfma_util"],
                # the whole step against the same HBM peak: what the method must move per step
                "step_bytes_algorithmic": step_bytes,
                "step_frac": step_bytes / (T / K) / 1e9 / HBM_PEAK_GBS,
                "step_us": T / K * 1e6,
                "w_slice_cache_resident": bool(resident),
                "note": ("the W slice (%.0f MB) stays in the 256 MB memory-side cache from step to "
                         "step: bytes/time is a rate out of that cache, not an HBM figure" % (w_bytes / 1e6))
                if resident else "W is streamed from HBM every step (non-temporal loads)"}

    out = {
        "metric": "window_positions_verified_per_s",
        "value": med["verified"] / T,
        "unit": "positions/s",
        "tokens_per_s": med["tokens"] / T,
        "n_gpus": 1, "steps": K, "warmup": Wm, "repeats": R,
        "ms_per_step": T / K * 1e3,
        "ms_per_step_min": passes[order[0]]["T"] / K * 1e3,
        "ms_per_step_max": passes[order[-1]]["T"] / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} CFG={'on' if w.C == 2 else 'off'} L={w.L} "
                               f"N={w.N} V={w.V} allowed={n} d={w.d} top_k={w.top_k} top_p={w.top_p} "
                               f"lambda={w.cfg_lambda} seed={w.seed} coupling={a.coupling} sjd_mix={a.sjd_mix} "
                               f"(synthetic drift model)",
                   "decode_iterations": int(nfe) if whole else None,
                   "tokens_per_iteration": w.B * w.N / nfe if whole else None,
                   "timed": f"{R} passes of {K} steps of one decode after {Wm} warm-up steps"
                            + (" (a pass = one whole decode)" if whole and K == nfe and Wm == 0 else
                               f", {gap} untimed steps between passes (evenly spread over the decode)" if gap
                               else ", back to back"),
                   "first_step_of_each_pass": [p["first_step"] for p in passes],
                   "ms_per_step_all_passes": [p["T"] / K * 1e3 for p in passes],
                   "ms_per_step_with_events": None if T_ev is None else T_ev / K * 1e3,
                   "host_enqueue_us_per_step": med["enqueue_us"],
                   "setup_s": t_setup},
        "roofline": roof,
    }
    # flagged / adopted decisions of this workload's lock-step parity run against the CPU oracle
    # (a tracked record of the GPU tests; the bench itself compares nothing)
    fpath = os.path.join(ROOT, "profiles", "parity_flags.json")
    plain = a.coupling == "mc" and a.sjd_mix == 0.0      # the record is of the default coupling
    out["parity_flags"] = (json.load(open(fpath)).get(w.name) if plain and os.path.exists(fpath) else None)
    if a.diagnostics:       # means over the rows of the recorded decode (Sec. 3 of the paper)
        ds, hs_ = diag_sum.cpu().numpy(), hamm_sum.cpu().numpy()
        rows = max(ds[3], 1.0)
        out["diagnostics"] = {"rows": int(ds[3]), "mean_acceptance_rate_1_minus_tv": ds[0] / rows,
                              "mean_independent_collision_probability": ds[1] / rows,
                              "mean_renyi2_collision_bound": ds[2] / rows,
                              "changed_drafts": int(hs_[0]), "surviving_positions": int(hs_[1]),
                              "hamming_fraction": float(hs_[0]) / max(float(hs_[1]), 1.0),
                              "hamming_fraction_2_iterations_apart": float(hs_[2]) / max(float(hs_[3]), 1.0),
                              "hamming_fraction_3_iterations_apart": float(hs_[4]) / max(float(hs_[5]), 1.0)}
    del chunks, hs, totals, pos_after
    return out, w


if __name__ == "__main__":
    main()
