#!/usr/bin/env python3
"""Benchmark of the SCD draft-and-verify step on one MI355X.

A "step" is one whole decode iteration (scd_step: LM-head GEMM + CFG +
temperature, top-k select + softmax normaliser, vectorised MRS, first
rejection / emit / window slide) over the synthetic workload's current Jacobi
windows.  The windows' hidden states (which depend on the decode state) are
assembled for every step by an untimed recording decode, so all inputs are
resident in HBM before the timed region starts; nothing crosses PCIe inside it.

Prints ONE JSON line.  `value` = window positions verified per second over the
timed steps; `tokens_per_s` = emitted tokens per second over the same steps.
`roofline` describes the dominant kernel (the LM-head stream over W), timed with
HIP events attached to the LM-head dispatch inside scd_step (they take the kernel's own
start and stop time on the stream it runs on), in a repeat of the timed steps (a step
launched that way is about a microsecond slower, so `value`
comes from the pass without them; `config.ms_per_step_with_events` is the other).  `cpu_baseline`
is the NumPy oracle timed on the host cores on a bounded sample of the same
workload.
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
    ap.add_argument("--workload", default="C2",
                    help="C1 | C2 | C2-fullV | C3 | C4 (see paper_2510_24211_amd/workload.py)")
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
    ap.add_argument("--events-in-step", action="store_true",
                    help="record the LM-head events in the pass that gives `value` (default: in an "
                         "identical second pass, because the events slow the step down)")
    ap.add_argument("--no-full-vocab", action="store_true",
                    help="C2 only: skip the companion measurement with all 65536 ids allowed")
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
    repeated until the time is up; the last one may be cut short)."""
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
        o.step(z_rows)
        steps += 1
    T = time.perf_counter() - t0 - t_in
    positions += o.positions_verified
    tokens += int(sum(o.i))
    return {"value": positions / T, "unit": "positions/s", "cores": int(threads),
            "kind": "oracle", "tokens_per_s": float(tokens) / T,
            "sample": f"{steps} iterations of {w.name} ({decodes} whole decodes and the start of the "
                      f"next; {positions} window positions, {tokens} tokens) in {T:.1f} s, NumPy fp64"}


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

    out, w = measure(a, a.workload, inputs := {})
    if a.workload == "C2" and not a.quick and not a.no_full_vocab:
        # the same step with every one of the V = 65536 ids allowed (LM head streams all of W)
        fv, _ = measure(a, "C2-fullV", inputs)
        out["full_vocab_variant"] = {k: fv[k] for k in ("value", "unit", "tokens_per_s", "steps",
                                                         "ms_per_step", "config", "roofline")}
    inputs.clear()
    if not a.no_cpu_baseline:
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
        inputs.update(key=key, W=to_dev(wl.lm_head_weight(w)), table=to_dev(wl.HiddenTable(w).full()))
    W, table = inputs["W"], inputs["table"]
    cfg = B.config_from_workload(w)
    cfg.coupling = B.COUPLING_GS if a.coupling == "gs" else B.COUPLING_MC
    cfg.sjd_mix = a.sjd_mix
    cfg.diagnostics = int(a.diagnostics)
    s = B.Scd(cfg, dev)
    st = s.alloc_state()
    h = torch.empty((w.B, w.C, w.L, w.d), dtype=torch.bfloat16, device=dev)
    t_setup = time.perf_counter() - t_setup

    # ---- recording pass (untimed; also the warm-up) ------------------------------------
    # The hidden states of a step depend on the decode state (window start and ages), which
    # lives on the device.  One untimed decode assembles every step's [B, C, L, d] input with
    # the device-side gather and keeps it, so that the timed steps below find their inputs
    # resident in HBM and consist of scd_step alone.  The trajectory is deterministic (same
    # seed, same kernels), which the token comparison after the timed pass confirms.
    CH = 64
    chunks = []

    def h_of(i):
        while i // CH >= len(chunks):
            chunks.append(torch.empty((CH, w.B, w.C, w.L, w.d), dtype=torch.bfloat16, device=dev))
        return chunks[i // CH][i % CH]

    diag_sum = torch.zeros(4, dtype=torch.float64, device=dev)     # beta, C, bound, live rows
    hamm_sum = torch.zeros(6, dtype=torch.int64, device=dev)       # (differing, compared) for 1, 2, 3 iterations apart

    def record(limit):
        """Decode from a fresh state, at most `limit` steps; returns the iteration count."""
        s.reset(st)
        i = 0
        while i < limit:
            for _ in range(min(16, limit - i)):
                hi = h_of(i)
                s.gather_hidden(table, w.age_cap, st, hi)
                s.step(hi, W, st)
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

    if a.quick:
        assert a.steps > 0 and a.warmup > 0, "--quick needs --steps and --warmup"
        nfe = record(a.steps + a.warmup)          # the decode may end earlier: then steps wrap
        verified_per_decode = int(s.state_field(st, B.F_VERIFIED).sum().item())
    else:
        nfe = record(1 << 30)                     # whole decode
        verified_per_decode = int(s.state_field(st, B.F_VERIFIED).sum().item())
    tokens_ref = s.state_field(st, B.F_OUT).clone()
    K = a.steps if a.steps > 0 else nfe
    Wm = a.warmup
    first = 0                                     # recorded step the timed pass starts at
    s.reset(st)
    if Wm > 0:
        for i in range(Wm):
            if first == nfe:
                s.reset(st)
                first = 0
            s.step(h_of(first), W, st)
            first += 1
        if not a.quick:                           # default: the timed pass starts a fresh decode
            s.reset(st)
            first = 0

    use_events = not a.no_events
    ev = HipEvents(K) if use_events else None
    enqueue_us = []                               # host time per step to enqueue (first pass = value's)

    hs = [h_of(i) for i in range(nfe)]            # views, made outside the timed loops

    def timed_pass(with_events):
        v0 = int(s.state_field(st, B.F_VERIFIED).sum().item())   # non-zero only after --quick warm-up
        p0 = int(s.state_field(st, B.F_POS).sum().item())
        torch.cuda.synchronize()
        done_decodes, in_decode = 0, first
        t0 = time.perf_counter()
        for i in range(K):
            if in_decode == nfe:                  # sequence(s) finished: start the next decode
                s.reset(st)
                done_decodes, in_decode = done_decodes + 1, 0
            if with_events:
                s.set_lm_head_events(*ev.pair(i))
            s.step(hs[in_decode], W, st)
            in_decode += 1
        t_enq = time.perf_counter() - t0
        torch.cuda.synchronize()
        T = time.perf_counter() - t0
        enqueue_us.append(t_enq / K * 1e6)
        if with_events:
            s.set_lm_head_events(None, None)
        verified = done_decodes * verified_per_decode - v0 + int(s.state_field(st, B.F_VERIFIED).sum().item())
        tokens = done_decodes * w.B * w.N - p0 + int(s.state_field(st, B.F_POS).sum().item())
        if in_decode == nfe and not a.quick:      # ended on a whole decode: same tokens as recorded
            assert torch.equal(s.state_field(st, B.F_OUT), tokens_ref), "decode is not reproducible"
        return T, verified, tokens

    # A step whose LM head carries the events is about a microsecond slower (the dispatch then
    # reports its timestamps; recorded event PAIRS cost 2-6 us: two more packets between the
    # kernels), so the throughput comes from a pass without them and the LM-head timing from
    # an identical pass with them, right after (--events-in-step: one pass for both).
    T_ev = None
    if use_events and not a.events_in_step:
        T, verified, tokens = timed_pass(False)
        if a.quick:                               # the second pass repeats the same steps
            s.reset(st)
            redo = 0
            for i in range(Wm):
                if redo == nfe:
                    s.reset(st)
                    redo = 0
                s.step(h_of(redo), W, st)
                redo += 1
        else:
            s.reset(st)
        T_ev, _, _ = timed_pass(True)
    else:
        T, verified, tokens = timed_pass(use_events)
        T_ev = T if use_events else None
    rc, flags = s.status(st)
    assert rc == B.SCD_OK

    lm_ms = None
    if use_events:
        lm_ms = float(np.mean([ev.elapsed_ms(i) for i in range(K)]))
        ev.destroy()

    n = w.n_allowed
    w_bytes = 2 * w.d * n
    h_bytes = 2 * w.M * w.d
    alg_bytes = w_bytes + h_bytes               # per LM-head launch (W slice once + hidden rows)
    flops = 2.0 * w.M * w.d * n
    roof = None
    if lm_ms:
        gbs = alg_bytes / (lm_ms * 1e-3) / 1e9
        traffic = None
        tpath = os.path.join(ROOT, "profiles", f"traffic_{w.name}.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
        roof = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "traffic": traffic, "kernel": s.lm_head_kernel_name(),
                "avg_launch_us": lm_ms * 1e3, "algorithmic_bytes_per_launch": alg_bytes,
                "mfma_tflops": flops / (lm_ms * 1e-3) / 1e12,
                "mfma_frac": flops / (lm_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}

    out = {
        "metric": "window_positions_verified_per_s",
        "value": verified / T,
        "unit": "positions/s",
        "tokens_per_s": tokens / T,
        "n_gpus": 1, "steps": K, "warmup": Wm if Wm > 0 else nfe,
        "ms_per_step": T / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} CFG={'on' if w.C == 2 else 'off'} L={w.L} "
                               f"N={w.N} V={w.V} allowed={n} d={w.d} top_k={w.top_k} top_p={w.top_p} "
                               f"lambda={w.cfg_lambda} seed={w.seed} coupling={a.coupling} sjd_mix={a.sjd_mix} "
                               f"(synthetic drift model)",
                   "decode_iterations": None if a.quick else int(nfe),
                   "tokens_per_iteration": None if a.quick else w.B * w.N / nfe,
                   "step_bytes_algorithmic": alg_bytes + 2 * w.B * w.L * min(n, w.top_k or n) * 8,
                   "step_hbm_frac": (alg_bytes + 2 * w.B * w.L * min(n, w.top_k or n) * 8)
                   / (T / K) / 1e9 / HBM_PEAK_GBS,
                   "lm_head_events": ("none" if not use_events else "same pass as value"
                                      if a.events_in_step else "repeat of the timed steps"),
                   "ms_per_step_with_events": None if T_ev is None else T_ev / K * 1e3,
                   "host_enqueue_us_per_step": enqueue_us[0],
                   "setup_s": t_setup},
        "roofline": roof,
    }
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
    return out, w


if __name__ == "__main__":
    main()
