"""GPU parity tests: the HIP path, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Stage tests first (LM head, select/softmax,
MRS, verify), then lock-step decodes of the five workloads (small ones whole,
large ones a prefix of iterations in the benchmark's launch configuration),
then edge cases."""
import numpy as np
import pytest
import torch

from oracle import logits as lg
from oracle import mrs as omrs
from oracle import philox
from paper_2510_24211_amd import binding as B
from paper_2510_24211_amd import workload as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bf16(bits):
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


@pytest.fixture(scope="module", autouse=True)
def _require_gpu_and_library():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.load()


# ---------------------------------------------------------------- LM head
@pytest.mark.parametrize("Bn,L,d,V,v_lo,v_hi,lam,tau", [
    (1, 32, 256, 1024, 0, 1024, 0.0, 1.0),      # one tile column set, no CFG
    (1, 32, 1280, 2000, 0, 2000, 0.0, 1.0),     # ragged vocabulary tail (2000 = 15*128 + 80)
    (1, 32, 512, 4096, 4, 1300, 3.0, 1.0),      # CFG + unaligned id range
    (2, 64, 520, 777, 0, 777, 3.0, 0.7),        # d not a multiple of the k tile, tau != 1
    (3, 8, 64, 300, 10, 290, 3.0, 1.0),         # window shorter than a row block
    (5, 40, 128, 640, 0, 640, 1.5, 1.0),        # L not a multiple of 32, odd B
    (1, 1, 64, 256, 0, 256, 0.0, 1.0),          # L = 1
    (16, 32, 256, 512, 0, 512, 3.0, 1.0),       # several row-block tiles share a W slab
    # split-k kernel with XCD-affine row groups of G = 128 KB / row bytes rows, ragged against 8 G,
    # first allowed row not on a block boundary:
    (1, 32, 2048, 4096, 3, 4000, 3.0, 1.0),     # G = 32, 4 k parts
    (1, 32, 1024, 3000, 0, 3000, 0.0, 1.0),     # G = 64
    (1, 32, 8192, 1500, 5, 1400, 3.0, 1.0),     # G = 8, 8 k parts
    (2, 32, 4096, 2500, 7, 2407, 3.0, 1.0),     # G = 16, two row blocks per workgroup
    (4, 32, 4096, 1000, 0, 1000, 3.0, 1.0),     # G = 16 available but many row blocks: wide kernel
    # exactly 4 (or 3) row blocks and a wide vocabulary: the all-rows-in-one-workgroup kernel
    (2, 64, 256, 52000, 0, 52000, 3.0, 1.0),
    (1, 100, 192, 51300, 5, 51290, 3.0, 1.0),   # ragged n, ragged L, odd number of k tiles
    (3, 20, 136, 51210, 0, 51210, 0.0, 0.9),    # 3 row blocks, no CFG, d not a multiple of the k tile
    (2, 64, 128, 51200, 0, 51200, 3.0, 1.0),    # its shortest k loop: 2 tiles
])
def test_lm_head_against_oracle(Bn, L, d, V, v_lo, v_hi, lam, tau):
    g = np.random.default_rng(hash((Bn, L, d, V)) % 2 ** 32)
    C = 2 if lam else 1
    h = wl.f32_to_bf16_bits(g.standard_normal((Bn, C, L, d)).astype(np.float32))
    W = wl.f32_to_bf16_bits((g.standard_normal((V, d)) * 0.05).astype(np.float32))
    cfg = B.make_config(B=Bn, L=L, N=10 * L, V=V, d=d, v_lo=v_lo, v_hi=v_hi, cfg_lambda=lam,
                        temperature=tau)
    s = B.Scd(cfg, DEV)
    n = v_hi - v_lo
    z = torch.full((Bn, L, n), float("nan"), device=DEV)
    s.lm_head(_bf16(h), _bf16(W), z)
    torch.cuda.synchronize()
    zg = z.cpu().numpy()
    W64 = lg.bf16_bits_to_f64(W[v_lo:v_hi])
    for b in range(Bn):
        c = lg.lm_head(h[b, 0], W64)
        u = lg.lm_head(h[b, 1], W64) if C == 2 else None
        zo = lg.process_logits(c, u, lam, tau)
        diff = np.abs(zg[b].astype(np.float64) - zo)
        scale = np.maximum(np.abs(zo), np.sqrt(np.mean(zo.astype(np.float64) ** 2)))
        assert (diff / scale).max() <= 2e-3          # the stated bf16-GEMM bar
        assert diff.max() <= 2e-5 * (1 + 2 * lam) * max(1.0, np.abs(zo).max())   # what fp32 accumulation gives


# ------------------------------------------------------- select / softmax
def _select_case(z, top_k, top_p=0.0):
    rows, n = z.shape
    cfg = B.make_config(B=1, L=1, N=1, V=n, top_k=top_k, top_p=top_p)
    s = B.Scd(cfg, DEV)
    thr = torch.empty(rows, device=DEV)
    lse = torch.empty(rows, device=DEV)
    nk = torch.empty(rows, dtype=torch.int32, device=DEV)
    s.select(torch.from_numpy(z).to(DEV), rows, thr, lse, nk)
    torch.cuda.synchronize()
    thr, lse, nk = thr.cpu().numpy(), lse.cpu().numpy(), nk.cpu().numpy()
    adopted = 0
    for r in range(rows):
        p, thr_o, lse_o = lg.distribution(z[r], top_k, top_p)
        if top_p and thr[r] != thr_o:
            # the nucleus boundary is a comparison of fp sums: within 2e-6 of the target mass
            # either side is right, and the GPU's threshold must be a logit of the row there
            keep_k = z[r] >= lg.topk_threshold(z[r], top_k)
            t_in = lg.nucleus_threshold(z[r], keep_k, top_p - 2e-6)
            t_out = lg.nucleus_threshold(z[r], keep_k, top_p + 2e-6)
            assert t_out <= thr[r] <= t_in and (z[r] == thr[r]).any(), (r, thr[r], thr_o, t_out, t_in)
            thr_o = thr[r]
            p, lse_o = lg.softmax_kept(z[r], thr_o)
            adopted += 1
        assert thr[r] == thr_o, (r, thr[r], thr_o)                   # exact order statistic
        assert nk[r] == int((p > 0).sum()) or nk[r] == int((z[r] >= thr_o).sum())
        assert abs(float(lse[r]) - lse_o) <= 1e-6 * max(1.0, abs(lse_o))
        # probabilities of the kept ids from the GPU's (thr, lse) against the oracle's softmax
        keep = z[r] >= thr[r]
        pg = np.where(keep, np.exp(z[r].astype(np.float64) - float(lse[r])), 0.0)
        assert np.abs(pg - p).max() <= 1e-6
    return adopted


@pytest.mark.parametrize("n,top_k", [(1024, 0), (1024, 100), (1000, 1), (1000, 999), (1000, 1000),
                                     (1000, 5000), (8192, 2000), (65536, 2000), (16384, 1000),
                                     (64000, 2000), (5, 2), (1, 1), (4097, 33),
                                     (40000, 3500), (65536, 10000), (20000, 19999), (30001, 7),
                                     # rows longer than the fused kernel takes: the per-stage kernels
                                     (65537, 2000), (70000, 500), (131072, 2000), (100003, 0),
                                     (131072, 131071)])
def test_select_softmax_against_oracle(n, top_k):
    g = np.random.default_rng(n * 31 + top_k)
    z = (g.standard_normal((6, n)) * 3).astype(np.float32)
    if n >= 1000:
        z[1, g.integers(0, n, 50)] = -np.inf          # masked-out ids inside the row
        z[2] = np.round(z[2] * 4) / 4                 # heavy ties, also at the threshold
        z[3] = -np.abs(z[3]) - 100                    # all negative, large magnitude
        z[4, :] = z[4, 0]                             # constant row
    _select_case(z, top_k)


@pytest.mark.parametrize("rows,n,top_k", [(300, 8192, 2000), (257, 3001, 100), (700, 640, 0),
                                          (520, 4097, 4000), (300, 8193, 2000)])
def test_select_on_more_rows_than_compute_units(rows, n, top_k):
    # more than 256 rows of at most 8192 ids run the 512-thread build of the row kernel, two
    # workgroups per compute unit (8 or 16 logits per thread); 8193 ids: the 1024-thread one
    g = np.random.default_rng(rows * 7 + n)
    z = (g.standard_normal((rows, n)) * 3).astype(np.float32)
    z[1, g.integers(0, n, 20)] = -np.inf
    z[2] = np.round(z[2] * 4) / 4
    z[3] = -np.abs(z[3]) - 100
    z[4, :] = z[4, 0]
    z[rows - 1] = np.round(z[rows - 1])                # ties in the last row too
    _select_case(z, top_k)


def test_select_nucleus_on_more_rows_than_compute_units():
    # the nucleus instances keep 1024 threads per row whatever the number of rows
    g = np.random.default_rng(4242)
    z = (g.standard_normal((300, 3000)) * 3).astype(np.float32)
    z[2] = np.round(z[2] * 4) / 4
    z[4, :] = z[4, 0]
    assert _select_case(z, 500, 0.8) <= 2


@pytest.mark.parametrize("n,top_k,top_p", [(1024, 0, 0.8), (1000, 100, 0.8), (1000, 0, 0.02), (1000, 0, 0.9999),
                                           (8192, 2000, 0.8), (16384, 0, 0.8), (12000, 3000, 0.95),
                                           (64000, 0, 0.8), (65536, 2000, 0.5), (40000, 0, 0.3),
                                           (5, 0, 0.7), (2, 0, 0.5), (1, 0, 0.8), (4097, 33, 0.6),
                                           (40000, 5000, 0.9), (65536, 12000, 0.97), (30001, 0, 0.6)])
def test_select_nucleus_against_oracle(n, top_k, top_p):
    g = np.random.default_rng(n * 37 + top_k)
    z = (g.standard_normal((7, n)) * 3).astype(np.float32)
    if n >= 1000:
        z[1, g.integers(0, n, 50)] = -np.inf          # masked-out ids inside the row
        z[2] = np.round(z[2] * 4) / 4                 # heavy ties, also at the boundary
        z[3] = -np.abs(z[3]) - 100                    # all negative, large magnitude
        z[4, :] = z[4, 0]                             # constant row: every id tied, all kept
        z[5] = z[5] * 2                               # peaked: the nucleus is a handful of ids
        z[6] = z[6] * 0.05                            # flat: the nucleus is most of the row
    adopted = _select_case(z, top_k, top_p)
    assert adopted <= 2                               # boundary cases are rare


# ------------------------------------------------------------- MRS stage
@pytest.mark.parametrize("Bn,L,n,top_k,N,pos0,top_p", [
    (1, 8, 1024, 0, 64, [0], 0.0),
    (2, 16, 1000, 100, 40, [3, 30], 0.0),      # ragged n (scalar loads), second window clipped to 10 rows
    (1, 32, 8192, 2000, 2304, [100], 0.0),
    (3, 5, 37, 7, 50, [0, 45, 49], 0.0),       # tiny vocabulary, windows of 5 / 5 / 1 rows
    (2, 16, 4096, 500, 100, [0, 90], 0.7),     # nucleus filter after top-k
    (1, 24, 20000, 0, 64, [5], 0.9),           # nucleus filter alone on a long row (in-place path)
    # rows longer than 65536 ids: select_kernel -> mrs_kernel -> commit_kernel
    (2, 6, 70000, 500, 40, [0, 37], 0.0),      # second window clipped to 3 rows
    (1, 5, 131072, 2000, 64, [9], 0.0),
    (1, 4, 100003, 0, 64, [62], 0.0),          # no filter, ragged n, window clipped to 2 rows
    # more window rows than compute units: the two-workgroups-per-CU build of the row kernel
    (10, 32, 2048, 200, 400, [0, 37, 74, 111, 148, 185, 222, 259, 296, 390], 0.0),
    (33, 8, 5000, 0, 64, list(range(32)) + [60], 0.0),   # last window clipped to 4 rows
])
def test_couple_draft_and_verify_against_oracle(Bn, L, n, top_k, N, pos0, top_p):
    g = np.random.default_rng(n + L)
    seed, it = 0xABCDEF0123456789, 7
    base = (g.standard_normal((Bn, L, n)) * 2).astype(np.float32)
    scale = np.float32(0.5) ** g.integers(0, 12, (Bn, L, 1)).astype(np.float32)
    z_prev = base
    z_cur = (base + scale * g.standard_normal((Bn, L, n)).astype(np.float32)).astype(np.float32)
    z_cur[:, -1] = z_prev[:, -1]                         # identical rows: must accept
    fresh = (g.random((Bn, L)) < 0.25).astype(np.uint8)
    fresh[:, -1] = 0
    # drafts: x ~ q
    x = np.zeros((Bn, L), dtype=np.int32)
    for b in range(Bn):
        for s in range(L):
            if fresh[b, s]:
                x[b, s] = g.integers(0, n)
            else:
                q, _, _ = lg.distribution(z_prev[b, s], top_k, top_p)
                x[b, s] = g.choice(n, p=q)
    cfg = B.make_config(B=Bn, L=L, N=N, V=n, top_k=top_k, top_p=top_p, seed=seed)
    sc = B.Scd(cfg, DEV)
    t = lambda a: torch.from_numpy(a).to(DEV)
    y = torch.empty((Bn, L), dtype=torch.int32, device=DEV)
    k = torch.empty((Bn, L), dtype=torch.uint8, device=DEV)
    pos_t = t(np.array(pos0, dtype=np.int32))
    sc.couple_draft(t(z_cur), t(z_prev), t(x), t(fresh), pos_t, it, y, k)
    acc = torch.empty(Bn, dtype=torch.int32, device=DEV)
    out = torch.full((Bn, N), -7, dtype=torch.int32, device=DEV)
    sc.verify(k, y, pos_t, acc, out)
    torch.cuda.synchronize()
    y, k, acc, out = y.cpu().numpy(), k.cpu().numpy(), acc.cpu().numpy(), out.cpu().numpy()
    n_rej = 0
    for b in range(Bn):
        live = min(L, N - pos0[b])
        first = live
        for s in range(L):
            if s >= live:
                assert y[b, s] == -1 and k[b, s] == 1
                continue
            j = pos0[b] + s
            p, _, _ = lg.distribution(z_cur[b, s], top_k, top_p)
            q = np.full(n, np.float64(np.float32(1.0) / np.float32(n))) if fresh[b, s] \
                else lg.distribution(z_prev[b, s], top_k, top_p)[0]
            u = philox.uniform_scalar(seed, b, j, it, philox.STREAM_ACCEPT)
            r = omrs.mrs(p, q, int(x[b, s]), u,
                         lambda: philox.uniform_per_vocab(seed, b, j, it, philox.STREAM_RESID, n))
            if k[b, s] != r["k"]:
                assert r["flag_accept"], (b, s)
            elif r["k"] == 0 and y[b, s] != r["y"]:
                assert r["flag_resid"], (b, s)
            else:
                assert y[b, s] == r["y"]
            n_rej += 1 - int(k[b, s])
            if k[b, s] == 0 and first == live:
                first = s
        a = min(first + 1, live)
        assert acc[b] == a
        assert np.array_equal(out[b, pos0[b]:pos0[b] + a], y[b, :a])       # v_lo = 0
        assert (out[b, :pos0[b]] == -7).all() and (out[b, pos0[b] + a:] == -7).all()
    assert (k[:, -1] == 1).all() or any(min(L, N - p) < L for p in pos0)    # identical rows accepted
    assert n_rej > 0                                                         # the race was exercised


# ------------------------------------------------------ lock-step decodes
def _lockstep(w, max_steps=None, **kw):
    import json, os
    from lockstep import LockStep
    ls = LockStep(w, DEV, **kw)
    st = ls.run(max_steps)
    print(f"\n[{w.name}] {st}")
    # flagged draws are rare; adopted ones rarer
    assert st["adopt_accept"] + st["adopt_resid"] <= max(3, 1e-3 * st["draws"])
    assert st["adopt_topk"] <= max(3, 1e-2 * st["draws"])
    # the counts the parity statement rests on, one line per lock-step run
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
    with open(os.path.join(root, "gpurun_out", "parity_flags.jsonl"), "a") as f:
        f.write(json.dumps(dict(workload=w.name, B=w.B, L=w.L, N=w.N, n=w.n_allowed, d=w.d, top_k=w.top_k,
                                top_p=w.top_p, options={k: v for k, v in kw.items()},
                                whole_decode=bool(ls.oracle.done()), **st)) + "\n")
    return ls, st


def test_lockstep_C0_full_and_golden():
    import json, os
    ls, st = _lockstep(wl.WORKLOADS["C0"])
    want = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "c0_golden.json")))
    assert [int(x) for x in ls.oracle.out[0]] == want["tokens"]
    assert ls.oracle.t[0] == want["nfe"] and ls.oracle.accept_hist[0] == want["accept_len"]
    assert st["adopt_accept"] == st["adopt_resid"] == st["adopt_topk"] == 0


@pytest.mark.parametrize("kw", [
    dict(N=40, L=8, seed=11),
    dict(N=33, L=1, seed=12),                       # plain autoregressive sampling
    dict(N=5, L=8, seed=13),                        # sequence shorter than the window
    dict(N=50, L=16, seed=14, top_k=64),
    dict(N=70, L=8, seed=15, B=3, V=1000),          # batch, ragged n
    dict(N=64, L=64, seed=16, top_k=10, V=300),
    dict(N=300, L=128, seed=17, V=512),             # window longer than a wavefront
    dict(N=12, L=4, seed=18, V=70000, top_k=500, age_cap=4),   # rows too long for the LDS-resident kernel
    dict(N=20, L=4, seed=19, V=65536, top_k=2000, age_cap=4),  # longest row of the LDS-resident kernel
    dict(N=600, L=256, seed=20, V=256, age_cap=6),             # the longest window the library takes
    dict(N=40, L=8, seed=28, V=777, top_k=5000),               # top_k above the vocabulary: no filter
    dict(N=30, L=8, seed=29, V=2, B=2),                        # two-id vocabulary
])
def test_lockstep_toy_variants(kw):
    _lockstep(wl.scaled(wl.WORKLOADS["C0"], name="toy", **kw))


@pytest.mark.parametrize("kw", [
    dict(name="C1s", N=96, V=2048, d=256, top_k=200),
    dict(name="C1r", N=50, V=1000, d=72, top_k=100, L=8, B=2),      # ragged everything
])
def test_lockstep_scaled_lm_head(kw):
    _lockstep(wl.scaled(wl.WORKLOADS["C1"], **kw))


def test_lockstep_scaled_cfg_masked_batched():
    # C3-like: CFG, unaligned allowed range, 4 sequences that finish at different iterations
    _lockstep(wl.scaled(wl.WORKLOADS["C3"], name="C3s", B=4, N=80, V=4096, d=256, v_lo=4, v_hi=1028,
                        top_k=250))


def test_lockstep_scaled_cfg_temperature():
    _lockstep(wl.scaled(wl.WORKLOADS["C2"], name="C2t", N=64, V=4096, d=320, v_lo=100, v_hi=3000,
                        top_k=300, temperature=0.8))


@pytest.mark.parametrize("kw", [
    dict(N=40, L=8, seed=30, V=1000, top_p=0.8),                   # 8 logits per thread, no top-k
    dict(N=40, L=8, seed=31, V=12000, top_k=3000, top_p=0.9, age_cap=4),   # 16 per thread, after top-k
    dict(N=12, L=4, seed=32, V=65536, top_p=0.8, age_cap=4),       # in-place path
    dict(N=12, L=4, seed=33, V=40000, top_k=2000, top_p=0.5, age_cap=4),   # slice kernel + candidates
    dict(N=30, L=8, seed=34, V=2000, top_p=0.999),                 # nearly everything kept
    dict(N=30, L=8, seed=35, V=2000, top_p=0.001, B=2),            # the mode alone
])
def test_lockstep_nucleus_toy_variants(kw):
    _lockstep(wl.scaled(wl.WORKLOADS["C0"], name="toy", **kw))


def test_lockstep_nucleus_scaled_and_video_prefix():
    _lockstep(wl.scaled(wl.WORKLOADS["C4-topp"], name="C4ps", N=8 * 24, V=2000, d=512, L=64))
    _lockstep(wl.scaled(wl.WORKLOADS["C2"], name="C2p", N=64, V=4096, d=320, v_lo=100, v_hi=3000,
                        top_k=300, top_p=0.8), coupling="gs")
    _lockstep(wl.WORKLOADS["C4-topp"], max_steps=3)


@pytest.mark.parametrize("kw,opts", [
    (dict(N=64, L=8, seed=0), dict()),                                     # 8 logits per thread
    (dict(N=70, L=8, seed=36, B=3, V=1000, top_k=100), dict(coupling="gs")),   # batch, ragged n, pi_GS
    (dict(N=40, L=8, seed=37, V=12000, top_k=300, age_cap=4), dict(sjd_mix=0.5)),   # 16 per thread, alpha = 0.5
    (dict(N=16, L=4, seed=38, V=20000, age_cap=4), dict()),                # in-place path
    (dict(N=16, L=4, seed=39, V=40000, top_k=2000, age_cap=4), dict()),    # slice kernel + candidates
    (dict(N=40, L=8, seed=40, V=3000, top_p=0.8), dict()),                 # with the nucleus filter
    (dict(N=300, L=128, seed=41, V=512), dict()),                          # window longer than a wavefront
    (dict(N=70, L=8, seed=42, B=3, V=1000), dict(sjd_mix=1.0)),            # vanilla SJD, ragged finish
    (dict(N=600, L=256, seed=44, V=256, age_cap=6), dict()),               # the longest window
])
def test_lockstep_statistics_toy_variants(kw, opts):
    ls, st = _lockstep(wl.scaled(wl.WORKLOADS["C0"], name="toy", **kw), diagnostics=True, **opts)
    assert st["max_stat_rel"] < 2e-5


def test_lockstep_every_option_combined():
    # top-k, nucleus, Gumbel sharing, the alpha switch and the statistics in one decode
    _lockstep(wl.scaled(wl.WORKLOADS["C0"], name="toy", N=80, L=16, seed=45, V=5000, top_k=800, top_p=0.85, B=2),
              coupling="gs", sjd_mix=0.3, diagnostics=True)
    _lockstep(wl.scaled(wl.WORKLOADS["C2"], name="C2o", N=64, V=4096, d=320, v_lo=100, v_hi=3000, top_k=300,
                        top_p=0.9), coupling="gs", sjd_mix=0.5, diagnostics=True)


def test_lockstep_statistics_scaled_and_C2_prefix():
    _lockstep(wl.scaled(wl.WORKLOADS["C3"], name="C3s", B=4, N=80, V=4096, d=256, v_lo=4, v_hi=1028,
                        top_k=250), diagnostics=True)
    _lockstep(wl.WORKLOADS["C2"], max_steps=10, diagnostics=True)


def test_lockstep_nucleus_after_topk_C2_full():
    # the benchmark's shape with the nucleus filter on top of top-k, the whole decode: holds rows
    # whose boundary falls on an exact tie of two logits that the GPU's GEMM rounding splits
    ls, st = _lockstep(wl.scaled(wl.WORKLOADS["C2"], name="C2p", top_p=0.8))
    assert ls.oracle.done()


def test_lockstep_scaled_video():
    _lockstep(wl.scaled(wl.WORKLOADS["C4"], name="C4s", N=8 * 24, V=2000, d=512, top_k=300, L=64))


def test_lockstep_C1_full():
    _lockstep(wl.WORKLOADS["C1"])


def test_lockstep_C2_full():
    # the benchmark's workload, the whole decode (404 iterations, 12863 rows)
    ls, st = _lockstep(wl.WORKLOADS["C2"])
    assert ls.oracle.done() and st["steps"] == 404


def test_lockstep_C2_prefix_with_logits():
    _lockstep(wl.WORKLOADS["C2"], max_steps=12)


def test_lockstep_C2_fullV_full():
    # the full-vocabulary variant of the benchmark's workload: logits checked on a prefix, then
    # the whole decode (415 iterations, 13210 rows; the W stream uses the non-temporal loads)
    _lockstep(wl.WORKLOADS["C2-fullV"], max_steps=5)
    ls, st = _lockstep(wl.WORKLOADS["C2-fullV"])
    assert ls.oracle.done() and st["steps"] == 415


# ------------------- first half of the top-k selection inside the LM head's epilogue (wide vocabularies)
@pytest.mark.parametrize("kw", [
    dict(name="fvs", N=96, V=52000, d=128, top_k=2000, v_lo=0, v_hi=52000),              # 204 column tiles of 256
    dict(name="fvr", N=70, L=20, V=60000, d=136, top_k=1500, v_lo=5, v_hi=51290),         # ragged ids, window, k
    dict(name="fvg", N=200, L=64, B=2, V=52000, d=128, top_k=2000, v_lo=0, v_hi=52000),   # all rows in one workgroup
    dict(name="fv3", N=60, L=20, B=3, V=51210, d=192, top_k=1800, v_lo=0, v_hi=51210),    # 3 row blocks, ragged tile
])
def test_lockstep_epilogue_candidates_scaled(kw):
    _lockstep(wl.scaled(wl.WORKLOADS["C2"], **kw))


def test_lockstep_epilogue_candidates_with_ties_that_overflow_a_tile():
    # 40 identical weight rows inside one 256-column tile, with a large norm: in about half of the
    # window rows their (identical) logits are the row's largest, more than a tile's list holds;
    # those rows must fall back to reading the whole row.  300 more identical rows spread over the
    # vocabulary tie at the top-k boundary region without overflowing any list.
    import lockstep
    w = wl.scaled(wl.WORKLOADS["C2"], name="fvt", N=64, V=52000, d=128, top_k=2000, v_lo=0, v_hi=52000, seed=77)
    W = wl.lm_head_weight(w)
    g = np.random.default_rng(5)
    hot = wl.f32_to_bf16_bits((g.standard_normal(w.d) * 0.1).astype(np.float32))
    W[1000:1040] = hot                                   # one tile (columns 768..1023 + 1024..1279: rows 1000-1023 / 1024-1039)
    W[3100:3140] = hot                                   # inside one tile (3072..3327)
    warm = wl.f32_to_bf16_bits((g.standard_normal(w.d) * 0.03).astype(np.float32))
    W[np.arange(300) * 170 + 7] = warm
    key = (w.seed, w.V, w.d, w.w_std, w.v_lo, w.v_hi, str(DEV))
    lockstep._W_CACHE.clear()
    lockstep._W_CACHE[key] = (_bf16(W), lg.bf16_bits_to_f64(W[w.v_lo:w.v_hi]))
    try:
        ls, st = _lockstep(w)
    finally:
        lockstep._W_CACHE.clear()
    assert ls.oracle.done()


# ----------------------------------------- Gumbel-sharing coupling (pi_GS)
@pytest.mark.parametrize("kw", [
    dict(N=64, L=8, seed=0),                        # the toy workload itself
    dict(N=33, L=1, seed=22),                       # plain autoregressive sampling
    dict(N=50, L=16, seed=23, top_k=64),
    dict(N=70, L=8, seed=24, B=3, V=1000),          # batch, ragged n
    dict(N=40, L=8, seed=25, V=12000, top_k=300, age_cap=4),   # 16 logits per thread
    dict(N=20, L=4, seed=26, V=65536, top_k=2000, age_cap=4),  # slice kernel + candidate path
    dict(N=16, L=4, seed=27, V=20000, age_cap=4),              # no top-k on a long row: in-place path
])
def test_lockstep_gs_toy_variants(kw):
    ls, st = _lockstep(wl.scaled(wl.WORKLOADS["C0"], name="toy-gs", **kw), coupling="gs")
    assert st["adopt_gs"] <= max(2, 1e-3 * st["draws"])


def test_lockstep_gs_scaled_cfg_masked_batched():
    ls, st = _lockstep(wl.scaled(wl.WORKLOADS["C3"], name="C3s-gs", B=4, N=80, V=4096, d=256, v_lo=4,
                                 v_hi=1028, top_k=250), coupling="gs")
    assert st["adopt_gs"] <= max(2, 1e-3 * st["draws"])


def test_lockstep_on_more_rows_than_compute_units():
    # 9 x 32 = 288 window rows of 1024 ids: the 512-thread build of the row kernel, under the
    # maximal coupling, under Gumbel sharing and under the alpha-coupling (its two hot instances)
    kw = dict(B=9, N=72, V=4096, d=128, v_lo=4, v_hi=1028, top_k=250)
    _lockstep(wl.scaled(wl.WORKLOADS["C3"], name="C3b", **kw))
    ls, st = _lockstep(wl.scaled(wl.WORKLOADS["C3"], name="C3b-gs", **kw), coupling="gs")
    assert st["adopt_gs"] <= max(2, 1e-3 * st["draws"])
    _lockstep(wl.scaled(wl.WORKLOADS["C3"], name="C3b-alpha", **kw), coupling="mc", sjd_mix=0.5)


def test_lockstep_gs_C1_full_and_C2_prefix():
    _lockstep(wl.WORKLOADS["C1"], coupling="gs")
    _lockstep(wl.WORKLOADS["C2"], max_steps=25, coupling="gs")


@pytest.mark.parametrize("coupling,sjd_mix,kw", [
    ("mc", 1.0, dict(N=64, L=8, seed=0)),                      # vanilla SJD: every redraft independent
    ("mc", 0.5, dict(N=50, L=16, seed=33, top_k=64)),
    ("gs", 0.25, dict(N=70, L=8, seed=34, B=3, V=1000)),
    ("mc", 0.7, dict(N=20, L=4, seed=35, V=65536, top_k=2000, age_cap=4)),   # candidate path
])
def test_lockstep_alpha_coupling_toy_variants(coupling, sjd_mix, kw):
    ls, st = _lockstep(wl.scaled(wl.WORKLOADS["C0"], name="toy-alpha", **kw), coupling=coupling,
                       sjd_mix=sjd_mix)
    assert st["adopt_gs"] <= max(2, 1e-3 * st["draws"])


def test_lockstep_alpha_coupling_C2_prefix():
    _lockstep(wl.WORKLOADS["C2"], max_steps=20, coupling="mc", sjd_mix=0.5)


def test_gs_redraft_is_stable_where_mc_is_not_required_to_be():
    # p == q bit for bit (ages past the cap): the Gumbel draft of a position repeats exactly,
    # iteration after iteration, because its noise does not depend on the iteration.
    from lockstep import LockStep
    w = wl.scaled(wl.WORKLOADS["C0"], name="toy-gs-const", N=24, L=8, seed=31, age_cap=0)
    ls = LockStep(w, DEV, coupling="gs")
    ls.step()                                   # every window position evaluated once
    X1 = ls.v["X"].cpu().numpy().copy()
    pos1 = int(ls.v["pos"].cpu().numpy()[0])
    ls.step()
    X2 = ls.v["X"].cpu().numpy()
    pos2 = int(ls.v["pos"].cpu().numpy()[0])
    for j in range(pos2, min(pos1 + w.L, w.N)):  # positions that were in both windows and survive
        assert X1[j % w.L] == X2[j % w.L]


# --------------------------------------------------------------- edge cases
def test_determinism_and_finished_sequences_untouched():
    w = wl.scaled(wl.WORKLOADS["C1"], name="det", N=64, V=1024, d=128, top_k=100, B=2)
    cfg = B.config_from_workload(w)
    W = _bf16(wl.lm_head_weight(w))
    tab = wl.HiddenTable(w)
    table = _bf16(tab.full())
    outs = []
    for rep in range(2):
        s = B.Scd(cfg, DEV)
        st = s.alloc_state()
        s.reset(st)
        h = torch.empty((w.B, w.C, w.L, w.d), dtype=torch.bfloat16, device=DEV)
        for _ in range(w.N + 5):                   # more steps than any decode needs
            s.gather_hidden(table, w.age_cap, st, h)
            s.step(h, W, st)
        rc, flags = s.status(st)
        assert rc == B.SCD_OK and flags[1] == 1
        outs.append((s.state_field(st, B.F_OUT).cpu().numpy().copy(),
                     s.state_field(st, B.F_ITER).cpu().numpy().copy(),
                     s.state_field(st, B.F_POS).cpu().numpy().copy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    assert (outs[0][0] >= 0).all() and (outs[0][2] == w.N).all()
    assert (outs[0][1] < w.N).all()               # extra steps after the end did not count


def test_gather_matches_host_gather():
    w = wl.scaled(wl.WORKLOADS["C2"], name="g", N=70, V=512, d=64, v_lo=0, v_hi=512, B=2)
    cfg = B.config_from_workload(w)
    s = B.Scd(cfg, DEV)
    st = s.alloc_state()
    s.reset(st)
    tab = wl.HiddenTable(w)
    table = _bf16(tab.full(drop_cache=False))
    pos = np.array([3, 60], dtype=np.int32)
    age = np.random.default_rng(0).integers(0, 30, (w.B, w.L)).astype(np.int32)
    s.state_field(st, B.F_POS).copy_(torch.from_numpy(pos))
    s.state_field(st, B.F_AGE).copy_(torch.from_numpy(age.ravel()))
    h = torch.empty((w.B, w.C, w.L, w.d), dtype=torch.bfloat16, device=DEV)
    s.gather_hidden(table, w.age_cap, st, h)
    torch.cuda.synchronize()
    ages = [[age[b, (pos[b] + k) % w.L] for k in range(w.L)] for b in range(w.B)]
    want = tab.window(list(pos), ages)
    assert np.array_equal(h.view(torch.int16).cpu().numpy().view(np.uint16), want)


def test_numeric_fault_is_reported():
    w = wl.scaled(wl.WORKLOADS["C0"], name="nan", N=16, L=4, V=256)
    cfg = B.config_from_workload(w)
    s = B.Scd(cfg, DEV)
    st = s.alloc_state()
    s.reset(st)
    z = torch.zeros((1, 4, 256), device=DEV)
    z[0, 1, 5] = float("nan")
    s.step_logits(z, st)
    rc, flags = s.status(st)
    assert rc == B.SCD_ENUMERIC and flags[0] != 0


def test_determinism_batched_rows_of_a_sequence_on_many_workgroups():
    # C3-like: 16 sequences x 32 rows, every row its own workgroup, the rows of a sequence spread
    # over the chip; the sequence's last workgroup to finish reads what the others stored.  Two
    # decodes side by side must agree after EVERY step (first difference stops the test).
    w = wl.scaled(wl.WORKLOADS["C3"], name="det16", N=200, V=8200, d=512, v_lo=4, v_hi=8196)
    cfg = B.config_from_workload(w)
    W = _bf16(wl.lm_head_weight(w))
    table = _bf16(wl.HiddenTable(w).full())
    runs = []
    for rep in range(2):
        s = B.Scd(cfg, DEV)
        st = s.alloc_state()
        s.reset(st)
        runs.append((s, st, torch.empty((w.B, w.C, w.L, w.d), dtype=torch.bfloat16, device=DEV)))
    fields = (B.F_POS, B.F_ITER, B.F_X, B.F_AGE, B.F_Y, B.F_K, B.F_ACCEPT, B.F_OUT)
    steps = 0
    while True:
        for s, st, h in runs:
            s.gather_hidden(table, w.age_cap, st, h)
            s.step(h, W, st)
        for f in fields:
            a, b = (s.state_field(st, f) for s, st, _ in runs)
            assert torch.equal(a, b), f"step {steps}: field {f} differs between two identical decodes"
        steps += 1
        rc, flags = runs[0][0].status(runs[0][1])
        assert rc == B.SCD_OK
        if flags[1]:
            break
        assert steps <= w.N
    assert steps >= 20


# ------------------------------------ whole decodes of the large workloads (kept last: the longest)
# Each is cut into parts of about a minute that continue one decode (a shared LockStep object), so
# that a test finishes -- and the runner prints -- at least that often.
_LONG = {}


def _long_part(key, w, upto, **kw):
    """Continues the lock-step decode `key` until `upto` iterations are done (None: to the end)."""
    import json, os
    from lockstep import LockStep
    if key not in _LONG:
        _LONG.clear()                               # one large decode at a time
        _LONG[key] = LockStep(w, DEV, **kw)
    ls = _LONG[key]
    st = ls.run(upto)
    if upto is None or ls.oracle.done():
        print(f"\n[{w.name}] {st}")
        assert st["adopt_accept"] + st["adopt_resid"] <= max(3, 1e-3 * st["draws"])
        assert st["adopt_topk"] <= max(3, 1e-2 * st["draws"])
    return ls, st


def _log_long(key, w):
    import json, os
    ls = _LONG.pop(key)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    with open(os.path.join(root, "gpurun_out", "parity_flags.jsonl"), "a") as f:
        f.write(json.dumps(dict(workload=w.name, B=w.B, L=w.L, N=w.N, n=w.n_allowed, d=w.d, top_k=w.top_k,
                                top_p=w.top_p, options={}, whole_decode=bool(ls.oracle.done()),
                                **ls.stats)) + "\n")


@pytest.mark.parametrize("upto", [140, 280, None])
def test_lockstep_C3_full(upto):
    # 16 ragged sequences, the whole decode (410 iterations, 204 759 rows), logits compared on every row
    w = wl.WORKLOADS["C3"]
    ls, st = _long_part("C3", w, upto)
    if upto is None:
        assert ls.oracle.done() and st["steps"] == 410
        _log_long("C3", w)


def test_lockstep_C4_shape_to_the_sequence_end():
    # the video shape (V = 64000, d = 4096, L = 64, B = 2; same kernels and launch shapes as C4)
    # on 8 short frames, decoded to the end: frame boundaries and the clipped last windows
    ls, st = _lockstep(wl.scaled(wl.WORKLOADS["C4"], name="C4-short", N=8 * 48))
    assert ls.oracle.done()


@pytest.mark.parametrize("upto", [175, 350, 525, 700])
def test_lockstep_C4_across_frame_boundaries(upto):
    # C4 itself from the start across three frame boundaries (frames of 1600 tokens; the hidden
    # states of a frame are correlated with the previous frame's)
    w = wl.WORKLOADS["C4"]
    ls, st = _long_part("C4", w, upto)
    if upto == 700:
        assert min(ls.oracle.i) >= 3 * (w.N // w.frames) + w.L, ls.oracle.i
        print(f"\n[{w.name}, 700 iterations] {st}")
        assert st["adopt_accept"] + st["adopt_resid"] <= max(3, 1e-3 * st["draws"])
        assert st["adopt_topk"] <= max(3, 1e-2 * st["draws"])
        _log_long("C4", w)
