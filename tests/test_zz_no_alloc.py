"""scd_couple_draft_static (the entry point that allocates nothing: its scratch is a static
device array inside the library) against scd_couple_draft (scratch in the caller's workspace),
through the C ABI: same inputs, identical outputs, on two calls in a row, the second smaller."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2510_24211_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(Bn, L, n, top_k, N, pos0, seed, it, top_p=0.0, both=False):
    g = np.random.default_rng(seed)
    z_prev = (g.standard_normal((Bn, L, n)) * 2).astype(np.float32)
    scale = np.float32(0.5) ** g.integers(0, 10, (Bn, L, 1)).astype(np.float32)
    z_cur = (z_prev + scale * g.standard_normal((Bn, L, n)).astype(np.float32)).astype(np.float32)
    fresh = (g.random((Bn, L)) < 0.25).astype(np.uint8)
    x = g.integers(0, n, (Bn, L)).astype(np.int32)
    # drafts of evaluated positions must lie in the support of q: take the row's largest logit
    x = np.where(fresh == 1, x, z_prev.argmax(-1).astype(np.int32)).astype(np.int32)
    cfg = B.make_config(B=Bn, L=L, N=N, V=n, top_k=top_k, top_p=top_p, seed=seed)
    sc = B.Scd(cfg, DEV)
    t = lambda a: torch.from_numpy(a).to(DEV)
    args = (t(z_cur), t(z_prev), t(x), t(fresh), t(np.array(pos0, dtype=np.int32)), it)
    outs = []
    for fn in (sc.couple_draft, sc.couple_draft_static):
        y = torch.full((Bn, L), -5, dtype=torch.int32, device=DEV)
        k = torch.full((Bn, L), 9, dtype=torch.uint8, device=DEV)
        fn(*args, y, k)
        torch.cuda.synchronize()
        outs.append((y.cpu().numpy(), k.cpu().numpy()))
    (y0, k0), (y1, k1) = outs
    assert np.array_equal(k0, k1), "accept bits differ between the two entry points"
    assert np.array_equal(y0, y1), "tokens differ between the two entry points"
    live = [min(L, N - p) for p in pos0]
    assert all((k0[b, :live[b]] <= 1).all() and (y0[b, :live[b]] >= 0).all() for b in range(Bn))
    if both:                                           # both branches of the MRS call were taken
        assert (k0 == 0).any() and (k0[0, :live[0]] == 1).any()
    return sc


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    torch.cuda.set_device(0)
    B.load()
    # first call: rows long enough for the slice kernel (candidate lists + per-row scalars in scratch)
    _case(Bn=2, L=16, n=40000, top_k=2000, N=200, pos0=[3, 190], seed=101, it=5, both=True)
    # second call, smaller in every dimension: the scratch still holds the first call's contents
    _case(Bn=1, L=8, n=20000, top_k=500, N=64, pos0=[0], seed=102, it=2)
    # and one whose rows do not use the candidate lists at all
    _case(Bn=3, L=5, n=1000, top_k=100, N=50, pos0=[0, 45, 49], seed=103, it=1)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    torch.cuda.set_device(0)
    lib = B.load()
    # 8 x 32 rows of 40000 ids: 256 x 49216 bytes of candidate lists > 8 MiB
    cfg = B.make_config(B=8, L=32, N=100, V=40000, top_k=2000)
    sc = B.Scd(cfg, DEV)
    z = torch.zeros((8, 32, 40000), device=DEV)
    x = torch.zeros((8, 32), dtype=torch.int32, device=DEV)
    pos = torch.zeros(8, dtype=torch.int32, device=DEV)
    y = torch.empty((8, 32), dtype=torch.int32, device=DEV)
    k = torch.empty((8, 32), dtype=torch.uint8, device=DEV)
    p = lambda t_: ctypes.c_void_p(t_.data_ptr())
    rc = lib.scd_couple_draft_static(sc.ctx, p(z), p(z), p(x), None, p(pos), 0, p(y), p(k))
    assert rc == B.SCD_ESCRATCH and "SCD_STATIC_SCRATCH_BYTES" in B.strerror(rc)
    # the same rows without top-k need 24 bytes per row only
    cfg2 = B.make_config(B=8, L=32, N=100, V=40000)
    sc2 = B.Scd(cfg2, DEV)
    assert lib.scd_couple_draft_static(sc2.ctx, p(z), p(z), p(x), None, p(pos), 0, p(y), p(k)) == B.SCD_OK
    torch.cuda.synchronize()
    assert lib.scd_couple_draft_static(None, p(z), p(z), p(x), None, p(pos), 0, p(y), p(k)) == B.SCD_EINVAL
