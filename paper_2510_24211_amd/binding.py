"""Thin ctypes binding of libscd.so (the C ABI in include/scd.h).

Argument marshalling only: every step of the decode iteration runs in the HIP
kernels.  PyTorch is used for device memory and the current HIP stream.  The
functions carry the same names as the C entry points.  There is no CPU
fallback: if the shared library is missing, loading raises.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libscd.so")

SCD_OK, SCD_EINVAL, SCD_EWORKSPACE, SCD_EHIP, SCD_ENUMERIC, SCD_EUNSUPPORTED, SCD_ESCRATCH = 0, -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 8 << 20

# scd_field
(F_POS, F_ITER, F_X, F_AGE, F_OUT, F_ACCEPT, F_Y, F_K, F_PX, F_QX, F_THR, F_LSE, F_NKEPT, F_Z,
 F_FLAGS, F_VERIFIED, F_TICKET, F_G, F_DIAG, F_S2, F_HAMM, F_XHIST, F_PHIST) = range(23)
F_COUNT = 23
COUPLING_MC, COUPLING_GS = 0, 1

_FIELD_DTYPE = {
    F_POS: torch.int32, F_ITER: torch.int32, F_X: torch.int32, F_AGE: torch.int32,
    F_OUT: torch.int32, F_ACCEPT: torch.int32, F_Y: torch.int32, F_K: torch.uint8,
    F_PX: torch.float32, F_QX: torch.float32, F_THR: torch.float32, F_LSE: torch.float32,
    F_NKEPT: torch.int32, F_Z: torch.float32, F_FLAGS: torch.int32, F_VERIFIED: torch.int32,
    F_TICKET: torch.int32, F_G: torch.int32, F_DIAG: torch.float32, F_S2: torch.float32,
    F_HAMM: torch.int32, F_XHIST: torch.int32, F_PHIST: torch.int32,
}


class ScdConfig(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("L", ctypes.c_int32), ("N", ctypes.c_int32),
                ("V", ctypes.c_int32), ("d", ctypes.c_int32), ("v_lo", ctypes.c_int32),
                ("v_hi", ctypes.c_int32), ("top_k", ctypes.c_int32),
                ("temperature", ctypes.c_float), ("cfg_lambda", ctypes.c_float),
                ("coupling", ctypes.c_int32), ("sjd_mix", ctypes.c_float),
                ("top_p", ctypes.c_float), ("diagnostics", ctypes.c_int32),
                ("seed", ctypes.c_uint64)]


class ScdError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {code} ({strerror(code)})")
        self.code = code


_lib = None


def load():
    """Loads libscd.so (built in-tree by paper_2510_24211_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("SCD_LIB", LIB_PATH)      # SCD_LIB: an alternative build of the library
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with "
                           "`python -m paper_2510_24211_amd.build` (there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    cfgp = ctypes.POINTER(ScdConfig)
    lib.scd_workspace_bytes.restype = sz
    lib.scd_workspace_bytes.argtypes = [cfgp]
    lib.scd_state_bytes.restype = sz
    lib.scd_state_bytes.argtypes = [cfgp]
    lib.scd_create.argtypes = [ctypes.POINTER(vp), cfgp, vp, sz, vp]
    lib.scd_destroy.argtypes = [vp]
    lib.scd_reset.argtypes = [vp, vp]
    lib.scd_state_field.argtypes = [vp, vp, ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(sz)]
    lib.scd_lm_head.argtypes = [vp, vp, vp, vp]
    lib.scd_select.argtypes = [vp, vp, i32, vp, vp, vp]
    lib.scd_couple_draft.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.scd_couple_draft_static.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.scd_verify.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.scd_step.argtypes = [vp, vp, vp, vp]
    lib.scd_step_logits.argtypes = [vp, vp, vp]
    lib.scd_set_lm_head_events.argtypes = [vp, vp, vp]
    lib.scd_lm_head_kernel_name.argtypes = [vp, ctypes.c_char_p, sz]
    lib.scd_status.argtypes = [vp, vp, ctypes.POINTER(i32 * 4)]
    lib.scd_strerror.restype = ctypes.c_char_p
    lib.scd_strerror.argtypes = [ctypes.c_int]
    lib.scdw_gather_hidden.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.scdw_copy.argtypes = [vp, vp, vp, sz]
    for name in ("scd_create", "scd_destroy", "scd_reset", "scd_state_field", "scd_lm_head",
                 "scd_select", "scd_couple_draft", "scd_couple_draft_static", "scd_verify", "scd_step", "scd_step_logits",
                 "scd_set_lm_head_events", "scd_lm_head_kernel_name",
                 "scd_status", "scdw_gather_hidden", "scdw_copy"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(code):
    return load().scd_strerror(int(code)).decode()


def make_config(B, L, N, V, d=0, v_lo=0, v_hi=-1, top_k=0, temperature=1.0, cfg_lambda=0.0,
                seed=0, coupling=0, sjd_mix=0.0, top_p=0.0, diagnostics=0):
    return ScdConfig(B, L, N, V, d, v_lo, V if v_hi < 0 else v_hi, top_k, temperature, cfg_lambda,
                     coupling, sjd_mix, top_p, diagnostics, seed & 0xFFFFFFFFFFFFFFFF)


def workspace_bytes(cfg):
    return load().scd_workspace_bytes(ctypes.byref(cfg))


def state_bytes(cfg):
    return load().scd_state_bytes(ctypes.byref(cfg))


def _ptr(t, dtypes, numel, what):
    """Device pointer of a contiguous CUDA tensor after checking dtype and size."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what}: expected a CUDA tensor")
    if t.dtype not in dtypes:
        raise TypeError(f"{what}: dtype {t.dtype}, expected one of {dtypes}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: tensor must be contiguous")
    if t.numel() < numel:
        raise ValueError(f"{what}: {t.numel()} elements, need {numel}")
    return ctypes.c_void_p(t.data_ptr())


_BF16 = (torch.bfloat16, torch.int16, torch.uint16)


class Scd:
    """One scd_ctx plus its workspace.  Methods = the C entry points."""

    def __init__(self, cfg: ScdConfig, device="cuda:0", stream=None):
        self.lib = load()
        self.cfg = cfg
        self.device = torch.device(device)
        self.n = cfg.v_hi - cfg.v_lo
        self.C = 2 if cfg.cfg_lambda != 0.0 else 1
        need = self.lib.scd_workspace_bytes(ctypes.byref(cfg))
        if need == 0:
            raise ScdError(SCD_EINVAL, "scd_workspace_bytes")
        self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        ctx = ctypes.c_void_p()
        rc = self.lib.scd_create(ctypes.byref(ctx), ctypes.byref(cfg),
                                 ctypes.c_void_p(self.workspace.data_ptr()), need,
                                 ctypes.c_void_p(self.stream.cuda_stream))
        if rc != SCD_OK:
            raise ScdError(rc, "scd_create")
        self.ctx = ctx

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.scd_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        self.close()

    @staticmethod
    def _check(rc, what):
        if rc != SCD_OK:
            raise ScdError(rc, what)

    # -- state ------------------------------------------------------------
    def alloc_state(self):
        nbytes = self.lib.scd_state_bytes(ctypes.byref(self.cfg))
        return torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    def state_field(self, state, field):
        """A tensor view of one field of the state buffer."""
        p, nb = ctypes.c_void_p(), ctypes.c_size_t()
        self._check(self.lib.scd_state_field(self.ctx, ctypes.c_void_p(state.data_ptr()), field,
                                             ctypes.byref(p), ctypes.byref(nb)), "scd_state_field")
        off = p.value - state.data_ptr()
        return state[off: off + nb.value].view(_FIELD_DTYPE[field])

    def reset(self, state):
        self._check(self.lib.scd_reset(self.ctx, _ptr(state, (torch.uint8,),
                                                      state_bytes(self.cfg), "state")), "scd_reset")

    def status(self, state):
        flags = (ctypes.c_int32 * 4)()
        rc = self.lib.scd_status(self.ctx, ctypes.c_void_p(state.data_ptr()), ctypes.byref(flags))
        return rc, list(flags)

    # -- stages -------------------------------------------------------------
    def lm_head(self, h, W, z):
        c = self.cfg
        self._check(self.lib.scd_lm_head(
            self.ctx, _ptr(h, _BF16, c.B * self.C * c.L * c.d, "h"),
            _ptr(W, _BF16, c.V * c.d, "W"),
            _ptr(z, (torch.float32,), c.B * c.L * self.n, "z")), "scd_lm_head")

    def select(self, z, rows, thr, lse, nkept):
        self._check(self.lib.scd_select(
            self.ctx, _ptr(z, (torch.float32,), rows * self.n, "z"), rows,
            _ptr(thr, (torch.float32,), rows, "thr"), _ptr(lse, (torch.float32,), rows, "lse"),
            _ptr(nkept, (torch.int32,), rows, "nkept")), "scd_select")

    def couple_draft_static(self, z_cur, z_prev, x, fresh, pos0, it, y, k):
        """scd_couple_draft with its scratch in the library's static device array."""
        c = self.cfg
        r = c.B * c.L
        self._check(self.lib.scd_couple_draft_static(
            self.ctx, _ptr(z_cur, (torch.float32,), r * self.n, "z_cur"),
            _ptr(z_prev, (torch.float32,), r * self.n, "z_prev"),
            _ptr(x, (torch.int32,), r, "x"), _ptr(fresh, (torch.uint8,), r, "fresh"),
            _ptr(pos0, (torch.int32,), c.B, "pos0"), int(it),
            _ptr(y, (torch.int32,), r, "y"), _ptr(k, (torch.uint8,), r, "k")), "scd_couple_draft_static")

    def couple_draft(self, z_cur, z_prev, x, fresh, pos0, it, y, k):
        c = self.cfg
        r = c.B * c.L
        self._check(self.lib.scd_couple_draft(
            self.ctx, _ptr(z_cur, (torch.float32,), r * self.n, "z_cur"),
            _ptr(z_prev, (torch.float32,), r * self.n, "z_prev"),
            _ptr(x, (torch.int32,), r, "x"), _ptr(fresh, (torch.uint8,), r, "fresh"),
            _ptr(pos0, (torch.int32,), c.B, "pos0"), int(it),
            _ptr(y, (torch.int32,), r, "y"), _ptr(k, (torch.uint8,), r, "k")), "scd_couple_draft")

    def verify(self, k, y, pos0, accept_len, out):
        c = self.cfg
        r = c.B * c.L
        self._check(self.lib.scd_verify(
            self.ctx, _ptr(k, (torch.uint8,), r, "k"), _ptr(y, (torch.int32,), r, "y"),
            _ptr(pos0, (torch.int32,), c.B, "pos0"),
            _ptr(accept_len, (torch.int32,), c.B, "accept_len"),
            _ptr(out, (torch.int32,), c.B * c.N, "out")), "scd_verify")

    def step(self, h, W, state):
        c = self.cfg
        self._check(self.lib.scd_step(
            self.ctx, _ptr(h, _BF16, c.B * self.C * c.L * c.d, "h"),
            _ptr(W, _BF16, c.V * c.d, "W"),
            _ptr(state, (torch.uint8,), state_bytes(c), "state")), "scd_step")

    def set_lm_head_events(self, ev_start, ev_stop):
        """ev_*: hipEvent_t handles as integers (or None, None to turn off)."""
        self._check(self.lib.scd_set_lm_head_events(
            self.ctx, ctypes.c_void_p(ev_start) if ev_start else None,
            ctypes.c_void_p(ev_stop) if ev_stop else None), "scd_set_lm_head_events")

    def lm_head_kernel_name(self):
        buf = ctypes.create_string_buffer(96)
        self._check(self.lib.scd_lm_head_kernel_name(self.ctx, buf, 96), "scd_lm_head_kernel_name")
        return buf.value.decode()

    def step_logits(self, z, state):
        c = self.cfg
        self._check(self.lib.scd_step_logits(
            self.ctx, _ptr(z, (torch.float32,), c.B * c.L * self.n, "z"),
            _ptr(state, (torch.uint8,), state_bytes(c), "state")), "scd_step_logits")

    # -- benchmark plumbing ---------------------------------------------------
    def gather_hidden(self, table, age_cap, state, h):
        c = self.cfg
        rows = c.B * self.C * c.N * (age_cap + 1)
        rc = self.lib.scdw_gather_hidden(
            ctypes.c_void_p(self.stream.cuda_stream), _ptr(table, _BF16, rows * c.d, "table"),
            c.B, self.C, c.L, c.N, c.d, age_cap,
            ctypes.c_void_p(self.state_field(state, F_POS).data_ptr()),
            ctypes.c_void_p(self.state_field(state, F_AGE).data_ptr()),
            _ptr(h, _BF16, c.B * self.C * c.L * c.d, "h"))
        self._check(rc, "scdw_gather_hidden")


def device_copy(src, dst, stream=None):
    """dst <- src by the library's plain copy kernel (profiler counter calibration)."""
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    st = stream if stream is not None else torch.cuda.current_stream(src.device)
    rc = load().scdw_copy(ctypes.c_void_p(st.cuda_stream), ctypes.c_void_p(src.data_ptr()),
                          ctypes.c_void_p(dst.data_ptr()), nbytes)
    if rc != 0:
        raise RuntimeError(f"scdw_copy failed with {rc}")
    return nbytes


def config_from_workload(w):
    """ScdConfig for a paper_2510_24211_amd.workload.Workload."""
    return make_config(B=w.B, L=w.L, N=w.N, V=w.V, d=w.d, v_lo=w.v_lo, v_hi=w.v_hi, top_k=w.top_k,
                       temperature=w.temperature, cfg_lambda=w.cfg_lambda, seed=w.seed, top_p=w.top_p)
