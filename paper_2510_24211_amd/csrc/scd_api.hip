// Host side of the C ABI declared in include/scd.h: argument validation, the
// layout of the device-resident decode state, and the launch sequence of one
// SCD iteration.  No device memory is allocated here and nothing synchronises
// except scd_status.
#include "../../include/scd.h"

#include <atomic>
#include <cmath>
#include <cstring>
#include <new>

#include "scd_kernels.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t off[SCD_F_COUNT];
  size_t bytes[SCD_F_COUNT];
  size_t total;
};

bool valid_config(const scd_config* c) {
  if (!c) return false;
  if (c->B < 1 || c->B > (1 << 20)) return false;
  if (c->L < 1 || c->L > 256) return false;
  if (c->N < 1 || c->V < 1) return false;
  if (c->d < 0 || (c->d % 8) != 0) return false;
  if (c->v_lo < 0 || c->v_hi <= c->v_lo || c->v_hi > c->V) return false;
  // the kernels index the logits of one sequence's window with 32 bits
  if (static_cast<int64_t>(c->L) * (c->v_hi - c->v_lo) >= (static_cast<int64_t>(1) << 31)) return false;
  if (c->top_k < 0) return false;
  if (!(c->temperature > 0.f) || !std::isfinite(c->temperature)) return false;
  if (!std::isfinite(c->cfg_lambda)) return false;
  if (!(c->sjd_mix >= 0.f && c->sjd_mix <= 1.f)) return false;
  if (c->coupling < 0) return false;
  if (!(c->top_p >= 0.f && c->top_p <= 1.f)) return false;
  if (c->diagnostics != 0 && c->diagnostics != 1) return false;
  return true;
}

// round(top_p * 2^24); 0 where the nucleus filter is off (top_p = 0 or 1, or so small that it
// rounds to nothing: then the most probable id alone would be kept, which 1 expresses)
uint32_t top_p24_of(const scd_config& c) {
  if (!(c.top_p > 0.f && c.top_p < 1.f)) return 0u;
  const long v = std::lround(static_cast<double>(c.top_p) * 16777216.0);
  return static_cast<uint32_t>(v < 1 ? 1 : v);
}

Layout make_layout(const scd_config& c) {
  const size_t B = c.B, L = c.L, N = c.N, n = c.v_hi - c.v_lo;
  size_t sz[SCD_F_COUNT];
  sz[SCD_F_POS] = 4 * B;
  sz[SCD_F_ITER] = 4 * B;
  sz[SCD_F_X] = 4 * B * L;
  sz[SCD_F_AGE] = 4 * B * L;
  sz[SCD_F_OUT] = 4 * B * N;
  sz[SCD_F_ACCEPT] = 4 * B;
  sz[SCD_F_Y] = 4 * B * L;
  sz[SCD_F_K] = B * L;
  sz[SCD_F_PX] = 4 * B * L;
  sz[SCD_F_QX] = 4 * B * L;
  sz[SCD_F_THR] = 4 * 2 * B * L;
  sz[SCD_F_LSE] = 4 * 2 * B * L;
  sz[SCD_F_NKEPT] = 4 * 2 * B * L;
  sz[SCD_F_Z] = 4 * 2 * B * L * n;
  sz[SCD_F_FLAGS] = 16;
  sz[SCD_F_VERIFIED] = 4 * B;
  sz[SCD_F_TICKET] = 4 * B;
  sz[SCD_F_G] = 4 * B * L;
  sz[SCD_F_DIAG] = 4 * 4 * B * L;
  sz[SCD_F_S2] = 4 * 2 * B * L;
  sz[SCD_F_HAMM] = 4 * 6 * B;
  sz[SCD_F_XHIST] = 4 * 3 * B * L;
  sz[SCD_F_PHIST] = 4 * 3 * B;
  Layout lay;
  size_t o = 0;
  for (int f = 0; f < SCD_F_COUNT; ++f) {
    lay.off[f] = o;
    lay.bytes[f] = sz[f];
    o += align_up(sz[f]);
  }
  lay.total = o;
  return lay;
}

// Workspace: thresholds / normalisers / kept counts of the two logit arrays of
// a stand-alone scd_couple_draft call ...
size_t small_need(const scd_config& c) {
  const size_t rows = static_cast<size_t>(c.B) * c.L;
  return 6 * align_up(4 * rows);
}
// ... followed by the per-row candidate scratch of the slice kernel.
size_t workspace_need(const scd_config& c) {
  return small_need(c) + align_up(scd::row_candidate_bytes(c.B * c.L));
}

// ---- scratch of the entry point that allocates nothing -----------------------------------
// scd_couple_draft_static keeps what scd_couple_draft keeps in the caller's workspace (the
// thresholds / normalisers / kept counts of its two logit arrays and the candidate lists of the
// slice kernel) in this array.  Every GPU the library runs on holds its own copy at its own
// address until the process ends; `scratch` itself is only the host-side name of the symbol, so
// host code uses the per-device address that hipGetSymbolAddress returned, never the name.
__device__ __align__(256) unsigned char scratch[SCD_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];      // device address of `scratch` per device

// Address of the current device's copy; looked up once per device (racing threads store the
// same value).  Allocates nothing.
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return SCD_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return SCD_EUNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SCD_EHIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return SCD_OK;
}

}  // namespace

struct scd_ctx {
  scd_config cfg;
  Layout lay;
  void* ws;
  size_t ws_bytes;
  hipStream_t stream;
  int n;   // allowed ids
  int C;   // LM-head rows per window position
  hipEvent_t ev_start, ev_stop;   // optional instrumentation around the LM-head kernel
  size_t row_lds[2];              // dynamic-LDS limit already set for the row kernels (launch_row, both builds)
};

namespace {

template <typename T>
inline T* field(const scd_ctx* c, void* st, int f) {
  return reinterpret_cast<T*>(static_cast<char*>(st) + c->lay.off[f]);
}
inline int hip_rc(hipError_t e) { return e == hipSuccess ? SCD_OK : SCD_EHIP; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int run_tail(scd_ctx* c, void* st, int tiles = 0) {
  // z of this iteration is in place in the ring.
  const size_t half = static_cast<size_t>(c->cfg.B) * c->cfg.L * c->n;
  if (c->n <= scd::kRowKernelMaxN) {
    // one fused launch: select + softmax + MRS per row, commit by each sequence's last row
    scd::RowArgs ra{};
    ra.alpha = 1.0f;
    ra.mode = scd::kRowRing;
    ra.z_cur = field<float>(c, st, SCD_F_Z);
    ra.parity_stride = half;
    ra.thr = field<float>(c, st, SCD_F_THR);
    ra.lse = field<float>(c, st, SCD_F_LSE);
    ra.nkept = field<int32_t>(c, st, SCD_F_NKEPT);
    ra.x = field<int32_t>(c, st, SCD_F_X);
    ra.age = field<int32_t>(c, st, SCD_F_AGE);
    ra.pos = field<int32_t>(c, st, SCD_F_POS);
    ra.iter = field<int32_t>(c, st, SCD_F_ITER);
    ra.y = field<int32_t>(c, st, SCD_F_Y);
    ra.k = field<uint8_t>(c, st, SCD_F_K);
    ra.px = field<float>(c, st, SCD_F_PX);
    ra.qx = field<float>(c, st, SCD_F_QX);
    ra.flags = field<int32_t>(c, st, SCD_F_FLAGS);
    ra.ticket = field<int32_t>(c, st, SCD_F_TICKET);
    ra.X = field<int32_t>(c, st, SCD_F_X);
    ra.age_w = field<int32_t>(c, st, SCD_F_AGE);
    ra.verified = field<int32_t>(c, st, SCD_F_VERIFIED);
    ra.accept_len = field<int32_t>(c, st, SCD_F_ACCEPT);
    ra.out = field<int32_t>(c, st, SCD_F_OUT);
    ra.rows = c->cfg.B * c->cfg.L;
    ra.B = c->cfg.B; ra.L = c->cfg.L; ra.N = c->cfg.N; ra.n = c->n; ra.top_k = c->cfg.top_k;
    ra.top_p24 = top_p24_of(c->cfg);
    ra.v_lo = c->cfg.v_lo; ra.seed = c->cfg.seed;
    ra.cand_base = static_cast<char*>(c->ws) + small_need(c->cfg);
    ra.tiles = tiles;            // > 0: the LM head has already written the candidate lists
    ra.gumbel = c->cfg.coupling == SCD_COUPLING_GS;
    ra.alpha = 1.0f - c->cfg.sjd_mix;
    ra.g = field<int32_t>(c, st, SCD_F_G);
    if (c->cfg.diagnostics) {
      ra.diag = field<float>(c, st, SCD_F_DIAG);
      ra.s2 = field<float>(c, st, SCD_F_S2);
      ra.hamm = field<int32_t>(c, st, SCD_F_HAMM);
      ra.xhist = field<int32_t>(c, st, SCD_F_XHIST);
      ra.phist = field<int32_t>(c, st, SCD_F_PHIST);
    }
    return hip_rc(scd::launch_row(ra, c->stream, c->row_lds));
  }
  // rows too long for the LDS-resident kernel: select -> MRS -> commit
  scd::SelectArgs sa{};
  sa.z = field<float>(c, st, SCD_F_Z);
  sa.parity_stride = half;
  sa.pos = field<int32_t>(c, st, SCD_F_POS);
  sa.iter = field<int32_t>(c, st, SCD_F_ITER);
  sa.thr = field<float>(c, st, SCD_F_THR);
  sa.lse = field<float>(c, st, SCD_F_LSE);
  sa.nkept = field<int32_t>(c, st, SCD_F_NKEPT);
  sa.flags = field<int32_t>(c, st, SCD_F_FLAGS);
  sa.rows = c->cfg.B * c->cfg.L;
  sa.B = c->cfg.B; sa.L = c->cfg.L; sa.N = c->cfg.N; sa.n = c->n; sa.top_k = c->cfg.top_k;
  if (hipError_t e = scd::launch_select(sa, c->stream); e != hipSuccess) return SCD_EHIP;

  scd::MrsArgs ma{};
  ma.z_cur = field<float>(c, st, SCD_F_Z);
  ma.parity_stride = half;
  ma.thr_cur = field<float>(c, st, SCD_F_THR);
  ma.lse_cur = field<float>(c, st, SCD_F_LSE);
  ma.x = field<int32_t>(c, st, SCD_F_X);
  ma.age = field<int32_t>(c, st, SCD_F_AGE);
  ma.pos = field<int32_t>(c, st, SCD_F_POS);
  ma.iter = field<int32_t>(c, st, SCD_F_ITER);
  ma.ring = 1;
  ma.y = field<int32_t>(c, st, SCD_F_Y);
  ma.k = field<uint8_t>(c, st, SCD_F_K);
  ma.px = field<float>(c, st, SCD_F_PX);
  ma.qx = field<float>(c, st, SCD_F_QX);
  ma.B = c->cfg.B; ma.L = c->cfg.L; ma.N = c->cfg.N; ma.n = c->n; ma.seed = c->cfg.seed;
  if (hipError_t e = scd::launch_mrs(ma, c->stream); e != hipSuccess) return SCD_EHIP;

  scd::CommitArgs ca{};
  ca.k = field<uint8_t>(c, st, SCD_F_K);
  ca.y = field<int32_t>(c, st, SCD_F_Y);
  ca.pos = field<int32_t>(c, st, SCD_F_POS);
  ca.iter = field<int32_t>(c, st, SCD_F_ITER);
  ca.X = field<int32_t>(c, st, SCD_F_X);
  ca.age = field<int32_t>(c, st, SCD_F_AGE);
  ca.verified = field<int32_t>(c, st, SCD_F_VERIFIED);
  ca.accept_len = field<int32_t>(c, st, SCD_F_ACCEPT);
  ca.out = field<int32_t>(c, st, SCD_F_OUT);
  ca.slide = 1;
  ca.B = c->cfg.B; ca.L = c->cfg.L; ca.N = c->cfg.N; ca.n = c->n; ca.v_lo = c->cfg.v_lo;
  ca.seed = c->cfg.seed;
  return hip_rc(scd::launch_commit(ca, c->stream));
}

}  // namespace

extern "C" {

size_t scd_workspace_bytes(const scd_config* cfg) {
  return valid_config(cfg) ? workspace_need(*cfg) : 0;
}

size_t scd_state_bytes(const scd_config* cfg) {
  return valid_config(cfg) ? make_layout(*cfg).total : 0;
}

int scd_create(scd_ctx** out, const scd_config* cfg, void* d_workspace, size_t workspace_bytes,
               void* hip_stream) {
  if (!out || !valid_config(cfg)) return SCD_EINVAL;
  if (cfg->coupling != SCD_COUPLING_MC && cfg->coupling != SCD_COUPLING_GS) return SCD_EUNSUPPORTED;
  // the Gumbel draw lives in the fused row kernel only
  if (top_p24_of(*cfg) != 0u && cfg->v_hi - cfg->v_lo > scd::kRowKernelMaxN) return SCD_EUNSUPPORTED;
  if (cfg->diagnostics && cfg->v_hi - cfg->v_lo > scd::kRowKernelMaxN) return SCD_EUNSUPPORTED;
  if ((cfg->coupling == SCD_COUPLING_GS || cfg->sjd_mix > 0.f) &&
      cfg->v_hi - cfg->v_lo > scd::kRowKernelMaxN)
    return SCD_EUNSUPPORTED;
  if (!d_workspace || !aligned(d_workspace, kAlign) || workspace_bytes < workspace_need(*cfg))
    return SCD_EWORKSPACE;
  scd_ctx* c = new (std::nothrow) scd_ctx;
  if (!c) return SCD_EINVAL;
  c->cfg = *cfg;
  c->lay = make_layout(*cfg);
  c->ws = d_workspace;
  c->ws_bytes = workspace_bytes;
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->n = cfg->v_hi - cfg->v_lo;
  c->C = cfg->cfg_lambda != 0.f ? 2 : 1;
  c->ev_start = nullptr;
  c->ev_stop = nullptr;
  c->row_lds[0] = c->row_lds[1] = 0;
  // Set-up for scd_couple_draft_static: look the scratch address of the current device up now,
  // outside any stream capture.  Best effort (a host without a GPU can still create a context to
  // query layouts); the entry point repeats the lookup if it is still missing.
  void* unused = nullptr;
  (void)static_scratch(&unused);
  (void)hipGetLastError();
  *out = c;
  return SCD_OK;
}

int scd_destroy(scd_ctx* ctx) {
  if (!ctx) return SCD_EINVAL;
  delete ctx;
  return SCD_OK;
}

int scd_state_field(const scd_ctx* ctx, void* d_state, int f, void** d_ptr, size_t* bytes) {
  if (!ctx || !d_state || f < 0 || f >= SCD_F_COUNT || !d_ptr || !bytes) return SCD_EINVAL;
  *d_ptr = static_cast<char*>(d_state) + ctx->lay.off[f];
  *bytes = ctx->lay.bytes[f];
  return SCD_OK;
}

int scd_reset(scd_ctx* c, void* st) {
  if (!c || !st || !aligned(st, kAlign)) return SCD_EINVAL;
  scd::ResetArgs a{};
  a.pos = field<int32_t>(c, st, SCD_F_POS);
  a.iter = field<int32_t>(c, st, SCD_F_ITER);
  a.X = field<int32_t>(c, st, SCD_F_X);
  a.age = field<int32_t>(c, st, SCD_F_AGE);
  a.out = field<int32_t>(c, st, SCD_F_OUT);
  a.accept_len = field<int32_t>(c, st, SCD_F_ACCEPT);
  a.verified = field<int32_t>(c, st, SCD_F_VERIFIED);
  a.flags = field<int32_t>(c, st, SCD_F_FLAGS);
  a.ticket = field<int32_t>(c, st, SCD_F_TICKET);
  a.phist = field<int32_t>(c, st, SCD_F_PHIST);
  a.B = c->cfg.B; a.L = c->cfg.L; a.N = c->cfg.N; a.n = c->n; a.seed = c->cfg.seed;
  return hip_rc(scd::launch_reset(a, c->stream));
}

int scd_lm_head(scd_ctx* c, const uint16_t* d_h, const uint16_t* d_W, float* d_z) {
  if (!c || !d_h || !d_W || !d_z) return SCD_EINVAL;
  if (c->cfg.d <= 0) return SCD_EINVAL;
  if (!aligned(d_h, 16) || !aligned(d_W, 16)) return SCD_EINVAL;
  scd::LmHeadArgs a{};
  a.h = d_h;
  a.W = d_W + static_cast<size_t>(c->cfg.v_lo) * c->cfg.d;
  a.z = d_z;
  a.B = c->cfg.B; a.C = c->C; a.L = c->cfg.L; a.N = c->cfg.N; a.d = c->cfg.d; a.n = c->n;
  a.lam = c->cfg.cfg_lambda;
  a.one_plus_lam = 1.0f + c->cfg.cfg_lambda;
  a.tau = c->cfg.temperature;
  return hip_rc(scd::launch_lm_head(a, c->stream));
}

}  // extern "C"

namespace {

// scd_select with the candidate scratch at `ws` (layout of the workspace: small_need bytes of
// per-row scalars, then the candidate lists)
int select_impl(scd_ctx* c, char* ws, const float* d_z, int32_t rows, float* d_thr, float* d_lse,
                int32_t* d_nkept) {
  if (!c || !d_z || rows < 0 || !d_thr || !d_lse || !d_nkept) return SCD_EINVAL;
  if (c->n <= scd::kRowKernelMaxN) {
    scd::RowArgs ra{};
    ra.alpha = 1.0f;
    ra.mode = scd::kRowSelectOnly;
    ra.z_cur = d_z; ra.thr = d_thr; ra.lse = d_lse; ra.nkept = d_nkept;
    ra.rows = rows;
    ra.B = c->cfg.B; ra.L = c->cfg.L; ra.N = c->cfg.N; ra.n = c->n; ra.top_k = c->cfg.top_k;
    ra.top_p24 = top_p24_of(c->cfg);
    if (rows <= c->cfg.B * c->cfg.L) ra.cand_base = ws + small_need(c->cfg);
    return hip_rc(scd::launch_row(ra, c->stream, c->row_lds));
  }
  scd::SelectArgs a{};
  a.z = d_z; a.thr = d_thr; a.lse = d_lse; a.nkept = d_nkept;
  a.rows = rows;
  a.B = c->cfg.B; a.L = c->cfg.L; a.N = c->cfg.N; a.n = c->n; a.top_k = c->cfg.top_k;
  return hip_rc(scd::launch_select(a, c->stream));
}

int couple_draft_impl(scd_ctx* c, char* w, const float* d_z_cur, const float* d_z_prev,
                      const int32_t* d_x, const uint8_t* d_fresh, const int32_t* d_pos0, int32_t iter,
                      int32_t* d_y, uint8_t* d_k) {
  if (!c || !d_z_cur || !d_z_prev || !d_x || !d_pos0 || !d_y || !d_k || iter < 0)
    return SCD_EINVAL;
  const int rows = c->cfg.B * c->cfg.L;
  const size_t seg = align_up(4 * static_cast<size_t>(rows));
  float* thr_c = reinterpret_cast<float*>(w);
  float* lse_c = reinterpret_cast<float*>(w + seg);
  int32_t* nk_c = reinterpret_cast<int32_t*>(w + 2 * seg);
  float* thr_p = reinterpret_cast<float*>(w + 3 * seg);
  float* lse_p = reinterpret_cast<float*>(w + 4 * seg);
  int32_t* nk_p = reinterpret_cast<int32_t*>(w + 5 * seg);
  if (int rc = select_impl(c, w, d_z_prev, rows, thr_p, lse_p, nk_p); rc != SCD_OK) return rc;
  if (c->n <= scd::kRowKernelMaxN) {
    scd::RowArgs ra{};
    ra.alpha = 1.0f;
    ra.mode = scd::kRowPlain;
    ra.z_cur = d_z_cur; ra.z_prev = d_z_prev;
    ra.thr = thr_c; ra.lse = lse_c; ra.nkept = nk_c;
    ra.thr_prev = thr_p; ra.lse_prev = lse_p;
    ra.x = d_x; ra.fresh = d_fresh; ra.pos = const_cast<int32_t*>(d_pos0);
    ra.iter_scalar = iter;
    ra.y = d_y; ra.k = d_k;
    ra.rows = rows;
    ra.B = c->cfg.B; ra.L = c->cfg.L; ra.N = c->cfg.N; ra.n = c->n; ra.top_k = c->cfg.top_k;
    ra.top_p24 = top_p24_of(c->cfg);
    ra.v_lo = c->cfg.v_lo; ra.seed = c->cfg.seed;
    ra.cand_base = w + small_need(c->cfg);
    return hip_rc(scd::launch_row(ra, c->stream, c->row_lds));
  }
  if (int rc = select_impl(c, w, d_z_cur, rows, thr_c, lse_c, nk_c); rc != SCD_OK) return rc;
  scd::MrsArgs a{};
  a.z_cur = d_z_cur; a.z_prev = d_z_prev;
  a.thr_cur = thr_c; a.lse_cur = lse_c; a.thr_prev = thr_p; a.lse_prev = lse_p;
  a.x = d_x; a.fresh = d_fresh; a.pos = d_pos0;
  a.iter_scalar = iter; a.ring = 0;
  a.y = d_y; a.k = d_k;
  a.B = c->cfg.B; a.L = c->cfg.L; a.N = c->cfg.N; a.n = c->n; a.seed = c->cfg.seed;
  return hip_rc(scd::launch_mrs(a, c->stream));
}

}  // namespace

extern "C" {

int scd_select(scd_ctx* c, const float* d_z, int32_t rows, float* d_thr, float* d_lse,
               int32_t* d_nkept) {
  if (!c) return SCD_EINVAL;
  return select_impl(c, static_cast<char*>(c->ws), d_z, rows, d_thr, d_lse, d_nkept);
}

int scd_couple_draft(scd_ctx* c, const float* d_z_cur, const float* d_z_prev, const int32_t* d_x,
                     const uint8_t* d_fresh, const int32_t* d_pos0, int32_t iter, int32_t* d_y,
                     uint8_t* d_k) {
  if (!c) return SCD_EINVAL;
  return couple_draft_impl(c, static_cast<char*>(c->ws), d_z_cur, d_z_prev, d_x, d_fresh, d_pos0, iter,
                           d_y, d_k);
}

int scd_couple_draft_static(scd_ctx* c, const float* d_z_cur, const float* d_z_prev, const int32_t* d_x,
                            const uint8_t* d_fresh, const int32_t* d_pos0, int32_t iter, int32_t* d_y,
                            uint8_t* d_k) {
  if (!c) return SCD_EINVAL;
  // what this configuration really uses of the workspace layout: the per-row scalars, and the
  // candidate lists only when its rows go through the slice kernel
  const bool cands = scd::row_uses_candidates(c->n, c->cfg.top_k);
  const size_t need = small_need(c->cfg) + (cands ? align_up(scd::row_candidate_bytes(c->cfg.B * c->cfg.L)) : 0);
  if (need > static_cast<size_t>(SCD_STATIC_SCRATCH_BYTES)) return SCD_ESCRATCH;
  void* base = nullptr;
  if (int rc = static_scratch(&base); rc != SCD_OK) return rc;
  // nothing in the scratch has to start at zero: the per-row scalars and, for every live row,
  // all slice counts / cuts the row kernel reads are written by the launches of this call first
  return couple_draft_impl(c, static_cast<char*>(base), d_z_cur, d_z_prev, d_x, d_fresh, d_pos0, iter,
                           d_y, d_k);
}

int scd_verify(scd_ctx* c, const uint8_t* d_k, const int32_t* d_y, const int32_t* d_pos0,
               int32_t* d_accept_len, int32_t* d_out) {
  if (!c || !d_k || !d_y || !d_pos0 || !d_accept_len || !d_out) return SCD_EINVAL;
  scd::CommitArgs a{};
  a.k = d_k; a.y = d_y; a.pos = const_cast<int32_t*>(d_pos0);
  a.accept_len = d_accept_len; a.out = d_out;
  a.slide = 0;
  a.B = c->cfg.B; a.L = c->cfg.L; a.N = c->cfg.N; a.n = c->n; a.v_lo = c->cfg.v_lo;
  a.seed = c->cfg.seed;
  return hip_rc(scd::launch_commit(a, c->stream));
}

int scd_step(scd_ctx* c, const uint16_t* d_h, const uint16_t* d_W, void* st) {
  if (!c || !d_h || !d_W || !st || !aligned(st, kAlign)) return SCD_EINVAL;
  if (c->cfg.d <= 0) return SCD_EINVAL;
  if (!aligned(d_h, 16) || !aligned(d_W, 16)) return SCD_EINVAL;
  scd::LmHeadArgs a{};
  a.h = d_h;
  a.W = d_W + static_cast<size_t>(c->cfg.v_lo) * c->cfg.d;
  a.z = field<float>(c, st, SCD_F_Z);
  a.pos = field<int32_t>(c, st, SCD_F_POS);
  a.iter = field<int32_t>(c, st, SCD_F_ITER);
  a.parity_stride = static_cast<size_t>(c->cfg.B) * c->cfg.L * c->n;
  a.B = c->cfg.B; a.C = c->C; a.L = c->cfg.L; a.N = c->cfg.N; a.d = c->cfg.d; a.n = c->n;
  a.lam = c->cfg.cfg_lambda;
  a.one_plus_lam = 1.0f + c->cfg.cfg_lambda;
  a.tau = c->cfg.temperature;
  // First half of the top-k selection inside the LM head's epilogue (per-tile candidate lists in
  // the workspace) when the kernel for this shape can do it and the lists are long enough: on
  // average a tile holds top_k / tiles of the row's top_k logits; demand twice that plus 8.
  int tiles = 0;
  if (scd::row_uses_candidates(c->n, c->cfg.top_k)) {
    const int t = scd::lm_head_tiles(a);
    if (t > 0 && 2L * c->cfg.top_k <= static_cast<long>(t) * (scd::kRowListCap / t - 8)) tiles = t;
  }
  if (tiles > 0) {
    scd::row_candidate_layout(static_cast<char*>(c->ws) + small_need(c->cfg), c->cfg.B * c->cfg.L, &a.cand,
                              &a.cand_cnt, &a.cand_cut);
    a.cand_cap = scd::kRowListCap / tiles;
    a.flags = field<int32_t>(c, st, SCD_F_FLAGS);
  }
  const bool timed = c->ev_start && c->ev_stop;
  if (hipError_t e = scd::launch_lm_head(a, c->stream, timed ? c->ev_start : nullptr, timed ? c->ev_stop : nullptr);
      e != hipSuccess)
    return SCD_EHIP;
  return run_tail(c, st, tiles);
}

int scd_set_lm_head_events(scd_ctx* c, void* ev_start, void* ev_stop) {
  if (!c || ((ev_start == nullptr) != (ev_stop == nullptr))) return SCD_EINVAL;
  c->ev_start = static_cast<hipEvent_t>(ev_start);
  c->ev_stop = static_cast<hipEvent_t>(ev_stop);
  return SCD_OK;
}

int scd_lm_head_kernel_name(scd_ctx* c, char* host_buf, size_t cap) {
  if (!c || !host_buf || cap == 0 || c->cfg.d <= 0) return SCD_EINVAL;
  scd::LmHeadArgs a{};
  a.B = c->cfg.B; a.C = c->C; a.L = c->cfg.L; a.d = c->cfg.d; a.n = c->n;
  const int len = scd::lm_head_kernel_name(a, host_buf, cap);
  return (len < 0 || static_cast<size_t>(len) >= cap) ? SCD_EINVAL : SCD_OK;
}

int scd_step_logits(scd_ctx* c, const float* d_z, void* st) {
  if (!c || !d_z || !st || !aligned(st, kAlign)) return SCD_EINVAL;
  scd::CopyInArgs a{};
  a.src = d_z;
  a.z = field<float>(c, st, SCD_F_Z);
  a.parity_stride = static_cast<size_t>(c->cfg.B) * c->cfg.L * c->n;
  a.pos = field<int32_t>(c, st, SCD_F_POS);
  a.iter = field<int32_t>(c, st, SCD_F_ITER);
  a.B = c->cfg.B; a.L = c->cfg.L; a.N = c->cfg.N; a.n = c->n;
  if (hipError_t e = scd::launch_copy_in(a, c->stream); e != hipSuccess) return SCD_EHIP;
  return run_tail(c, st);
}

int scd_status(scd_ctx* c, void* st, int32_t host_flags[4]) {
  if (!c || !st || !host_flags) return SCD_EINVAL;
  const int B = c->cfg.B;
  int32_t flags[4];
  if (hipMemcpyAsync(flags, field<int32_t>(c, st, SCD_F_FLAGS), sizeof(flags),
                     hipMemcpyDeviceToHost, c->stream) != hipSuccess)
    return SCD_EHIP;
  int32_t* hp = new (std::nothrow) int32_t[2 * static_cast<size_t>(B)];
  if (!hp) return SCD_EINVAL;
  hipError_t e = hipMemcpyAsync(hp, field<int32_t>(c, st, SCD_F_POS), 4 * static_cast<size_t>(B),
                                hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(hp + B, field<int32_t>(c, st, SCD_F_ITER), 4 * static_cast<size_t>(B),
                       hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) {
    delete[] hp;
    return SCD_EHIP;
  }
  int done = 1, tmax = 0;
  for (int b = 0; b < B; ++b) {
    if (hp[b] < c->cfg.N) done = 0;
    if (hp[B + b] > tmax) tmax = hp[B + b];
  }
  delete[] hp;
  host_flags[0] = flags[0];
  host_flags[1] = done;
  host_flags[2] = tmax;
  host_flags[3] = 0;
  return flags[0] ? SCD_ENUMERIC : SCD_OK;
}

const char* scd_strerror(int code) {
  switch (code) {
    case SCD_OK: return "ok";
    case SCD_EINVAL: return "invalid argument or configuration";
    case SCD_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SCD_EHIP: return "HIP runtime call or kernel launch failed";
    case SCD_ENUMERIC: return "a logit row had no finite value or contained NaN";
    case SCD_EUNSUPPORTED: return "not implemented in this build";
    case SCD_ESCRATCH:
      return "configuration needs more scratch than the library's static array (SCD_STATIC_SCRATCH_BYTES)";
    default: return "unknown error code";
  }
}

}  // extern "C"
