// Host-callable launchers of the gfx950 kernels behind the C ABI in
// include/scd.h.  Plain pointers and sizes only; every launcher enqueues on
// the given stream and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace scd {

// ---- LM head + CFG combine + temperature --------------------------------
struct LmHeadArgs {
  const uint16_t* h;    // bf16 [B, C, L, d]
  const uint16_t* W;    // bf16 [n, d]: first allowed row of the weight matrix
  float* z;             // fp32 [(2,) B, L, n]
  const int32_t* pos;   // [B] or null: row s is stored at ring slot (pos[b]+s) % L
  const int32_t* iter;  // [B] or null: store into half (iter[b] & 1) of z
  size_t parity_stride; // floats between the two halves of z
  int B, C, L, N, d, n;
  float lam, one_plus_lam, tau;
  // Optional (scd_step only, and only when lm_head_tiles() says the chosen kernel can): the
  // epilogue also emits, per window row and per 256-column tile, the tile's cand_cap largest
  // logits as (id, logit) pairs, their number and the cut below which nothing was emitted --
  // the input of the row kernel's candidate path, which then needs no slice kernel.  Layout as
  // row_candidate_layout() gives it; window row index = b * L + s.  All null / 0 => off.
  uint2* cand;
  uint32_t* cand_cnt;
  uint32_t* cand_cut;
  int cand_cap;         // pairs per (row, tile)
  int32_t* flags;       // numeric-fault bits (NaN logits are reported here), may be null
};
// ev_start / ev_stop (both or neither): events that take the kernel's own start and stop time
hipError_t launch_lm_head(const LmHeadArgs& a, hipStream_t s, hipEvent_t ev_start = nullptr,
                          hipEvent_t ev_stop = nullptr);
// Name (as a profiler prints it, without namespaces and arguments) of the kernel that
// launch_lm_head picks for these sizes (only B, C, L, d, n are read); snprintf semantics.
int lm_head_kernel_name(const LmHeadArgs& a, char* buf, size_t cap);
// Number of 256-column tiles per row if the kernel that launch_lm_head picks for these sizes can
// emit per-tile candidates, else 0 (only B, C, L, d, n are read).
int lm_head_tiles(const LmHeadArgs& a);

// ---- top-k threshold + softmax normaliser -------------------------------
struct SelectArgs {
  const float* z;       // rows of n floats
  size_t parity_stride; // floats between the two halves (ring mode)
  const int32_t* pos;   // ring mode: [B]; null => plain mode, row r at z + r*n
  const int32_t* iter;  // ring mode: [B]
  float* thr;           // plain: [rows]; ring: [2, B, L]
  float* lse;
  int32_t* nkept;
  int32_t* flags;       // numeric-fault bits (may be null)
  int rows;             // plain mode: number of rows; ring mode: B*L
  int B, L, N, n, top_k;
};
hipError_t launch_select(const SelectArgs& a, hipStream_t s);

// ---- vectorised Modified Rejection Sampling ------------------------------
struct MrsArgs {
  const float* z_cur;   // plain: [B, L, n]; ring: base of [2, B, L, n]
  const float* z_prev;  // plain: [B, L, n]; ring: unused
  size_t parity_stride; // ring: floats between the halves of z
  const float* thr_cur; // plain: [B*L];   ring: base of [2, B, L]
  const float* lse_cur;
  const float* thr_prev;
  const float* lse_prev;
  const int32_t* x;     // plain: [B, L] window order; ring: [B, L] by slot
  const uint8_t* fresh; // plain: [B, L] or null
  const int32_t* age;   // ring: [B, L] by slot (fresh <=> age == 0)
  const int32_t* pos;   // [B]
  const int32_t* iter;  // ring: [B]; plain: null (iter_scalar is used)
  int iter_scalar;
  int ring;
  int32_t* y;           // [B, L] window order
  uint8_t* k;           // [B, L] window order
  float* px;            // [B, L] or null
  float* qx;            // [B, L] or null
  int B, L, N, n;
  uint64_t seed;
};
hipError_t launch_mrs(const MrsArgs& a, hipStream_t s);

// ---- fused row kernel: select + softmax + MRS (+ commit by the last arriver) --
enum { kRowSelectOnly = 0, kRowPlain = 1, kRowRing = 2 };
constexpr int kRowKernelMaxN = 65536;   // the LDS copy of the key prefixes must fit
struct RowArgs {
  int mode;
  const float* z_cur;    // select-only: [rows, n]; plain: [B, L, n]; ring: base of [2, B, L, n]
  const float* z_prev;   // plain: [B, L, n]
  size_t parity_stride;  // ring: floats between the halves of z
  float* thr;            // select-only / plain: [rows]; ring: [2, B, L] (both parities)
  float* lse;
  int32_t* nkept;
  const float* thr_prev; // plain: [B*L]
  const float* lse_prev;
  const int32_t* x;      // plain: [B, L] window order; ring: [B, L] by slot (also written)
  const uint8_t* fresh;  // plain: [B, L] or null
  const int32_t* age;    // ring: [B, L] by slot
  int32_t* pos;          // [B]
  int32_t* iter;         // ring: [B]
  int iter_scalar;       // plain
  int32_t* y;            // [B, L] window order
  uint8_t* k;
  float* px;             // [B, L] or null
  float* qx;
  int32_t* flags;        // numeric-fault bits or null
  // ring mode: state updated by the last workgroup of each sequence
  int32_t* ticket;       // [B], zero between launches
  int32_t* X;            // [B, L] by slot
  int32_t* age_w;        // [B, L] by slot
  int32_t* verified;     // [B]
  int32_t* accept_len;   // [B]
  int32_t* out;          // [B, N]
  // Gumbel-sharing coupling: with gumbel != 0 and g non-null every row also draws
  // g = argmax_v(log p_v + G_v(position)) and the survivors' next drafts are g, not y
  int gumbel;
  // alpha-coupling: with alpha < 1 a row whose switch uniform exceeds alpha draws its redraft
  // independently from p (same race, noise keyed by the iteration too) and reports it in g
  float alpha;           // 1 => never
  int32_t* g;            // [B, L] window order; -1 where the row made no such draw
  int rows;              // select-only: rows; else B*L
  int B, L, N, n, top_k, v_lo;
  // nucleus filter: round(top_p * 2^24), 0 => off.  Applied to what top-k left.
  uint32_t top_p24;
  // per-position statistics (ring mode only; all three null => off)
  float* diag;           // [B, L, 4] window order: sum min(p,q), sum p q, sum p^2, sum q^2
  float* s2;             // [2, B, L] sum p^2 per parity and slot
  int32_t* hamm;         // [B, 6]    (differing, compared) drafts 1, 2, 3 iterations apart
  int32_t* xhist;        // [3, B, L] drafts at the start of the last three iterations, by ring slot
  int32_t* phist;        // [3, B]    window start of those iterations (far negative: none)
  uint64_t seed;
  // scratch for the slice kernel (rows longer than 8192 ids): row_candidate_bytes(rows)
  // bytes of device memory, 256-byte aligned, or null (then rows are processed whole)
  void* cand_base;
  // tiles > 0: the LM head's epilogue has already filled the candidate scratch with `tiles`
  // lists of kRowListCap / tiles pairs per row (launch_row then skips the slice kernel)
  int tiles;
  uint32_t cand_recip;   // set by launch_row: ceil(2^32 / pairs per candidate list)
  uint2* cand;           // set by launch_row
  uint32_t* cand_cnt;    // set by launch_row
  uint32_t* cand_cut;    // set by launch_row
};
size_t row_candidate_bytes(int rows);
// Where the candidate scratch (row_candidate_bytes(rows) bytes at base) keeps its parts: per row
// kRowListCap (id, logit) pairs, then kRowMaxTiles counts, then kRowMaxTiles cuts.
constexpr int kRowListCap = 6144;
constexpr int kRowMaxTiles = 256;
void row_candidate_layout(void* base, int rows, uint2** cand, uint32_t** cnt, uint32_t** cut);
// whether launch_row, given scratch, runs the slice kernel for rows of n ids under this top-k
bool row_uses_candidates(int n, int top_k);
// lds_configured: the caller's record (two words per context, initially 0) that the dynamic-LDS
// limit of the row kernels has been set on its device; null => set it on every launch
hipError_t launch_row(const RowArgs& a, hipStream_t s, size_t* lds_configured);
// The same kernels built with 512 threads per row for rows of at most kRowBatchedMaxN ids (two
// workgroups per compute unit); launch_row hands over to it when there are more rows than
// compute units.  lds_configured: one word.
constexpr int kRowBatchedMaxN = 8192;
hipError_t launch_row_batched(const RowArgs& a, hipStream_t s, size_t* lds_configured);

// ---- first rejection, emit, slide -----------------------------------------
struct CommitArgs {
  const uint8_t* k;     // [B, L]
  const int32_t* y;     // [B, L]
  int32_t* pos;         // [B]  (read; advanced only when slide != 0)
  int32_t* iter;        // [B]  (slide only)
  int32_t* X;           // [B, L] ring (slide only)
  int32_t* age;         // [B, L] ring (slide only)
  int32_t* verified;    // [B] (slide only)
  int32_t* accept_len;  // [B]
  int32_t* out;         // [B, N]
  int slide;
  int B, L, N, n, v_lo;
  uint64_t seed;
};
hipError_t launch_commit(const CommitArgs& a, hipStream_t s);

// ---- state initialisation / logits copy-in --------------------------------
struct ResetArgs {
  int32_t* pos; int32_t* iter; int32_t* X; int32_t* age; int32_t* out; int32_t* accept_len;
  int32_t* verified; int32_t* flags; int32_t* ticket;
  int32_t* phist;        // [3, B] -> far negative
  int B, L, N, n;
  uint64_t seed;
};
hipError_t launch_reset(const ResetArgs& a, hipStream_t s);

struct CopyInArgs {
  const float* src;     // [B, L, n] window order
  float* z;             // [2, B, L, n]
  size_t parity_stride;
  const int32_t* pos; const int32_t* iter;
  int B, L, N, n;
};
hipError_t launch_copy_in(const CopyInArgs& a, hipStream_t s);

}  // namespace scd
