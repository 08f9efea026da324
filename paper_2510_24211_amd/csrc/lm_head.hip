// LM head of the window ("Evaluate" step of the SCD / SJD algorithms):
//   logit[m, v] = sum_k h[m, k] * W[v, k]      bf16 x bf16 -> fp32 (MFMA)
// with the first logit processors fused into the epilogue (Sec. 4.3 defines
// p^(t) after post-processing; Sec. 5.1 gives the guidance mix):
//   z = fl(fl((1+lambda) * c) - fl(lambda * u)),   z <- z / tau
// Only the allowed vocabulary rows of W are streamed (the mask to -inf of the
// other ids is realised by never forming their columns).
//
// gfx950 mapping.  The contraction is skinny: M = B*C*L rows (32..1024) against
// n = |allowed| columns (8k..64k) over d = 1k..4k, i.e. a stream over W that
// must keep many bytes in flight per CU and must not stall on barriers.
//   * A wavefront owns 32 vocabulary rows of W.  It fetches its own slab with
//     coalesced 16-byte loads (8 lanes cover one 128-byte row segment), D k-tiles
//     ahead in registers, parks a tile in a wavefront-PRIVATE LDS region (pitch
//     144 bytes against bank conflicts) and reads it back in the operand layout
//     of v_mfma_f32_32x32x16_bf16 (lane l: row l%32, k-group l/32, 8 consecutive
//     k).  Private staging needs no workgroup barrier, so the wavefronts of a
//     workgroup drift apart and the W stream never drains.
//   * The NW wavefronts of a workgroup take NW x 32 neighbouring columns and
//     SHARE the h tile through LDS (double buffered, loaded two tiles ahead, one
//     barrier per h tile): h comes out of L2 once per workgroup, not per wavefront.
//   * The accumulators of a wavefront are RBW "row blocks" x C tiles: a row block
//     is 32 window positions of one sequence, its cond and uncond tiles live in
//     the SAME lanes, so the guidance mix needs no data movement.
//   * Every workgroup walks k cyclically from its own starting tile: rows of W
//     are d*2 bytes apart, and without the rotation all wavefronts of the chip
//     ask for the same address bits at the same time and camp on a few channels.
//   * Narrow vocabularies give too few 128-column tiles to fill 256 CUs.  They use
//     lm_head_splitk_kernel: a workgroup owns 32 columns, its KS wavefronts take a
//     1/KS part of k each, stage their own h tiles privately as well (no barrier in
//     the loop), and their partial sums are added in wavefront order through LDS at
//     the end (a fixed order: deterministic).
#include "scd_device.h"
#include "scd_kernels.h"

#include <hip/hip_ext.h>

#include <stdio.h>

namespace scd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16-byte register value; a native vector (the HIP struct type is copied with memcpy,
// which keeps arrays of it in scratch memory)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One 16-byte piece of W.  NT: non-temporal load -- the line is not kept in the caches it
// passes.  A slice of W that cannot stay in the 256 MB memory-side cache until the next step
// only evicts what could (the hidden rows in L2, the logits): streaming it past the caches
// took the full-vocabulary LM head from 96 to 87 us.  A slice that fits (C2: 67 MB) is served
// from that cache step after step and loses 3 us when loaded this way.
template <bool NT>
__device__ __forceinline__ u32x4 load_w(const u32x4* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

constexpr int BK = 64;          // k elements per W tile (128 bytes per row)
constexpr int PITCH = BK + 8;   // LDS row pitch in bf16 elements (144 bytes)

struct TrueT { static constexpr bool value = true; };
struct FalseT { static constexpr bool value = false; };
template <int N>
struct IntT { static constexpr int value = N; };

__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }
// Also a boundary for the machine scheduler, which otherwise treats loads of never-written
// global memory as freely movable and may sink a prefetch down to its use.
__device__ __forceinline__ void hard_fence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// Which rows of W (= columns of z) a workgroup works on.  Workgroup ids go round robin over
// the 8 XCDs.  Read bandwidth on this chip is markedly higher when every XCD keeps to its own
// residue class of 128 KB address blocks (block number mod 8 == XCD; measured: 5.8 against
// 4.5 TB/s for the same bytes otherwise).  So when a row of W divides 128 KB, rows are dealt
// out in groups of G = 128 KB / row bytes consecutive rows: group g (rows g*G .. g*G+G-1)
// belongs to XCD (g + rot) mod 8, where rot places group 0 in the class of the block that
// holds most of it, and the workgroups of an XCD take its rows in order.  Otherwise
// (gshift < 0) workgroup tile t simply owns rows t * BN .. t * BN + BN - 1.
struct RowMap {
  int gshift;   // log2 G, or -1
  int rot;      // residue class of group 0
};
// Row of W for position `local` of workgroup tile jt of XCD xcd; >= n: no such row.  Rows grow
// with `local`.
__device__ __forceinline__ int mapped_row(const RowMap& m, int xcd, int jt, int BN, int local) {
  if (m.gshift < 0) return (jt * 8 + xcd) * BN + local;
  const int idx = jt * BN + local;                        // idx-th row owned by this XCD
  const int g = ((idx >> m.gshift) << 3) + ((xcd - m.rot) & 7);
  return (g << m.gshift) + (idx & ((1 << m.gshift) - 1));
}

template <int RBW, int C, int NWV>
struct Cfg {
  static constexpr int NW = NWV;                  // wavefronts per workgroup
  static constexpr int THREADS = NW * 64;
  static constexpr int NBLK = RBW * C;            // accumulator tiles per wavefront
  static constexpr int HROWS = NBLK * 32;         // h rows per tile
  static constexpr int D = 4;                     // W tiles in flight per wavefront (registers)
  static constexpr int DH = 2;                    // h tiles in flight (registers)
  static constexpr int HT = NBLK <= 2 ? 2 : 1;    // W tiles per shared h tile
  static constexpr int BKH = BK * HT;
  static constexpr int PITCH_H = BKH + 8;
  static constexpr int BN = NW * 32;              // columns per workgroup
  static constexpr int W_LDS = NW * 32 * PITCH;   // elements
  static constexpr int H_LDS = 2 * HROWS * PITCH_H;
  static constexpr int LDS_BYTES = (W_LDS + H_LDS) * 2;
};

// Where the 32 window positions of row block rb (sequence b, positions sbase..sbase+31 of
// its window) are stored: ring slot (pos[b] + s) % L of half iter[b] & 1 when the decode
// state is given, row s otherwise.
struct RowBlockDst {
  float* zb;
  int b, sbase, p0, live;
  int lmask;    // L - 1 if L is a power of two (ring slot by masking), else -1 (by division)
};
__device__ __forceinline__ RowBlockDst row_block_dst(const LmHeadArgs& a, int rb, int nLb) {
  RowBlockDst r;
  r.b = rb / nLb;
  r.sbase = (rb % nLb) * 32;
  r.p0 = 0;
  r.live = a.L;
  r.zb = a.z;
  if (a.pos) {
    r.p0 = a.pos[r.b];
    r.live = min(a.L, a.N - r.p0);
  }
  if (a.iter) r.zb += static_cast<size_t>(a.iter[r.b] & 1) * a.parity_stride;
  r.lmask = (a.L & (a.L - 1)) == 0 ? a.L - 1 : -1;
  return r;
}
// Ring slot of window position s (an integer division per logit otherwise: 16 of them per lane)
__device__ __forceinline__ int ring_slot(const LmHeadArgs& a, const RowBlockDst& r, int s) {
  if (!a.pos) return s;
  return r.lmask >= 0 ? ((r.p0 + s) & r.lmask) : (r.p0 + s) % a.L;
}

// Guidance mix and temperature of one logit (cond sum c, uncond sum u): three fp32 roundings
// for the mix, one for the division (skipped for tau = 1, where it changes nothing).
template <int C>
__device__ __forceinline__ float processed_logit(const LmHeadArgs& a, float c, float u) {
  float z = c;
  if (C == 2) z = __fsub_rn(__fmul_rn(a.one_plus_lam, c), __fmul_rn(a.lam, u));
  return a.tau == 1.0f ? z : __fdiv_rn(z, a.tau);
}
// Stores processed logit z of window position s and allowed id v.
__device__ __forceinline__ void store_z(const LmHeadArgs& a, const RowBlockDst& r, int s, int v, float z) {
  if (s >= r.live) return;
  // the sequence's part of the address is uniform (scalar unit); slot * n + v fits 32 bits
  // (L * n < 2^31 is checked when the context is created)
  float* const zseq = r.zb + static_cast<size_t>(r.b) * a.L * a.n;
  zseq[static_cast<uint32_t>(ring_slot(a, r, s)) * static_cast<uint32_t>(a.n) + static_cast<uint32_t>(v)] = z;
}
template <int C>
__device__ __forceinline__ void store_logit(const LmHeadArgs& a, const RowBlockDst& r, int s, int v,
                                            float c, float u) {
  store_z(a, r, s, v, processed_logit<C>(a, c, u));
}

// Epilogue of a wavefront that holds whole sums.  Element j of lane (ln, lg) is row
// (j/4)*8 + lg*4 + j%4, column ln of the 32x32 tile.  zout takes the processed logits.
// rbd[rbw]: where row block rb0 + rbw goes (fetched at kernel start: window start and iteration
// parity come from memory, and the epilogue should not begin with that round trip).
template <int RBW, int C>
__device__ __forceinline__ void epilogue(const LmHeadArgs& a, const f32x16 (&acc)[RBW * C], int nRB, int rb0,
                                         const RowBlockDst (&rbd)[RBW], int v, int lg, float (&zout)[RBW][16]) {
#pragma unroll
  for (int rbw = 0; rbw < RBW; ++rbw)
#pragma unroll
    for (int j = 0; j < 16; ++j) zout[rbw][j] = processed_logit<C>(a, acc[rbw * C][j], acc[rbw * C + C - 1][j]);
  if (v >= a.n) return;
#pragma unroll
  for (int rbw = 0; rbw < RBW; ++rbw) {
    if (rb0 + rbw >= nRB) break;
    const RowBlockDst& r = rbd[rbw];
#pragma unroll
    for (int j = 0; j < 16; ++j)
      store_z(a, r, r.sbase + (j >> 2) * 8 + lg * 4 + (j & 3), v, zout[rbw][j]);
  }
}

// ---- per-tile top-k candidates (first half of the top-k selection, fused into the epilogue) ----
// A workgroup that owns 256 neighbouring columns parks its processed logits in LDS as a tile
// zt[row][kTilePitch] and every wavefront then reduces some rows of it: of the row's 256
// logits it emits the `cap` largest as (id, logit) pairs in a FIXED order (lane, then column),
// their number, and the cut = the smallest emitted logit (as a key): every logit of the tile row
// that was not emitted lies strictly below it.  The row kernel selects the K-th largest among the
// emitted logits of all tiles and accepts it only if it is not below any tile's cut (then no
// logit that was not emitted can reach it): exact, and certified per row.
//   The emitted set is found by bisection, not on the logits themselves but on a monotone
// 12-bit fixed-point image of them, q = trunc(1 + (z - min) * 4095 / (max - min)) (equal q:
// both emitted or neither).  Then the halving runs on the scalar unit (integer bounds in
// SGPRs); the vector unit only compares, one instruction per logit and halving, and wave
// ballots + population counts do the counting.  13 steps end exactly at the smallest q whose
// upper set holds at most `cap` logits.  If more than `cap` logits share the top q (massive
// ties, or a non-finite logit, which collapses the image) the tile reports an overflowing count
// and the row kernel reads the row whole.
constexpr int kTileCols = 256;
constexpr int kTilePitch = kTileCols + 8;   // floats; rows 4 apart fall into disjoint banks
constexpr int kTileQBits = 12;

// Rows q0 .. q0 + 3 of the tile; wrow[i] = window row index (b * L + s) of tile row q0 + i, or -1
// if it is not a live window row; v0 = id of the tile's first column; tile / T = its index and the
// number of tiles per row.  Uniform over the wavefront.
__device__ __forceinline__ void tile_candidates4(const LmHeadArgs& a, const float* zt, int lane, int q0,
                                                 const int (&wrow)[4], int v0, int tile, int T) {
  const int cap = a.cand_cap;
  const int nvalid = min(kTileCols, a.n - v0);           // columns of this tile that exist
  constexpr uint32_t QMAX = (1u << kTileQBits) - 1u;
  const bool ragged = nvalid < kTileCols;                // only the last tile of a row
  bool ok[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) ok[e] = 4 * lane + e < nvalid;
  float v[4][4];
  uint32_t q[4][4];                                      // 0 .. QMAX + 2; 0 also for a column that does not exist
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 t = *reinterpret_cast<const float4*>(&zt[(q0 + i) * kTilePitch + 4 * lane]);
    v[i][0] = t.x; v[i][1] = t.y; v[i][2] = t.z; v[i][3] = t.w;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float mx, mn;
    if (!ragged) {
      mx = fmaxf(fmaxf(v[i][0], v[i][1]), fmaxf(v[i][2], v[i][3]));
      mn = fminf(fminf(v[i][0], v[i][1]), fminf(v[i][2], v[i][3]));
    } else {
      mx = -INFINITY;
      mn = INFINITY;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[i][e] = ok[e] ? v[i][e] : 0.f;
        mx = ok[e] ? fmaxf(mx, v[i][e]) : mx;
        mn = ok[e] ? fminf(mn, v[i][e]) : mn;
      }
    }
    // a NaN (or +inf next to -inf) among the four poisons their sum
    const float sum4 = (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    if (sum4 != sum4 && a.flags && wrow[i] >= 0) atomicOr(a.flags, 1);
    const float hi = wave_max_f32(mx), lo = wave_min_f32(mn);
    // q = trunc(1 + (z - lo) * scale), one fused multiply-add per logit: monotone in z.  For
    // non-finite logits scale / shift degenerate, every q collapses and the tile row reports an
    // overflow below.
    const float scale = hi > lo ? __fdiv_rn(static_cast<float>(QMAX), hi - lo) : 0.f;
    const float shift = 1.0f - lo * scale;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      q[i][e] = static_cast<uint32_t>(fmaxf(__fmaf_rn(v[i][e], scale, shift), 0.f));
      if (ragged) q[i][e] = ok[e] ? q[i][e] : 0u;
    }
  }
  // The largest c with #(q >= c) > cap, built bit by bit from the top (q < 2^(kTileQBits + 1)); the
  // cut is c + 1.  One scalar unit serves the whole compute unit, so the loop is kept to ten scalar
  // operations per row and step.  #(q >= 0) is the whole tile row: above cap unless the row has at
  // most cap columns, which is handled apart.
  uint32_t cq[4] = {0u, 0u, 0u, 0u};
#pragma unroll 1
  for (uint32_t bit = 1u << kTileQBits; bit != 0u; bit >>= 1) {
    // the four rows side by side: all compares first, so that the scalar unit's population
    // counts do not each wait for a compare of their own
    unsigned long long m[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) m[i][e] = __builtin_amdgcn_ballot_w64(q[i][e] >= cq[i] + bit);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = __builtin_popcountll(m[i][0]) + __builtin_popcountll(m[i][1]) +
                    __builtin_popcountll(m[i][2]) + __builtin_popcountll(m[i][3]);
      cq[i] = n > cap ? cq[i] + bit : cq[i];
    }
  }
  const unsigned long long below = (1ull << lane) - 1ull;        // lanes before this one
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (wrow[i] < 0) continue;                           // uniform
    const bool all = nvalid <= cap;                      // the whole tile row is emitted: cut 0
    const uint32_t cutq = all ? 0u : cq[i] + 1u;
    // emitted logits in the fixed order (column within the lane, then lane)
    bool take[4];
    unsigned long long tm[4];
    float vmin = INFINITY;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      take[e] = q[i][e] >= cutq && (!ragged || ok[e]);
      tm[e] = __builtin_amdgcn_ballot_w64(take[e]);
      vmin = take[e] ? fminf(vmin, v[i][e]) : vmin;
    }
    const int c0 = __builtin_popcountll(tm[0]), c1 = __builtin_popcountll(tm[1]),
              c2 = __builtin_popcountll(tm[2]), c3 = __builtin_popcountll(tm[3]);
    const int total = c0 + c1 + c2 + c3;
    const int base[4] = {0, c0, c0 + c1, c0 + c1 + c2};
    vmin = wave_min_f32(vmin);                           // smallest emitted logit (NaNs are never smallest)
    const size_t slot = static_cast<size_t>(wrow[i]) * T + tile;
    const bool fits = total > 0 && total <= cap;         // nothing emitted: more than cap tie at the top
    if (fits) {
      uint2* dst = a.cand + (static_cast<size_t>(wrow[i]) * kRowListCap + static_cast<size_t>(tile) * cap);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (take[e])
          dst[base[e] + __builtin_popcountll(tm[e] & below)] =
              make_uint2(static_cast<uint32_t>(v0 + 4 * lane + e), __float_as_uint(v[i][e]));
    }
    if (lane == 0) {
      a.cand_cnt[slot] = fits ? static_cast<uint32_t>(total) : static_cast<uint32_t>(cap) + 1u;   // > cap: overflow
      a.cand_cut[slot] = all ? 0u : zkey(vmin);
    }
  }
}

template <int RBW, int C, int NWV, bool NT>
__global__ __launch_bounds__((Cfg<RBW, C, NWV>::THREADS)) void lm_head_kernel(
    const LmHeadArgs a, const int nLb, const int nRB, const int VT, const int MT, const RowMap rm) {
  using K = Cfg<RBW, C, NWV>;
  constexpr int NBLK = K::NBLK, HROWS = K::HROWS, D = K::D, DH = K::DH, HT = K::HT;
  constexpr int THREADS = K::THREADS;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[K::LDS_BYTES];
  uint16_t* const Ws_all = reinterpret_cast<uint16_t*>(lds_raw);
  uint16_t* const Hs_all = Ws_all + K::W_LDS;

  // Workgroups with consecutive ids land on different XCDs (round robin over 8).  The
  // MT row-block tiles that share one slab of W get ids 8 apart, i.e. the same XCD and
  // the same L2.
  const int id = blockIdx.x;
  const int xcd = id % 8, jt = id / (8 * MT);
  const int vt = jt * 8 + xcd;
  const int mt = (id / 8) % MT;
  if (mapped_row(rm, xcd, jt, Cfg<RBW, C, NWV>::BN, 0) >= a.n) return;   // no row left for this tile
  const int rb0 = mt * RBW;
  RowBlockDst rbd[RBW];
#pragma unroll
  for (int rbw = 0; rbw < RBW; ++rbw) rbd[rbw] = row_block_dst(a, min(rb0 + rbw, nRB - 1), nLb);

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int ln = lane & 31;     // row (A) / column (B) inside a 32x32 tile
  const int lg = lane >> 5;     // k-group
  const int chunk = lane & 7;   // 16-byte chunk inside a 128-byte row segment
  const int lrow = lane >> 3;   // 0..7

  const int d = a.d;
  const int KT = (d + BK - 1) / BK;
  const int ntiles = KT;
  const int ntiles_pad = (ntiles + D - 1) / D * D;
  // Row tiles that share a slab of W, and column tiles that share the same h rows, read the same
  // bytes; with several row tiles (MT > 1: the h rows no longer fit one L2 beside the W stream)
  // all workgroups of an XCD therefore start at the same k, so that they meet in L2 (C3: 86 -> 82 us).
  const int rot = (MT > 1 ? xcd * 5 : vt * 5) % ntiles_pad;
  // logical tile t -> k-tile index; `valid` is false for the padding tiles of the rotation
  // and for prefetches past the end.  Loads are NEVER predicated (a predicated load is a
  // branch, and branches keep the scheduler from batching the loads): an invalid tile reads
  // tile 0 of W (finite weights) against an h tile that is forced to zero.
  auto ktile = [&](int t, bool& valid) {
    int r = t + rot;
    if (r >= ntiles_pad) r -= ntiles_pad;
    valid = t < ntiles_pad && r < ntiles;
    return valid ? r : 0;
  };

  uint16_t* const Ws = Ws_all + wave * 32 * PITCH;          // private W staging

  // ---- W: coalesced private loads, D tiles ahead -----------------------------------
  // 32-bit byte offsets from the (uniform) base; rows past the end are clamped to the last
  // row (their columns are never stored), k past the end to the last 16-byte chunk.
  const char* const Wb = reinterpret_cast<const char*>(a.W);
  uint32_t woff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = mapped_row(rm, xcd, jt, K::BN, wave * 32 + lrow + 8 * i);
    woff[i] = static_cast<uint32_t>(min(v, a.n - 1)) * static_cast<uint32_t>(d) * 2u;
  }
  const uint32_t kclamp = static_cast<uint32_t>(d - 8) * 2u;
  u32x4 wreg[D][4];
  auto wload = [&](int slot, int t) {       // logical tile index t
    bool valid;
    const int kt = ktile(t, valid);
    const uint32_t kb = min(static_cast<uint32_t>(kt * BK + chunk * 8) * 2u, kclamp);
#pragma unroll
    for (int i = 0; i < 4; ++i) wreg[slot][i] = load_w<NT>(reinterpret_cast<const u32x4*>(Wb + (woff[i] + kb)));
  };
  auto wstore = [&](int slot) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<u32x4*>(&Ws[(lrow + 8 * i) * PITCH + chunk * 8]) = wreg[slot][i];
  };

  // ---- h: shared tile, BKH = HT * 64 wide --------------------------------------------
  constexpr int CH = K::BKH / 8;                 // 16-byte chunks per h row
  constexpr int CHW = BK / 8;                    // 16-byte chunks per W tile width
  constexpr int RPP = THREADS / CH;              // rows covered per pass of the workgroup
  constexpr int HL = HROWS / RPP;                // loads per thread per h tile
  static_assert(HROWS % RPP == 0, "h tile must divide over the workgroup");
  const int hchunk = tid % CH, hr0 = tid / CH;
  const char* const Hb = reinterpret_cast<const char*>(a.h);
  uint32_t hoff[HL];
  bool hok[HL];
#pragma unroll
  for (int i = 0; i < HL; ++i) {
    const int rr = hr0 + RPP * i;                // tile row 0..HROWS-1
    const int blk = rr >> 5, r = rr & 31;
    const int rb = rb0 + blk / C, c = blk % C;
    const int b = rb / nLb, s = (rb % nLb) * 32 + r;
    hok[i] = rb < nRB && s < a.L;
    hoff[i] = hok[i] ? static_cast<uint32_t>((b * C + c) * a.L + s) * static_cast<uint32_t>(d) * 2u : 0u;
  }
  u32x4 hreg[DH][HL];
  bool hkok[DH];
  // logical h tile st = logical W tiles st*HT .. st*HT+HT-1; after the rotation these
  // need not be neighbours in k (wrap-around), so every 64-wide part is placed on its own.
  // Loaded unconditionally from a clamped address, then zeroed where the row or k is not real.
  auto hload = [&](int slot, int st) {
    bool valid;
    const int kt = ktile(st * HT + hchunk / CHW, valid);
    const int k = kt * BK + (hchunk % CHW) * 8;
    const bool kok = valid && k < d;
    const uint32_t kb = min(static_cast<uint32_t>(k) * 2u, kclamp);
#pragma unroll
    for (int i = 0; i < HL; ++i) hreg[slot][i] = *reinterpret_cast<const u32x4*>(Hb + (hoff[i] + kb));
    hkok[slot] = kok;
  };
  // the zeroing waits for the load, so it happens here, when the tile moves to LDS
  auto hstore = [&](int slot, int buf) {
    uint16_t* dst = Hs_all + buf * HROWS * K::PITCH_H;
#pragma unroll
    for (int i = 0; i < HL; ++i) {
      const u32x4 t4 = hreg[slot][i];
      const bool keep = hok[i] && hkok[slot];
      *reinterpret_cast<u32x4*>(&dst[(hr0 + RPP * i) * K::PITCH_H + hchunk * 8]) =
          (keep ? t4 : u32x4{0u, 0u, 0u, 0u});
    }
  };

  f32x16 acc[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  // MFMAs of one W tile against h tile `Hs_tile` at column offset koff.  The operands of
  // k-step kk + 1 are read from LDS before the MFMAs of k-step kk are issued, so that the
  // matrix pipe does not wait for an LDS round trip per instruction.
  auto compute = [&](const uint16_t* Hs_tile, int koff) {
    constexpr int KK = BK / 16;
    u32x4 bq[2], aq[2][NBLK];
    auto fetch = [&](int buf, int kk) {
      bq[buf] = *reinterpret_cast<const u32x4*>(&Ws[ln * PITCH + kk * 16 + lg * 8]);
#pragma unroll
      for (int i = 0; i < NBLK; ++i)
        aq[buf][i] = *reinterpret_cast<const u32x4*>(
            &Hs_tile[(i * 32 + ln) * K::PITCH_H + koff + kk * 16 + lg * 8]);
    };
    fetch(0, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + 1 < KK) fetch((kk + 1) & 1, kk + 1);
      const bf16x8 bfrag = __builtin_bit_cast(bf16x8, bq[kk & 1]);
#pragma unroll
      for (int i = 0; i < NBLK; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aq[kk & 1][i]),
                                                         bfrag, acc[i], 0, 0, 0);
      if (kk + 1 < KK) {                       // keep that order: reads of kk + 1, MFMAs of kk
        __builtin_amdgcn_sched_group_barrier(0x100, NBLK + 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NBLK, 0);
      }
    }
  };

  // h tile st travels: registers (stage st % 2, loaded at the end of h tile st - 3), LDS
  // buffer st % 2 (moved at the end of h tile st - 1), consumed during h tile st.  One
  // barrier per h tile: it publishes the moved tile and ends the reads of the buffer that
  // the next move overwrites.
  static_assert(D % (2 * HT) == 0, "register stages of h must be static in the unrolled body");
#pragma unroll
  for (int j = 0; j < D; ++j) wload(j, j);
  hload(0, 0);
  hstore(0, 0);
  hload(1, 1);
  hload(0, 2);
  __syncthreads();
  // One pass over D tiles.  The last pass (PF false) issues no load that would fall past
  // the end: such a load would fetch real bytes a second time.
  auto body = [&](int t0, auto pf) {
    constexpr bool PF = decltype(pf)::value;
#pragma unroll
    for (int j = 0; j < D; ++j) {
      const int t = t0 + j;
      const int st = t / HT;
      const int stage = (j / HT) & 1;            // == st & 1 because t0 / HT is even
      compiler_fence();
      wstore(j);
      if (PF) wload(j, t + D);
      compiler_fence();
      compute(Hs_all + stage * HROWS * K::PITCH_H, (j % HT) * BK);
      compiler_fence();
      if (j % HT == HT - 1 && (PF || j / HT + 1 < D / HT)) {
        hstore(stage ^ 1, stage ^ 1);            // h tile st + 1 -> the other LDS buffer
        if (PF || j / HT + 3 < D / HT) hload(stage ^ 1, st + 3);
        __syncthreads();
      }
    }
  };
  for (int t0 = 0; t0 < ntiles_pad - D; t0 += D) body(t0, TrueT{});
  body(ntiles_pad - D, FalseT{});

  float zv[RBW][16];
  epilogue<RBW, C>(a, acc, nRB, rb0, rbd, mapped_row(rm, xcd, jt, K::BN, wave * 32 + ln), lg, zv);

  if constexpr (RBW == 1 && NWV == 8) {
    // ---- per-tile candidates for the row kernel (a.cand is uniform) --------------------------
    static_assert(K::BN == kTileCols && K::LDS_BYTES >= 32 * kTilePitch * 4, "logit tile must fit");
    if (a.cand == nullptr) return;
    __syncthreads();                       // every wavefront is done with the staging buffers
    float* const zt = reinterpret_cast<float*>(lds_raw);
#pragma unroll
    for (int j = 0; j < 16; ++j) zt[((j >> 2) * 8 + lg * 4 + (j & 3)) * kTilePitch + wave * 32 + ln] = zv[0][j];
    __syncthreads();
    const RowBlockDst& r = rbd[0];
    int wrow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int s = r.sbase + wave * 4 + i;
      wrow[i] = (rb0 < nRB && s < r.live) ? r.b * a.L + s : -1;
    }
    tile_candidates4(a, zt, lane, wave * 4, wrow, vt * K::BN, vt, VT);
  }
}

// Scheduling pattern "one MFMA, then its share of OPS memory-side operations (LDS reads, LDS
// writes, global loads)", NM times: the counts must be compile-time constants.
template <int M, int NM, int OPS>
struct Interleave {
  static __device__ __forceinline__ void run() {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x320, (OPS * (M + 1)) / NM - (OPS * M) / NM, 0);
    Interleave<M + 1, NM, OPS>::run();
  }
};
template <int NM, int OPS>
struct Interleave<NM, NM, OPS> {
  static __device__ __forceinline__ void run() {}
};

// ---- exactly 4 row blocks (B * ceil(L / 32) = 4, e.g. 2 sequences x 64 positions or one window
// of 128): one workgroup holds ALL rows, so W is read exactly once and nothing depends on L2 --------
// With 128-256 h rows per byte of W the matrix pipe and the LDS carry real load; the kernels above
// re-stage the whole h tile for every 128 columns.  Here a workgroup of 8 wavefronts owns 256
// columns x all 4 row blocks (half the LDS writes of h per column), tiled 4 x 2: wavefront (wc, wr)
// multiplies 64 columns by 2 row blocks (6 operand reads per 8 MFMAs).  W and h tiles are shared,
// double buffered in LDS, fetched ahead into registers by all 512 threads, one barrier per k-tile;
// inside a wavefront the operand reads of k-step kk + 1, the LDS writes of the next tile and the
// global loads of the tile after it are issued one by one between the MFMAs of k-step kk.
template <int C>
struct Gemm8Cfg {
  static constexpr int THREADS = 512;
  static constexpr int RBW = 4;
  static constexpr int BN = 256;
  static constexpr int HROWS = RBW * C * 32;
  static constexpr int NB = 2 * C;                 // h-row tiles per wavefront (2 row blocks)
  static constexpr int WL = BN * 8 / THREADS;      // 4
  static constexpr int HL = HROWS * 8 / THREADS;   // 4 (C = 2) or 2
  static constexpr int W_LDS = BN * PITCH;
  static constexpr int H_LDS = HROWS * PITCH;
  static constexpr int LDS_BYTES = 2 * (W_LDS + H_LDS) * 2;
};

template <int C, bool NT>
__global__ __launch_bounds__(512) void lm_head_gemm8_kernel(const LmHeadArgs a, const int nLb,
                                                            const int nRB, const int VT) {
  using K = Gemm8Cfg<C>;
  constexpr int NB = K::NB, WL = K::WL, HL = K::HL, KK = BK / 16;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[K::LDS_BYTES];
  uint16_t* const Ws_all = reinterpret_cast<uint16_t*>(lds_raw);
  uint16_t* const Hs_all = Ws_all + 2 * K::W_LDS;

  const int vt = blockIdx.x;
  if (vt >= VT) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wc = wave & 3, wr = wave >> 2;
  // where this wavefront's two row blocks go, and the row block whose candidates it selects:
  // fetched now, so that the epilogue does not begin with a round trip for the window starts
  RowBlockDst rbd[2];
#pragma unroll
  for (int r2 = 0; r2 < 2; ++r2) rbd[r2] = row_block_dst(a, min(wr * 2 + r2, nRB - 1), nLb);
  const RowBlockDst rbd_sel = row_block_dst(a, min(wave >> 1, nRB - 1), nLb);
  const int ln = lane & 31, lg = lane >> 5;
  const int chunk = tid & 7, trow = tid >> 3;          // row 0..63 of a 64-row pass
  const int d = a.d;
  const int KT = (d + BK - 1) / BK;
  const int rot = (vt * 5) % KT;
  const uint32_t kclamp = static_cast<uint32_t>(d - 8) * 2u;

  const char* const Wb = reinterpret_cast<const char*>(a.W);
  const char* const Hb = reinterpret_cast<const char*>(a.h);
  uint32_t woff[WL], hoff[HL];
  bool hok[HL];
#pragma unroll
  for (int i = 0; i < WL; ++i)
    woff[i] = static_cast<uint32_t>(min(vt * K::BN + trow + 64 * i, a.n - 1)) * static_cast<uint32_t>(d) * 2u;
#pragma unroll
  for (int i = 0; i < HL; ++i) {                       // tile row = 64 * i + trow
    const int blk = 2 * i + (trow >> 5);
    const int rb = blk / C, c = blk % C;
    const int b = rb / nLb, s = (rb % nLb) * 32 + (trow & 31);
    hok[i] = rb < nRB && s < a.L;
    hoff[i] = hok[i] ? static_cast<uint32_t>((b * C + c) * a.L + s) * static_cast<uint32_t>(d) * 2u : 0u;
  }
  u32x4 wreg[1][WL], hreg[1][HL];   // one stage: a second one would not fit 256 registers
  bool kok[1];
  auto gload = [&](int stage, int t) {
    int kt = min(t, KT - 1) + rot;
    if (kt >= KT) kt -= KT;
    const int k = kt * BK + chunk * 8;
    kok[stage] = t < KT && k < d;                      // a tile past the end counts as zeros
    const uint32_t kb = min(static_cast<uint32_t>(k) * 2u, kclamp);
#pragma unroll
    for (int i = 0; i < WL; ++i) wreg[stage][i] = load_w<NT>(reinterpret_cast<const u32x4*>(Wb + (woff[i] + kb)));
#pragma unroll
    for (int i = 0; i < HL; ++i) hreg[stage][i] = *reinterpret_cast<const u32x4*>(Hb + (hoff[i] + kb));
  };
  auto lstore = [&](int stage, int buf) {
    uint16_t* const Wd = Ws_all + buf * K::W_LDS;
    uint16_t* const Hd = Hs_all + buf * K::H_LDS;
#pragma unroll
    for (int i = 0; i < WL; ++i)
      *reinterpret_cast<u32x4*>(&Wd[(trow + 64 * i) * PITCH + chunk * 8]) = wreg[stage][i];
#pragma unroll
    for (int i = 0; i < HL; ++i) {
      const bool keep = hok[i] && kok[stage];
      *reinterpret_cast<u32x4*>(&Hd[(trow + 64 * i) * PITCH + chunk * 8]) =
          keep ? hreg[stage][i] : u32x4{0u, 0u, 0u, 0u};
    }
  };
  f32x16 acc[2][NB];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[c][i][j] = 0.f;

  // tile t: registers <- memory during tile t - 2; LDS buffer t % 2 <- registers during tile
  // t - 1; MFMAs during tile t.  The barrier that ends tile t - 1 publishes it.
  gload(0, 0);
  lstore(0, 0);
  gload(0, 1);
  __syncthreads();
  for (int t = 0; t < KT; t += 2) {            // an odd KT is padded by one all-zero tile
#pragma unroll
    for (int u = 0; u < 2; ++u) {              // tile t + u sits in buffer u
      hard_fence();
      const uint16_t* const Wt = Ws_all + u * K::W_LDS + (wc * 64 + ln) * PITCH + lg * 8;
      const uint16_t* const Ht = Hs_all + u * K::H_LDS + (wr * NB * 32 + ln) * PITCH + lg * 8;
      u32x4 bq[2][2], aq[2][NB];
      auto fetch = [&](int q, int kk) {
#pragma unroll
        for (int c = 0; c < 2; ++c) bq[q][c] = *reinterpret_cast<const u32x4*>(&Wt[c * 32 * PITCH + kk * 16]);
#pragma unroll
        for (int i = 0; i < NB; ++i) aq[q][i] = *reinterpret_cast<const u32x4*>(&Ht[i * 32 * PITCH + kk * 16]);
      };
      fetch(0, 0);
      lstore(0, u ^ 1);                        // tile t + u + 1 -> the other buffer
      gload(0, t + u + 2);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        if (kk + 1 < KK) fetch((kk + 1) & 1, kk + 1);
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int i = 0; i < NB; ++i)
            acc[c][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aq[kk & 1][i]),
                                                                __builtin_bit_cast(bf16x8, bq[kk & 1][c]),
                                                                acc[c][i], 0, 0, 0);
      }
      // first the operands of k-step 0, then one memory-side operation between two MFMAs
      constexpr int OPS = 2 * (WL + HL) + (KK - 1) * (NB + 2), NM = KK * 2 * NB;
      __builtin_amdgcn_sched_group_barrier(0x100, NB + 2, 0);
      Interleave<0, NM, OPS>::run();
      hard_fence();
      __syncthreads();
    }
  }

  float zv[2][2][16];                       // processed logits [column half][row block][element]
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
      for (int j = 0; j < 16; ++j) zv[c][r2][j] = processed_logit<C>(a, acc[c][r2 * C][j], acc[c][r2 * C + C - 1][j]);
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const int v = vt * K::BN + wc * 64 + c * 32 + ln;
    if (v >= a.n) continue;
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2) {
      const int rb = wr * 2 + r2;
      if (rb >= nRB) break;
      const RowBlockDst& r = rbd[r2];
#pragma unroll
      for (int j = 0; j < 16; ++j) store_z(a, r, r.sbase + (j >> 2) * 8 + lg * 4 + (j & 3), v, zv[c][r2][j]);
    }
  }

  if constexpr (K::LDS_BYTES >= 128 * kTilePitch * 4) {
    // ---- per-tile candidates for the row kernel (a.cand is uniform) --------------------------
    static_assert(K::BN == kTileCols, "logit tile width");
    if (a.cand == nullptr) return;
    __syncthreads();                       // (also the loop's last barrier) staging buffers are free
    float* const zt = reinterpret_cast<float*>(lds_raw);
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
        for (int j = 0; j < 16; ++j)
          zt[((wr * 2 + r2) * 32 + (j >> 2) * 8 + lg * 4 + (j & 3)) * kTilePitch + wc * 64 + c * 32 + ln] = zv[c][r2][j];
    __syncthreads();
#pragma unroll 1
    for (int g = 0; g < 4; ++g) {          // 16 tile rows per wavefront, four at a time
      const int q0 = wave * 16 + g * 4;
      const int rb = q0 >> 5;                // == wave >> 1
      int wrow[4] = {-1, -1, -1, -1};
      if (rb < nRB) {
        const RowBlockDst& r = rbd_sel;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int s = r.sbase + (q0 & 31) + i;
          wrow[i] = s < r.live ? r.b * a.L + s : -1;
        }
      }
      tile_candidates4(a, zt, lane, q0, wrow, vt * K::BN, vt, VT);
    }
  }
}

// ---- narrow vocabularies: k split over the wavefronts of a workgroup ---------------------
template <int RBW, int C, int KS>
struct SplitCfg {
  static constexpr int NW = KS;
  static constexpr int THREADS = NW * 64;
  static constexpr int NBLK = RBW * C;
  static constexpr int HROWS = NBLK * 32;
  static constexpr int D = KS == 8 ? 2 : 4;       // W tiles in flight per wavefront
  static constexpr int DH = 2;                    // h tiles in flight per wavefront
  static constexpr int STAGE_BYTES = NW * (32 + HROWS) * PITCH * 2;
  static constexpr int RED_BYTES = NW * NBLK * 16 * 64 * 4;
  static constexpr int LDS_BYTES = STAGE_BYTES > RED_BYTES ? STAGE_BYTES : RED_BYTES;
};

template <int RBW, int C, int KS>
__global__ __launch_bounds__((SplitCfg<RBW, C, KS>::THREADS)) void lm_head_splitk_kernel(
    // plain leading arguments: the hardware preloads them into SGPRs at wavefront launch, so the
    // first loads do not wait for a fetch of the kernel-argument segment
    const uint16_t* const W_, const uint16_t* const h_, const int d_, const int n_, const int L_,
    const int nLb, const int nRB, const int MT, const int rm_gshift, const int rm_rot,
    const LmHeadArgs a) {
  const RowMap rm{rm_gshift, rm_rot};
  using K = SplitCfg<RBW, C, KS>;
  constexpr int NBLK = K::NBLK, HROWS = K::HROWS, D = K::D, DH = K::DH, NWAVE = K::NW;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[K::LDS_BYTES];
  const int id = blockIdx.x;
  const int xcd = id % 8, jt = id / (8 * MT);
  const int vt = jt * 8 + xcd;
  const int mt = (id / 8) % MT;
  if (mapped_row(rm, xcd, jt, 32, 0) >= n_) return;   // no row left for this tile
  const int rb0 = mt * RBW;
  RowBlockDst rbd[RBW];                               // fetched now: not a round trip in the epilogue
#pragma unroll
  for (int rbw = 0; rbw < RBW; ++rbw) rbd[rbw] = row_block_dst(a, min(rb0 + rbw, nRB - 1), nLb);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int ln = lane & 31, lg = lane >> 5, chunk = lane & 7, lrow = lane >> 3;
  const int d = d_;
  const int KT = (d + BK - 1) / BK;
  const int ktq = (KT + NWAVE - 1) / NWAVE;
  const int kt_begin = wave * ktq;
  const int ntiles = max(0, min(KT, kt_begin + ktq) - kt_begin);
  // the cyclic walk covers exactly the wavefront's tiles: the last pass of the loop below runs
  // only as many tiles as are left (C1: 5 tiles per wavefront are one pass of 4 and one of 1)
  const int rot = ntiles > 0 ? (vt * 5 + wave * 3) % ntiles : 0;
  auto ktile = [&](int t, bool& valid) {     // see lm_head_kernel: loads are never predicated
    int r = t + rot;
    if (r >= ntiles) r -= ntiles;
    valid = t < ntiles;
    return valid ? kt_begin + r : 0;
  };
  uint16_t* const Ws = reinterpret_cast<uint16_t*>(lds_raw) + wave * (32 + HROWS) * PITCH;
  uint16_t* const Hs = Ws + 32 * PITCH;

  const char* const Wb = reinterpret_cast<const char*>(W_);
  const char* const Hb = reinterpret_cast<const char*>(h_);
  const uint32_t kclamp = static_cast<uint32_t>(d - 8) * 2u;
  uint32_t woff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = mapped_row(rm, xcd, jt, 32, lrow + 8 * i);
    woff[i] = static_cast<uint32_t>(min(v, n_ - 1)) * static_cast<uint32_t>(d) * 2u;
  }
  constexpr int HL = HROWS / 8;                  // loads per lane per h tile
  uint32_t hoff[HL];
  bool hok[HL];
#pragma unroll
  for (int i = 0; i < HL; ++i) {
    const int rr = lrow + 8 * i;
    const int blk = rr >> 5, r = rr & 31;
    const int rb = rb0 + blk / C, c = blk % C;
    const int b = rb / nLb, s = (rb % nLb) * 32 + r;
    hok[i] = rb < nRB && s < L_;
    hoff[i] = hok[i] ? static_cast<uint32_t>((b * C + c) * L_ + s) * static_cast<uint32_t>(d) * 2u : 0u;
  }
  u32x4 wreg[D][4], hreg[DH][HL];
  bool hkok[DH];
  auto wload = [&](int slot, int t) {
    bool valid;
    const int kt = ktile(t, valid);
    const uint32_t kb = min(static_cast<uint32_t>(kt * BK + chunk * 8) * 2u, kclamp);
#pragma unroll
    for (int i = 0; i < 4; ++i) wreg[slot][i] = load_w<false>(reinterpret_cast<const u32x4*>(Wb + (woff[i] + kb)));
  };
  auto hload = [&](int slot, int t) {
    bool valid;
    const int kt = ktile(t, valid);
    const int k = kt * BK + chunk * 8;
    const bool kok = valid && k < d;
    const uint32_t kb = min(static_cast<uint32_t>(k) * 2u, kclamp);
#pragma unroll
    for (int i = 0; i < HL; ++i) hreg[slot][i] = *reinterpret_cast<const u32x4*>(Hb + (hoff[i] + kb));
    hkok[slot] = kok;
  };
  f32x16 acc[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  static_assert(D % DH == 0, "register stages of h must be static in the unrolled body");
#pragma unroll
  for (int j = 0; j < D; ++j) wload(j, j);
#pragma unroll
  for (int j = 0; j < DH; ++j) hload(j, j);
  // one pass over CNT <= D tiles; PF false: the last pass, no loads past the end
  auto body = [&](int t0, auto pf, auto cnt) {
    constexpr bool PF = decltype(pf)::value;
    constexpr int CNT = decltype(cnt)::value;
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
      compiler_fence();
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<u32x4*>(&Ws[(lrow + 8 * i) * PITCH + chunk * 8]) = wreg[j][i];
#pragma unroll
      for (int i = 0; i < HL; ++i) {          // zeroing here: at the load it would wait for it
        const u32x4 t4 = hreg[j % DH][i];
        const bool keep = hok[i] && hkok[j % DH];
        *reinterpret_cast<u32x4*>(&Hs[(lrow + 8 * i) * PITCH + chunk * 8]) =
            (keep ? t4 : u32x4{0u, 0u, 0u, 0u});
      }
      if (PF) wload(j, t0 + j + D);
      if (PF || j + DH < CNT) hload(j % DH, t0 + j + DH);
      compiler_fence();
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        const u32x4 braw = *reinterpret_cast<const u32x4*>(&Ws[ln * PITCH + kk * 16 + lg * 8]);
        const bf16x8 bfrag = __builtin_bit_cast(bf16x8, braw);
#pragma unroll
        for (int i = 0; i < NBLK; ++i) {
          const u32x4 araw = *reinterpret_cast<const u32x4*>(&Hs[(i * 32 + ln) * PITCH + kk * 16 + lg * 8]);
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, araw), bfrag,
                                                           acc[i], 0, 0, 0);
        }
      }
      compiler_fence();
    }
  };
  {
    const int full = ntiles / D * D, rem = ntiles - full;
    const int prefetching = rem == 0 ? full - D : full;      // tiles of the passes that load ahead
    for (int t0 = 0; t0 < prefetching; t0 += D) body(t0, TrueT{}, IntT<D>{});
    if (rem == 0) {
      if (full > 0) body(full - D, FalseT{}, IntT<D>{});
    } else if (rem == 1) {
      body(full, FalseT{}, IntT<1>{});
    } else if constexpr (D > 2) {
      if (rem == 2) body(full, FalseT{}, IntT<2>{});
      else body(full, FalseT{}, IntT<3>{});
    }
  }
  // the partial accumulators meet in LDS
  __syncthreads();
  float* red = reinterpret_cast<float*>(lds_raw);
#pragma unroll
  for (int i = 0; i < NBLK; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) red[((wave * NBLK + i) * 16 + j) * 64 + lane] = acc[i][j];
  __syncthreads();
  // wavefront w adds up (partial sums in wavefront order 0, 1, 2, ...) and stores the
  // accumulator elements j = w, w + NWAVE, ... of every tile
  const int v = mapped_row(rm, xcd, jt, 32, ln);
  if (v >= a.n) return;
#pragma unroll
  for (int rbw = 0; rbw < RBW; ++rbw) {
    const int rb = rb0 + rbw;
    if (rb >= nRB) break;
    const RowBlockDst& r = rbd[rbw];
#pragma unroll
    for (int jj = 0; jj < 16 / NWAVE; ++jj) {
      const int j = wave + jj * NWAVE;
      float c = red[((0 * NBLK + rbw * C) * 16 + j) * 64 + lane];
      float u = red[((0 * NBLK + rbw * C + C - 1) * 16 + j) * 64 + lane];
#pragma unroll
      for (int w = 1; w < NWAVE; ++w) {
        c += red[((w * NBLK + rbw * C) * 16 + j) * 64 + lane];
        u += red[((w * NBLK + rbw * C + C - 1) * 16 + j) * 64 + lane];
      }
      store_logit<C>(a, r, r.sbase + (j >> 2) * 8 + lg * 4 + (j & 3), v, c, u);
    }
  }
}

// Row map for these operands and the number of workgroup tiles per XCD it needs.
RowMap make_row_map(const LmHeadArgs& a, int BN, int VT, bool affine, int* tiles_per_xcd) {
  RowMap m{-1, 0};
  *tiles_per_xcd = (VT + 7) / 8;
  if (!affine) return m;
  const size_t row_bytes = static_cast<size_t>(a.d) * 2;
  constexpr size_t kBlock = 128 * 1024;
  if (kBlock % row_bytes != 0) return m;
  const int G = static_cast<int>(kBlock / row_bytes);
  if ((G & (G - 1)) != 0) return m;
  int gs = 0;
  while ((1 << gs) < G) ++gs;
  m.gshift = gs;
  // block (mod 8) that holds the middle of group 0
  m.rot = static_cast<int>(((reinterpret_cast<uintptr_t>(a.W) + kBlock / 2) / kBlock) % 8);
  const long groups = (static_cast<long>(a.n) + G - 1) / G;
  const long rows_per_xcd = (groups + 7) / 8 * G;
  *tiles_per_xcd = static_cast<int>((rows_per_xcd + BN - 1) / BN);
  return m;
}

// Optional timing of the launch: the runtime attaches the two events to the dispatch itself
// (start and stop time of the kernel), so no marker packets of their own enter the stream.
struct LaunchEvents {
  hipEvent_t start, stop;
};
template <class Kern, class... Args>
void launch_kernel(Kern kernel, dim3 grid, dim3 block, hipStream_t s, const LaunchEvents& ev, Args... args) {
  if (ev.start && ev.stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ev.start, ev.stop, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
}

// W is streamed past the caches when its slice cannot stay in the memory-side cache anyway
bool stream_w(const LmHeadArgs& a) { return 2.0 * a.d * a.n > 192.0 * 1024 * 1024; }

template <int RBW, int C, int NWV>
hipError_t launch_wide(const LmHeadArgs& a, hipStream_t s, const LaunchEvents& ev) {
  using K = Cfg<RBW, C, NWV>;
  const int nLb = (a.L + 31) / 32;
  const int nRB = a.B * nLb;
  const int VT = (a.n + K::BN - 1) / K::BN;
  const int MT = (nRB + RBW - 1) / RBW;
  int JT;
  // The wavefronts of this kernel walk k in step (shared h tile): with all rows of a workgroup
  // in one residue class its requests would pile onto one channel at a time (measured: 124 us
  // against 94 us for the full vocabulary), so rows stay consecutive here.
  const RowMap rm = make_row_map(a, K::BN, VT, false, &JT);
  if (stream_w(a))
    launch_kernel(lm_head_kernel<RBW, C, NWV, true>, dim3(JT * 8 * MT), dim3(K::THREADS), s, ev, a, nLb, nRB, VT,
                  MT, rm);
  else
    launch_kernel(lm_head_kernel<RBW, C, NWV, false>, dim3(JT * 8 * MT), dim3(K::THREADS), s, ev, a, nLb, nRB, VT,
                  MT, rm);
  return hipGetLastError();
}

template <int RBW, int C, int KS>
hipError_t launch_split(const LmHeadArgs& a, hipStream_t s, const LaunchEvents& ev) {
  using K = SplitCfg<RBW, C, KS>;
  const int nLb = (a.L + 31) / 32;
  const int nRB = a.B * nLb;
  const int VT = (a.n + 31) / 32;
  const int MT = (nRB + RBW - 1) / RBW;
  int JT;
  const RowMap rm = make_row_map(a, 32, VT, true, &JT);
  launch_kernel(lm_head_splitk_kernel<RBW, C, KS>, dim3(JT * 8 * MT), dim3(K::THREADS), s, ev, a.W, a.h, a.d, a.n,
                a.L, nLb, nRB, MT, rm.gshift, rm.rot, a);
  return hipGetLastError();
}

template <int C>
hipError_t launch_gemm8(const LmHeadArgs& a, hipStream_t s, const LaunchEvents& ev) {
  using K = Gemm8Cfg<C>;
  const int nLb = (a.L + 31) / 32;
  const int VT = (a.n + K::BN - 1) / K::BN;
  if (stream_w(a))
    launch_kernel(lm_head_gemm8_kernel<C, true>, dim3(VT), dim3(K::THREADS), s, ev, a, nLb, a.B * nLb, VT);
  else
    launch_kernel(lm_head_gemm8_kernel<C, false>, dim3(VT), dim3(K::THREADS), s, ev, a, nLb, a.B * nLb, VT);
  return hipGetLastError();
}

// Which kernel serves a problem shape.
struct Variant {
  bool split;   // lm_head_splitk_kernel (else lm_head_kernel)
  int rbw, nw;  // row blocks per workgroup; wavefronts (= k parts for the split kernel)
  bool gemm8;   // lm_head_gemm8_kernel
};
Variant choose(const LmHeadArgs& a) {
  const int nRB = a.B * ((a.L + 31) / 32);
  const int KT = (a.d + BK - 1) / BK;
  // Narrow vocabularies: with 128-column workgroups fewer than ~1.5 per CU would exist;
  // split k inside the workgroup instead and give every workgroup 32 columns.
  const bool narrow = (a.n + 127) / 128 < 384 && KT >= 16;
  // many row blocks: 2 per workgroup.  4 per workgroup would read W from L2 half as often, but
  // its 91 KB of LDS and ~390 registers allow one workgroup per CU, and with one wavefront per
  // SIMD the load / LDS / MFMA phases of a tile run back to back (C3: 98 us against 85 us).
  // all rows in one workgroup when there are 3 or 4 row blocks and enough 256-column tiles to
  // fill the chip
  if ((nRB == 4 || nRB == 3) && (a.n + 255) / 256 >= 200) return {false, 4, 8, true};
  if (nRB >= 4) return {false, 2, 4, false};
  if (nRB >= 2) return {narrow, 2, 4, false};
  if (narrow) return {true, 1, KT >= 48 ? 8 : 4, false};
  // wide vocabulary: 8 wavefronts share each h tile (halves the h traffic out of L2)
  return {false, 1, (a.n + 255) / 256 >= 200 ? 8 : 4, false};
}

template <int C>
hipError_t launch_c(const LmHeadArgs& a, hipStream_t s, const LaunchEvents& ev) {
  const Variant v = choose(a);
  if (v.gemm8) return launch_gemm8<C>(a, s, ev);
  if (v.split) {
    if (v.rbw == 2) return launch_split<2, C, 4>(a, s, ev);
    return v.nw == 8 ? launch_split<1, C, 8>(a, s, ev) : launch_split<1, C, 4>(a, s, ev);
  }
  if (v.rbw == 2) return launch_wide<2, C, 4>(a, s, ev);
  return v.nw == 8 ? launch_wide<1, C, 8>(a, s, ev) : launch_wide<1, C, 4>(a, s, ev);
}

}  // namespace

hipError_t launch_lm_head(const LmHeadArgs& a, hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const LaunchEvents ev{ev_start, ev_stop};
  return a.C == 2 ? launch_c<2>(a, s, ev) : launch_c<1>(a, s, ev);
}

int lm_head_tiles(const LmHeadArgs& a) {
  const Variant v = choose(a);
  const int tiles = (a.n + kTileCols - 1) / kTileCols;
  if (tiles > kRowMaxTiles) return 0;
  if (v.gemm8) return Gemm8Cfg<2>::LDS_BYTES >= 128 * kTilePitch * 4 && a.C == 2 ? tiles : 0;
  if (!v.split && v.rbw == 1 && v.nw == 8) return tiles;
  return 0;
}

int lm_head_kernel_name(const LmHeadArgs& a, char* buf, size_t cap) {
  const Variant v = choose(a);
  const char* nt = stream_w(a) ? "true" : "false";
  if (v.gemm8) return snprintf(buf, cap, "lm_head_gemm8_kernel<%d, %s>", a.C, nt);
  if (v.split) return snprintf(buf, cap, "lm_head_splitk_kernel<%d, %d, %d>", v.rbw, a.C, v.nw);
  return snprintf(buf, cap, "lm_head_kernel<%d, %d, %d, %s>", v.rbw, a.C, v.nw, nt);
}

}  // namespace scd
