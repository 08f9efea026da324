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
//     k).  Private staging needs no workgroup barrier, so the four wavefronts of
//     a workgroup drift apart and the W stream never drains.
//   * The accumulators of a wavefront are RBW "row blocks" x C tiles: a row block
//     is 32 window positions of one sequence, its cond and uncond tiles live in
//     the SAME lanes, so the guidance mix needs no data movement.
//   * KS = 1 (wide vocabularies): the 4 wavefronts take 4 x 32 neighbouring
//     columns and SHARE the h tile through LDS (double buffered, one barrier per
//     h tile).  KS = 4 (narrow vocabularies, too few column tiles to fill 256
//     CUs): the 4 wavefronts take the same 32 columns and a quarter of k each,
//     stage h privately too, and their partial sums are added in a fixed order
//     through LDS at the end (deterministic).
#include "scd_kernels.h"

namespace scd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;          // k elements per W tile (128 bytes per row)
constexpr int PITCH = BK + 8;   // LDS row pitch in bf16 elements (144 bytes)
__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }

template <int RBW, int C, int KS, int NWV>
struct Cfg {
  static constexpr int NW = KS == 1 ? NWV : KS;   // wavefronts per workgroup
  static constexpr int THREADS = NW * 64;
  static constexpr int NBLK = RBW * C;            // accumulator tiles per wavefront
  static constexpr int HROWS = NBLK * 32;         // h rows per tile
  // W tiles in flight per wavefront (registers)
  static constexpr int D = KS == 1 ? 4 : (KS == 8 ? 2 : 4);
  static constexpr int DH = 2;                    // h tiles in flight (registers)
  static constexpr int HT = (KS == 1 && NBLK <= 2) ? 2 : 1;   // W tiles per shared h tile
  static constexpr int BKH = BK * HT;
  static constexpr int PITCH_H = BKH + 8;
  static constexpr int BN = KS == 1 ? NW * 32 : 32;   // columns per workgroup
  static constexpr int W_LDS = NW * 32 * PITCH;                     // elements
  static constexpr int H_LDS = KS == 1 ? 2 * HROWS * PITCH_H : NW * HROWS * PITCH;
  static constexpr int RED_BYTES = KS == 1 ? 0 : NW * NBLK * 16 * 64 * 4;
  static constexpr int STAGE_BYTES = (W_LDS + H_LDS) * 2;
  static constexpr int LDS_BYTES = STAGE_BYTES > RED_BYTES ? STAGE_BYTES : RED_BYTES;
};

template <int RBW, int C, int KS, int NWV>
__global__ __launch_bounds__((Cfg<RBW, C, KS, NWV>::THREADS)) void lm_head_kernel(const LmHeadArgs a, const int nLb,
                                                          const int nRB, const int VT,
                                                          const int MT) {
  using K = Cfg<RBW, C, KS, NWV>;
  constexpr int NBLK = K::NBLK, HROWS = K::HROWS, D = K::D, DH = K::DH, HT = K::HT;
  constexpr int NWAVE = K::NW, THREADS = K::THREADS;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[K::LDS_BYTES];
  uint16_t* const Ws_all = reinterpret_cast<uint16_t*>(lds_raw);
  uint16_t* const Hs_all = Ws_all + K::W_LDS;

  // Workgroups with consecutive ids land on different XCDs (round robin over
  // 8); the MT row-block tiles that share one slab of W get ids 8 apart, i.e.
  // the same XCD and the same L2.
  const int id = blockIdx.x;
  const int vt = (id / (8 * MT)) * 8 + (id % 8);
  const int mt = (id / 8) % MT;
  if (vt >= VT) return;
  const int rb0 = mt * RBW;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int ln = lane & 31;     // row (A) / column (B) inside a 32x32 tile
  const int lg = lane >> 5;     // k-group
  const int chunk = lane & 7;   // 16-byte chunk inside a 128-byte row segment
  const int lrow = lane >> 3;   // 0..7

  const int d = a.d;
  const int KT = (d + BK - 1) / BK;
  // this wavefront's columns and k-tiles
  const int v0 = vt * K::BN + (KS == 1 ? wave * 32 : 0);
  const int ktq = KS == 1 ? KT : (KT + NWAVE - 1) / NWAVE;
  const int kt_begin = KS == 1 ? 0 : wave * ktq;
  const int kt_end = KS == 1 ? KT : min(KT, kt_begin + ktq);
  const int ntiles = max(0, kt_end - kt_begin);
  const int ntiles_pad = (ntiles + D - 1) / D * D;
  // Every workgroup walks k from a different starting tile (cyclically).  Rows of W
  // are d*2 bytes apart, so without the rotation all wavefronts of the chip would ask
  // for the same address bits (mod the row pitch) at the same time and camp on a few
  // memory channels.  An odd multiplier spreads the starts over every tile offset.
  const int rot = ntiles_pad > 0 ? (vt * 5 + (KS == 1 ? 0 : wave * 3)) % ntiles_pad : 0;
  auto ktile = [&](int t) {          // logical tile t of this wavefront -> k-tile index, -1 if none
    if (t >= ntiles_pad) return -1;
    int r = t + rot;
    if (r >= ntiles_pad) r -= ntiles_pad;
    return r < ntiles ? kt_begin + r : -1;
  };

  uint16_t* const Ws = Ws_all + wave * 32 * PITCH;          // private W staging

  // ---- W: coalesced private loads, D tiles ahead -----------------------------------
  const uint16_t* wsrc[4];
  bool wok[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = v0 + lrow + 8 * i;
    wok[i] = v < a.n;
    wsrc[i] = a.W + static_cast<size_t>(wok[i] ? v : 0) * d;
  }
  uint4 wreg[D][4];
  auto wload = [&](int slot, int t) {       // logical tile index t
    const int kt = ktile(t);
    const int k = kt * BK + chunk * 8;
    const bool kok = kt >= 0 && k < d;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      wreg[slot][i] = (wok[i] && kok) ? *reinterpret_cast<const uint4*>(wsrc[i] + k)
                                      : make_uint4(0, 0, 0, 0);
  };
  auto wstore = [&](int slot) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<uint4*>(&Ws[(lrow + 8 * i) * PITCH + chunk * 8]) = wreg[slot][i];
  };

  // ---- h rows -----------------------------------------------------------------------
  auto hrow_ptr = [&](int rr, bool& ok) -> const uint16_t* {   // rr = tile row 0..HROWS-1
    const int blk = rr >> 5, r = rr & 31;
    const int rb = rb0 + blk / C, c = blk % C;
    const int b = rb / nLb, s = (rb % nLb) * 32 + r;
    ok = rb < nRB && s < a.L;
    return a.h + (ok ? (static_cast<size_t>(b * C + c) * a.L + s) * d : 0);
  };

  f32x16 acc[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  // MFMAs of one W tile; Hs_tile points at the h rows, column offset koff, row pitch hp
  auto compute = [&](const uint16_t* Hs_tile, int hp, int koff) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const uint4 braw = *reinterpret_cast<const uint4*>(&Ws[ln * PITCH + kk * 16 + lg * 8]);
      const bf16x8 bfrag = __builtin_bit_cast(bf16x8, braw);
#pragma unroll
      for (int i = 0; i < NBLK; ++i) {
        const uint4 araw =
            *reinterpret_cast<const uint4*>(&Hs_tile[(i * 32 + ln) * hp + koff + kk * 16 + lg * 8]);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, araw), bfrag,
                                                         acc[i], 0, 0, 0);
      }
    }
  };

  if constexpr (KS == 1) {
    // ======== shared h tile (BKH = HT * 64 wide), double buffered =====================
    constexpr int CH = K::BKH / 8;                 // 16-byte chunks per h row
    constexpr int RPP = THREADS / CH;              // rows covered per pass of the workgroup
    constexpr int HL = HROWS / RPP;                // loads per thread per h tile
    const int hchunk = tid % CH, hr0 = tid / CH;
    const uint16_t* hsrc[HL];
    bool hok[HL];
#pragma unroll
    for (int i = 0; i < HL; ++i) hsrc[i] = hrow_ptr(hr0 + RPP * i, hok[i]);
    uint4 hreg[DH][HL];
    // logical h tile st = logical W tiles st*HT .. st*HT+HT-1; after the rotation these
    // need not be neighbours in k (wrap-around), so every 64-wide part is placed on its own
    constexpr int CHW = BK / 8;            // 16-byte chunks per W tile width
    auto hload = [&](int slot, int st) {
      const int kt = ktile(st * HT + hchunk / CHW);
      const int k = kt * BK + (hchunk % CHW) * 8;
      const bool kok = kt >= 0 && k < d;
#pragma unroll
      for (int i = 0; i < HL; ++i)
        hreg[slot][i] = (hok[i] && kok) ? *reinterpret_cast<const uint4*>(hsrc[i] + k)
                                        : make_uint4(0, 0, 0, 0);
    };
    auto hstore = [&](int slot, int buf) {
      uint16_t* dst = Hs_all + buf * HROWS * K::PITCH_H;
#pragma unroll
      for (int i = 0; i < HL; ++i)
        *reinterpret_cast<uint4*>(&dst[(hr0 + RPP * i) * K::PITCH_H + hchunk * 8]) = hreg[slot][i];
    };
    // h tile st is loaded into register stage st % 2 two h tiles ahead, moved to LDS
    // buffer st % 2 at the end of h tile st - 1, and consumed during h tile st.
    static_assert(D % (2 * HT) == 0, "register stages of h must be static in the unrolled body");
#pragma unroll
    for (int j = 0; j < D; ++j) wload(j, j);
    hload(0, 0);
    hload(1, 1);
    hstore(0, 0);
    __syncthreads();
    for (int t0 = 0; t0 < ntiles_pad; t0 += D) {
#pragma unroll
      for (int j = 0; j < D; ++j) {
        const int t = t0 + j;
        const int st = t / HT;
        const int stage = (j / HT) & 1;            // == st & 1 because t0 / HT is even
        compiler_fence();
        wstore(j);
        wload(j, t + D);
        compiler_fence();
        compute(Hs_all + stage * HROWS * K::PITCH_H, K::PITCH_H, (j % HT) * BK);
        compiler_fence();
        if (j % HT == HT - 1) {
          hstore(stage ^ 1, stage ^ 1);            // h tile st + 1 -> the other LDS buffer
          hload(stage, st + 2);                    // h tile st + 2 -> the register stage just freed
          __syncthreads();
        }
      }
    }
  } else {
    // ======== split k: everything private to the wavefront, no barrier in the loop =====
    constexpr int HL = HROWS / 8;                  // loads per lane per h tile
    uint16_t* const Hs = Hs_all + wave * HROWS * PITCH;
    const uint16_t* hsrc[HL];
    bool hok[HL];
#pragma unroll
    for (int i = 0; i < HL; ++i) hsrc[i] = hrow_ptr(lrow + 8 * i, hok[i]);
    uint4 hreg[DH][HL];
    auto hload = [&](int slot, int t) {
      const int kt = ktile(t);
      const int k = kt * BK + chunk * 8;
      const bool kok = kt >= 0 && k < d;
#pragma unroll
      for (int i = 0; i < HL; ++i)
        hreg[slot][i] = (hok[i] && kok) ? *reinterpret_cast<const uint4*>(hsrc[i] + k)
                                        : make_uint4(0, 0, 0, 0);
    };
    auto hstore = [&](int slot) {
#pragma unroll
      for (int i = 0; i < HL; ++i)
        *reinterpret_cast<uint4*>(&Hs[(lrow + 8 * i) * PITCH + chunk * 8]) = hreg[slot][i];
    };
    static_assert(D % DH == 0, "register stages of h must be static in the unrolled body");
#pragma unroll
    for (int j = 0; j < D; ++j) wload(j, j);
#pragma unroll
    for (int j = 0; j < DH; ++j) hload(j, j);
    for (int t0 = 0; t0 < ntiles_pad; t0 += D) {
#pragma unroll
      for (int j = 0; j < D; ++j) {
        compiler_fence();
        wstore(j);
        hstore(j % DH);
        wload(j, t0 + j + D);
        hload(j % DH, t0 + j + DH);
        compiler_fence();
        compute(Hs, PITCH, 0);
        compiler_fence();
      }
    }
    if constexpr (KS > 1) {
    // fixed-order sum of the partial accumulators through LDS
    __syncthreads();
    float* red = reinterpret_cast<float*>(lds_raw);
#pragma unroll
    for (int i = 0; i < NBLK; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) red[((wave * NBLK + i) * 16 + j) * 64 + lane] = acc[i][j];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NBLK; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        float sum = red[((0 * NBLK + i) * 16 + j) * 64 + lane];
#pragma unroll
        for (int w = 1; w < NWAVE; ++w) sum += red[((w * NBLK + i) * 16 + j) * 64 + lane];
        acc[i][j] = sum;
      }
    }
  }

  // ---- epilogue.  Accumulator element j of lane (ln, lg) is row (j/4)*8 + lg*4 + j%4,
  // column ln of the 32x32 tile.  With split k every wavefront holds the full sums and
  // stores the accumulator elements j with j % (number of wavefronts) == its index.
  const int v = v0 + ln;
  if (v >= a.n) return;
#pragma unroll
  for (int rbw = 0; rbw < RBW; ++rbw) {
    const int rb = rb0 + rbw;
    if (rb >= nRB) break;
    const int b = rb / nLb;
    const int sbase = (rb % nLb) * 32;
    int p0 = 0, live = a.L;
    float* zb = a.z;
    if (a.pos) {
      p0 = a.pos[b];
      live = min(a.L, a.N - p0);
    }
    if (a.iter) zb += static_cast<size_t>(a.iter[b] & 1) * a.parity_stride;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (KS > 1 && (j % NWAVE) != wave) continue;
      const int s = sbase + (j >> 2) * 8 + lg * 4 + (j & 3);
      if (s >= live) continue;
      float z;
      if (C == 2) {
        const float t0 = __fmul_rn(a.one_plus_lam, acc[rbw * C][j]);
        const float t1 = __fmul_rn(a.lam, acc[rbw * C + C - 1][j]);
        z = __fsub_rn(t0, t1);
      } else {
        z = acc[rbw * C][j];
      }
      z = __fdiv_rn(z, a.tau);
      const int slot = a.pos ? (p0 + s) % a.L : s;
      zb[(static_cast<size_t>(b) * a.L + slot) * a.n + v] = z;
    }
  }
}

template <int RBW, int C, int KS, int NWV = 4>
hipError_t launch_t(const LmHeadArgs& a, hipStream_t s) {
  using K = Cfg<RBW, C, KS, NWV>;
  const int nLb = (a.L + 31) / 32;
  const int nRB = a.B * nLb;
  const int VT = (a.n + K::BN - 1) / K::BN;
  const int MT = (nRB + RBW - 1) / RBW;
  const int VT8 = (VT + 7) / 8 * 8;
  const int grid = VT8 * MT;
  hipLaunchKernelGGL((lm_head_kernel<RBW, C, KS, NWV>), dim3(grid), dim3(K::THREADS), 0, s, a, nLb, nRB,
                     VT, MT);
  return hipGetLastError();
}

template <int C>
hipError_t launch_c(const LmHeadArgs& a, hipStream_t s) {
  const int nRB = a.B * ((a.L + 31) / 32);
  const int KT = (a.d + BK - 1) / BK;
  // Narrow vocabularies: with 128-column workgroups fewer than ~1.5 per CU would
  // exist; split k inside the workgroup instead and give every workgroup 32 columns.
  const bool narrow = (a.n + 127) / 128 < 384 && KT >= 16;
  if (nRB >= 4) return launch_t<4, C, 1>(a, s);
  if (nRB >= 2) return narrow ? launch_t<2, C, 4>(a, s) : launch_t<2, C, 1>(a, s);
  if (narrow && KT >= 48) return launch_t<1, C, 8>(a, s);
  if (narrow) return launch_t<1, C, 4>(a, s);
  // wide vocabulary: 8 wavefronts share each h tile (halves the h traffic out of L2)
  return (a.n + 255) / 256 >= 200 ? launch_t<1, C, 1, 8>(a, s) : launch_t<1, C, 1, 4>(a, s);
}

}  // namespace

hipError_t launch_lm_head(const LmHeadArgs& a, hipStream_t s) {
  return a.C == 2 ? launch_c<2>(a, s) : launch_c<1>(a, s);
}

}  // namespace scd
