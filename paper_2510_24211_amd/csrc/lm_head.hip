// LM head of the window ("Evaluate" step of the SCD / SJD algorithms):
//   logit[m, v] = sum_k h[m, k] * W[v, k]      bf16 x bf16 -> fp32 (MFMA)
// with the first logit processors fused into the epilogue (Sec. 4.3 defines
// p^(t) after post-processing; Sec. 5.1 gives the guidance mix):
//   z = fl(fl((1+lambda) * c) - fl(lambda * u)),   z <- z / tau
// Only the allowed vocabulary rows of W are streamed (the mask to -inf of the
// other ids is realised by never forming their columns).
//
// gfx950 mapping.  The contraction is skinny: M = B*C*L rows (32..1024) against
// n = |allowed| columns (8k..64k) over d = 1k..4k, so the kernel is a stream
// over W.  A workgroup of 4 wavefronts owns a slab of BN = 128 vocabulary rows
// of W and RBW "row blocks" of h; a row block is 32 window positions of one
// sequence, carried as C accumulator tiles (cond, uncond) in the SAME lanes so
// that the guidance mix needs no data movement.  Both operands are k-contiguous
// in memory, so 16-byte loads fill v_mfma_f32_32x32x16_bf16 operands directly
// (lane l: row l%32, k-group l/32, 8 consecutive k).  Tiles are staged through
// LDS with full 128-byte row segments per 8 lanes (coalesced) and a row pitch
// of 144 bytes against bank conflicts; the next k-tile's global loads are in
// flight while the current one feeds the matrix cores.
#include "scd_kernels.h"

namespace scd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;          // k elements per tile (128 bytes per row)
constexpr int BN = 128;         // vocabulary rows per workgroup (4 waves x 32)
constexpr int PITCH = BK + 8;   // LDS row pitch in bf16 elements (144 bytes)
constexpr int THREADS = 256;

template <int RBW, int C>
__global__ __launch_bounds__(THREADS) void lm_head_kernel(const LmHeadArgs a, const int nLb,
                                                          const int nRB, const int VT,
                                                          const int MT) {
  constexpr int NBLK = RBW * C;            // accumulator tiles per wave
  constexpr int HROWS = NBLK * 32;         // h rows staged per k-tile
  __shared__ __attribute__((aligned(16))) uint16_t Ws[BN * PITCH];
  __shared__ __attribute__((aligned(16))) uint16_t Hs[HROWS * PITCH];

  // Workgroups with consecutive ids land on different XCDs (round robin over
  // 8); the MT row-block tiles that share one slab of W get ids 8 apart, i.e.
  // the same XCD and the same L2.
  const int id = blockIdx.x;
  const int vt = (id / (8 * MT)) * 8 + (id % 8);
  const int mt = (id / 8) % MT;
  if (vt >= VT) return;
  const int v0 = vt * BN;
  const int rb0 = mt * RBW;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int ln = lane & 31;     // row (A) / column (B) inside a 32x32 tile
  const int lg = lane >> 5;     // k-group
  const int chunk = tid & 7;    // 16-byte chunk inside a 128-byte row segment
  const int lrow = tid >> 3;    // 0..31

  const int d = a.d;
  const int KT = (d + BK - 1) / BK;

  // Source rows of this thread's global loads (fixed over the k loop).
  const uint16_t* wsrc[4];
  bool wok[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = v0 + lrow + 32 * i;
    wok[i] = v < a.n;
    wsrc[i] = a.W + static_cast<size_t>(wok[i] ? v : 0) * d;
  }
  const uint16_t* hsrc[NBLK];
  bool hok[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i) {
    const int rb = rb0 + i / C;
    const int c = i % C;
    const int b = rb / nLb;
    const int s = (rb % nLb) * 32 + lrow;
    hok[i] = rb < nRB && s < a.L;
    hsrc[i] = a.h + (hok[i] ? (static_cast<size_t>(b * C + c) * a.L + s) * d : 0);
  }

  uint4 wreg[4], hreg[NBLK];
  auto load_tile = [&](int kt) {
    const int k = kt * BK + chunk * 8;
    const bool kok = k < d;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      wreg[i] = (wok[i] && kok) ? *reinterpret_cast<const uint4*>(wsrc[i] + k) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < NBLK; ++i)
      hreg[i] = (hok[i] && kok) ? *reinterpret_cast<const uint4*>(hsrc[i] + k) : make_uint4(0, 0, 0, 0);
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<uint4*>(&Ws[(lrow + 32 * i) * PITCH + chunk * 8]) = wreg[i];
#pragma unroll
    for (int i = 0; i < NBLK; ++i)
      *reinterpret_cast<uint4*>(&Hs[(i * 32 + lrow) * PITCH + chunk * 8]) = hreg[i];
  };

  f32x16 acc[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  load_tile(0);
  store_tile();
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    if (kt + 1 < KT) load_tile(kt + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const uint4 braw = *reinterpret_cast<const uint4*>(&Ws[(wave * 32 + ln) * PITCH + kk * 16 + lg * 8]);
      const bf16x8 bfrag = __builtin_bit_cast(bf16x8, braw);
#pragma unroll
      for (int i = 0; i < NBLK; ++i) {
        const uint4 araw = *reinterpret_cast<const uint4*>(&Hs[(i * 32 + ln) * PITCH + kk * 16 + lg * 8]);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, araw), bfrag,
                                                         acc[i], 0, 0, 0);
      }
    }
    __syncthreads();
    if (kt + 1 < KT) {
      store_tile();
      __syncthreads();
    }
  }

  // Epilogue.  Accumulator element j of lane (ln, lg) is row (j/4)*8 + lg*4 + j%4,
  // column ln of the 32x32 tile.
  const int v = v0 + wave * 32 + ln;
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

template <int RBW, int C>
hipError_t launch_t(const LmHeadArgs& a, hipStream_t s) {
  const int nLb = (a.L + 31) / 32;
  const int nRB = a.B * nLb;
  const int VT = (a.n + BN - 1) / BN;
  const int MT = (nRB + RBW - 1) / RBW;
  const int VT8 = (VT + 7) / 8 * 8;
  const int grid = VT8 * MT;
  hipLaunchKernelGGL((lm_head_kernel<RBW, C>), dim3(grid), dim3(THREADS), 0, s, a, nLb, nRB, VT, MT);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_lm_head(const LmHeadArgs& a, hipStream_t s) {
  const int nRB = a.B * ((a.L + 31) / 32);
  if (a.C == 2) {
    if (nRB >= 4) return launch_t<4, 2>(a, s);
    if (nRB >= 2) return launch_t<2, 2>(a, s);
    return launch_t<1, 2>(a, s);
  }
  if (nRB >= 4) return launch_t<4, 1>(a, s);
  if (nRB >= 2) return launch_t<2, 1>(a, s);
  return launch_t<1, 1>(a, s);
}

}  // namespace scd
