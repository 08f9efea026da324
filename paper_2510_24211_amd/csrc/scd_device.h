// Device-side helpers shared by the gfx950 kernels of the SCD step:
// Philox4x32-10 (Salmon et al., SC'11), the 23-bit uniform mapping, the
// order-preserving float <-> uint32 key map used by the radix select, and
// block-wide reductions for 64-lane wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace scd {

constexpr int kWave = 64;

enum : uint32_t {
  kStreamInit = 0, kStreamAccept = 1, kStreamResid = 2, kStreamGumbel = 3, kStreamAlpha = 4, kStreamIndep = 5
};

__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one widening multiply per product (v_mad_u64_u32) instead of a high and a low one
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c.x;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c.z;
    c = make_uint4(static_cast<uint32_t>(p1 >> 32) ^ c.y ^ k.x, static_cast<uint32_t>(p1),
                   static_cast<uint32_t>(p0 >> 32) ^ c.w ^ k.y, static_cast<uint32_t>(p0));
    k.x += 0x9E3779B9u;
    k.y += 0xBB67AE85u;
  }
  return c;
}

// ((bits >> 9) + 1/2) * 2^-23: every step is exact in fp32, result in (0,1).
__device__ __forceinline__ float u01(uint32_t bits) {
  return (static_cast<float>(bits >> 9) + 0.5f) * 1.1920928955078125e-07f;
}

__device__ __forceinline__ uint2 seed_key(uint64_t seed) {
  return make_uint2(static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
}

// Uniform initial draft of a never-evaluated position: floor(r64 * n / 2^64).
__device__ __forceinline__ int32_t init_token(uint64_t seed, int b, int pos, int n) {
  const uint4 r = philox4x32_10(make_uint4(0u, static_cast<uint32_t>(pos), 0u,
                                           (static_cast<uint32_t>(b) << 8) | kStreamInit),
                                seed_key(seed));
  const uint64_t r64 = (static_cast<uint64_t>(r.x) << 32) | r.y;
  return static_cast<int32_t>(__umul64hi(r64, static_cast<uint64_t>(n)));
}

// Larger float <-> larger key (total order; -0 < +0; NaNs sort above +inf or
// below -inf by sign).
__device__ __forceinline__ uint32_t float_to_key(float f) {
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}
// key with -0 folded onto +0, so that key order == float order for non-NaNs
__device__ __forceinline__ uint32_t zkey(float f) { return float_to_key(f == 0.f ? 0.f : f); }

// ---- wavefront collectives ---------------------------------------------------------
// Lane exchanges through the vector ALU's data-parallel primitives (DPP) and v_readlane:
// no round trip through the LDS crossbar, which a shuffle costs.  All of them must be
// called with the whole wavefront active.
enum : int {
  kDppXor1 = 0xB1,        // quad_perm [1,0,3,2]: lane ^ 1
  kDppXor2 = 0x4E,        // quad_perm [2,3,0,1]: lane ^ 2
  kDppHalfMirror = 0x141, // lane i <-> 7 - i inside groups of 8
  kDppMirror = 0x140,     // lane i <-> 15 - i inside rows of 16
  kDppRowShr = 0x110,     // + n: lane i reads lane i - n of its row of 16 (0 if there is none)
};
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return static_cast<uint32_t>(dpp_i32<CTRL>(static_cast<int>(v)));
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(dpp_i32<CTRL>(__float_as_int(v)));
}
__device__ __forceinline__ float readlane_f32(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// Sum over the wavefront in a fixed order (pairs, quads, eights, rows of 16, then the four
// rows), the same value in every lane.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<kDppXor1>(v);
  v += dpp_f32<kDppXor2>(v);
  v += dpp_f32<kDppHalfMirror>(v);
  v += dpp_f32<kDppMirror>(v);
  return (readlane_f32(v, 0) + readlane_f32(v, 16)) + (readlane_f32(v, 32) + readlane_f32(v, 48));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  auto mx = [](uint32_t a, uint32_t b) { return a > b ? a : b; };
  v = mx(v, dpp_u32<kDppXor1>(v));
  v = mx(v, dpp_u32<kDppXor2>(v));
  v = mx(v, dpp_u32<kDppHalfMirror>(v));
  v = mx(v, dpp_u32<kDppMirror>(v));
  const int i = static_cast<int>(v);
  return mx(mx(static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 0)),
               static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 16))),
            mx(static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 32)),
               static_cast<uint32_t>(__builtin_amdgcn_readlane(i, 48))));
}
// Largest / smallest value over the wavefront (NaNs are ignored unless every lane holds one).
__device__ __forceinline__ float wave_max_f32(float v) {
  v = fmaxf(v, dpp_f32<kDppXor1>(v));
  v = fmaxf(v, dpp_f32<kDppXor2>(v));
  v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f32<kDppMirror>(v));
  return fmaxf(fmaxf(readlane_f32(v, 0), readlane_f32(v, 16)), fmaxf(readlane_f32(v, 32), readlane_f32(v, 48)));
}
__device__ __forceinline__ float wave_min_f32(float v) {
  v = fminf(v, dpp_f32<kDppXor1>(v));
  v = fminf(v, dpp_f32<kDppXor2>(v));
  v = fminf(v, dpp_f32<kDppHalfMirror>(v));
  v = fminf(v, dpp_f32<kDppMirror>(v));
  return fminf(fminf(readlane_f32(v, 0), readlane_f32(v, 16)), fminf(readlane_f32(v, 32), readlane_f32(v, 48)));
}
__device__ __forceinline__ int wave_sum_i32(int v) {
  v += dpp_i32<kDppXor1>(v);
  v += dpp_i32<kDppXor2>(v);
  v += dpp_i32<kDppHalfMirror>(v);
  v += dpp_i32<kDppMirror>(v);
  return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
         (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}
// Inclusive prefix sum over the lanes of the wavefront (lane = threadIdx.x % 64).
__device__ __forceinline__ int wave_inclusive_sum_i32(int v, int lane) {
  v += dpp_i32<kDppRowShr + 1>(v);
  v += dpp_i32<kDppRowShr + 2>(v);
  v += dpp_i32<kDppRowShr + 4>(v);
  v += dpp_i32<kDppRowShr + 8>(v);
  const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
            t2 = __builtin_amdgcn_readlane(v, 47);
  const int row = lane >> 4;
  return v + (row == 0 ? 0 : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2);
}
// Lexicographic minimum of (score, id) over the wavefront, in every lane.
__device__ __forceinline__ void wave_min_score_id(float& score, int& id) {
  auto take = [&](float os, int oi) {
    if (os < score || (os == score && oi < id)) {
      score = os;
      id = oi;
    }
  };
  take(dpp_f32<kDppXor1>(score), dpp_i32<kDppXor1>(id));
  take(dpp_f32<kDppXor2>(score), dpp_i32<kDppXor2>(id));
  take(dpp_f32<kDppHalfMirror>(score), dpp_i32<kDppHalfMirror>(id));
  take(dpp_f32<kDppMirror>(score), dpp_i32<kDppMirror>(id));
  const float s1 = readlane_f32(score, 16), s2 = readlane_f32(score, 32), s3 = readlane_f32(score, 48);
  const int i1 = __builtin_amdgcn_readlane(id, 16), i2 = __builtin_amdgcn_readlane(id, 32),
            i3 = __builtin_amdgcn_readlane(id, 48);
  score = readlane_f32(score, 0);
  id = __builtin_amdgcn_readlane(id, 0);
  take(s1, i1);
  take(s2, i2);
  take(s3, i3);
}

}  // namespace scd
