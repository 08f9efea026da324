// Device-side helpers shared by the gfx950 kernels of the SCD step:
// Philox4x32-10 (Salmon et al., SC'11), the 23-bit uniform mapping, the
// order-preserving float <-> uint32 key map used by the radix select, and
// block-wide reductions for 64-lane wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace scd {

constexpr int kWave = 64;

enum : uint32_t { kStreamInit = 0, kStreamAccept = 1, kStreamResid = 2 };

__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
    c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
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

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t w = static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), o, kWave));
    v = w > v ? w : v;
  }
  return v;
}
__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

}  // namespace scd
