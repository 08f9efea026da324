// Benchmark plumbing only (not the decoding method): gathers the hidden-state
// rows of the current windows from a pre-generated [B, C, N, age_cap+1, d]
// table on the device.  Pure 16-byte copies.
#include "../../include/scd_workload.h"

#include <hip/hip_runtime.h>

namespace {
__global__ void gather_kernel(const uint4* __restrict__ table, int B, int C, int L, int N, int d8,
                              int age_cap, const int32_t* __restrict__ pos,
                              const int32_t* __restrict__ age, uint4* __restrict__ h) {
  const int row = blockIdx.x;                 // (b*C + c)*L + s
  const int s = row % L, bc = row / L, b = bc / C;
  const int p = pos[b] + s;
  uint4* dst = h + static_cast<size_t>(row) * d8;
  if (p >= N) {
    for (int i = threadIdx.x; i < d8; i += blockDim.x) dst[i] = make_uint4(0, 0, 0, 0);
    return;
  }
  const int a = min(age[b * L + p % L], age_cap);
  const uint4* src = table + ((static_cast<size_t>(bc) * N + p) * (age_cap + 1) + a) * d8;
  for (int i = threadIdx.x; i < d8; i += blockDim.x) dst[i] = src[i];
}

__global__ void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride)
    dst[i] = src[i];
}
}  // namespace

extern "C" int scdw_copy(void* hip_stream, const void* d_src, void* d_dst, size_t bytes) {
  if (!d_src || !d_dst || bytes == 0 || (bytes & 15)) return -1;
  if ((reinterpret_cast<uintptr_t>(d_src) | reinterpret_cast<uintptr_t>(d_dst)) & 15) return -1;
  hipLaunchKernelGGL(copy_kernel, dim3(2048), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(d_src), static_cast<uint4*>(d_dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

extern "C" int scdw_gather_hidden(void* hip_stream, const uint16_t* d_table, int32_t B, int32_t C,
                                  int32_t L, int32_t N, int32_t d, int32_t age_cap,
                                  const int32_t* d_pos, const int32_t* d_age, uint16_t* d_h) {
  if (!d_table || !d_pos || !d_age || !d_h || B < 1 || C < 1 || L < 1 || N < 1 || d < 8 ||
      (d % 8) != 0 || age_cap < 0)
    return -1;
  if ((reinterpret_cast<uintptr_t>(d_table) | reinterpret_cast<uintptr_t>(d_h)) & 15) return -1;
  hipLaunchKernelGGL(gather_kernel, dim3(B * C * L), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream),
                     reinterpret_cast<const uint4*>(d_table), B, C, L, N, d / 8, age_cap, d_pos,
                     d_age, reinterpret_cast<uint4*>(d_h));
  return hipGetLastError() == hipSuccess ? 0 : -3;
}
