// First rejection, emission and window slide (appendix "Algorithms",
// Alg. SCD(pi_MC): "find first rejection index", i <- Accept + 1), plus the
// state initialisation ("p <- Random(), X ~ p": uniform initial drafts) and the
// copy of caller-supplied logits into the ring.
//
// Window of exactly L positions [i, i+L) clipped to N (Lw live rows).  With the
// first rejection at window offset r the step emits a = min(r+1, Lw) tokens
// (a = Lw when nothing was rejected).  Rows a..Lw-1 keep their MRS output as
// the next draft (coupled redraft) and age by one; rows 0..a-1 retire, and
// their ring slots receive the entering positions i+L .. i+L+a-1 (below N)
// with a uniform initial draft and age 0.
#include "scd_device.h"
#include "scd_kernels.h"

namespace scd {
namespace {

__global__ void commit_kernel(const CommitArgs a) {
  __shared__ int s_first;
  const int b = blockIdx.x;
  const int s = threadIdx.x;
  const int i = a.pos[b];
  const int live = max(0, min(a.L, a.N - i));
  if (s == 0) s_first = live;
  __syncthreads();
  if (live == 0) {
    if (s == 0) a.accept_len[b] = 0;
    return;
  }
  int y = -1;
  if (s < live) {
    y = a.y[static_cast<size_t>(b) * a.L + s];
    if (a.k[static_cast<size_t>(b) * a.L + s] == 0) atomicMin(&s_first, s);
  }
  __syncthreads();
  const int acc = min(s_first + 1, live);
  if (s < acc) a.out[static_cast<size_t>(b) * a.N + i + s] = a.v_lo + y;
  if (a.slide && s < live) {
    const size_t sidx = static_cast<size_t>(b) * a.L + (i + s) % a.L;
    if (s >= acc) {
      a.X[sidx] = y;
      a.age[sidx] += 1;
    } else {
      const int np = i + a.L + s;      // position entering this slot
      a.X[sidx] = np < a.N ? init_token(a.seed, b, np, a.n) : -1;
      a.age[sidx] = 0;
    }
  }
  if (s == 0) {
    a.accept_len[b] = acc;
    if (a.slide) {
      a.pos[b] = i + acc;
      a.iter[b] += 1;
      a.verified[b] += live;
    }
  }
}

__global__ void reset_kernel(const ResetArgs a) {
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;
  const int stride = gridDim.x * blockDim.x;
  for (size_t t = gid; t < static_cast<size_t>(a.B) * a.N; t += stride) a.out[t] = -1;
  for (int t = gid; t < a.B * a.L; t += stride) {
    const int b = t / a.L, slot = t % a.L;
    a.X[t] = slot < a.N ? init_token(a.seed, b, slot, a.n) : -1;
    a.age[t] = 0;
  }
  for (int t = gid; t < a.B; t += stride) {
    a.pos[t] = 0;
    a.iter[t] = 0;
    a.accept_len[t] = 0;
    a.verified[t] = 0;
    a.ticket[t] = 0;
  }
  for (int t = gid; t < 3 * a.B; t += stride) a.phist[t] = -(1 << 30);   // no earlier iteration
  if (gid < 4) a.flags[gid] = 0;
}

__global__ void copy_in_kernel(const CopyInArgs a) {
  const int r = blockIdx.x;
  const int b = r / a.L, s = r % a.L;
  const int p0 = a.pos[b];
  if (s >= min(a.L, a.N - p0)) return;
  const float* src = a.src + static_cast<size_t>(r) * a.n;
  float* dst = a.z + static_cast<size_t>(a.iter[b] & 1) * a.parity_stride +
               (static_cast<size_t>(b) * a.L + (p0 + s) % a.L) * a.n;
  for (int v = threadIdx.x; v < a.n; v += blockDim.x) dst[v] = src[v];
}

}  // namespace

hipError_t launch_commit(const CommitArgs& a, hipStream_t s) {
  const int threads = (a.L + 63) / 64 * 64;
  hipLaunchKernelGGL(commit_kernel, dim3(a.B), dim3(threads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_reset(const ResetArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(reset_kernel, dim3(256), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_copy_in(const CopyInArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(copy_in_kernel, dim3(a.B * a.L), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace scd
