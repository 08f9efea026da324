// Top-k threshold and softmax normaliser of one processed-logit row
// (logit post-processing that defines p^(t): Sec. 4.3, last sentence; top-k
// K = 2000 / 1000 and temperature in the appendix "Experimental Details").
//
//   thr  = K-th largest z   (exact order statistic; -inf when nothing is filtered)
//   kept = { v : z_v >= thr }   (ties with the K-th are all kept)
//   lse  = m + log( sum_kept exp(z_v - m) ),  m = max z
//   p_v  = [z_v >= thr] * exp(z_v - lse)      (never materialised)
//
// One workgroup per row.  The K-th largest value is found by a most-significant-
// digit radix select over order-preserving uint32 keys of the fp32 logits
// (12 + 10 + 10 bits): integer counting in an LDS histogram, no floating-point
// arithmetic, so the threshold is bit-exact.  The sum of exponentials uses a
// fixed per-thread order and a fixed reduction tree (run-to-run deterministic).
#include "scd_device.h"
#include "scd_kernels.h"

namespace scd {
namespace {

constexpr int THREADS = 1024;
constexpr int NW = THREADS / kWave;

struct RowShared {
  uint32_t hist[4096];
  uint32_t scan[THREADS];
  float fred[NW];
  uint32_t ured[NW];
  int ired[NW];
  uint32_t sel_bin;
  uint32_t sel_above;
};

// Among keys whose bits above `shift + bits` equal `prefix`, histogram the
// `bits`-wide digit at `shift`; find the digit holding the `need`-th largest
// such key.  Returns the digit and lowers `need` by the count of keys in higher
// digits.
template <int BITS>
__device__ void radix_pass(const float* __restrict__ row, int n, uint32_t prefix, int shift,
                           uint32_t& need, uint32_t& digit_out, RowShared& sh) {
  constexpr int NB = 1 << BITS;
  const int tid = threadIdx.x;
  for (int i = tid; i < NB; i += THREADS) sh.hist[i] = 0;
  __syncthreads();
  const int hi_shift = shift + BITS;
  for (int i = tid; i < n; i += THREADS) {
    const uint32_t key = float_to_key(row[i]);
    const bool match = hi_shift >= 32 ? true : ((key >> hi_shift) == (prefix >> hi_shift));
    if (match) atomicAdd(&sh.hist[(key >> shift) & (NB - 1)], 1u);
  }
  __syncthreads();
  // Each thread owns PER consecutive digits, highest digits in thread 0.
  constexpr int PER = (NB + THREADS - 1) / THREADS;
  uint32_t local = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int dgt = NB - 1 - (tid * PER + j);
    if (dgt >= 0) local += sh.hist[dgt];
  }
  // inclusive scan over threads (thread 0 = highest digits)
  sh.scan[tid] = local;
  __syncthreads();
  for (int o = 1; o < THREADS; o <<= 1) {
    const uint32_t add = tid >= o ? sh.scan[tid - o] : 0u;
    __syncthreads();
    sh.scan[tid] += add;
    __syncthreads();
  }
  const uint32_t incl = sh.scan[tid];
  const uint32_t excl = incl - local;
  if (excl < need && need <= incl) {   // exactly one thread
    uint32_t above = excl;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int dgt = NB - 1 - (tid * PER + j);
      if (dgt < 0) break;
      const uint32_t c = sh.hist[dgt];
      if (above + c >= need) {
        sh.sel_bin = static_cast<uint32_t>(dgt);
        sh.sel_above = above;
        break;
      }
      above += c;
    }
  }
  __syncthreads();
  digit_out = sh.sel_bin;
  need -= sh.sel_above;
  __syncthreads();
}

__global__ __launch_bounds__(THREADS) void select_kernel(const SelectArgs a) {
  __shared__ RowShared sh;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r = blockIdx.x;
  const float* row;
  size_t oidx;
  if (a.pos) {                       // ring mode: r = b*L + s over live window rows
    const int b = r / a.L, s = r % a.L;
    const int p0 = a.pos[b];
    if (s >= min(a.L, a.N - p0)) return;
    const int par = a.iter[b] & 1;
    const int slot = (p0 + s) % a.L;
    oidx = (static_cast<size_t>(par) * a.B + b) * a.L + slot;
    row = a.z + static_cast<size_t>(par) * a.parity_stride +
          (static_cast<size_t>(b) * a.L + slot) * a.n;
  } else {
    oidx = r;
    row = a.z + static_cast<size_t>(r) * a.n;
  }
  const int n = a.n;

  // row maximum (as key: integer max is exact and order-independent)
  uint32_t kmax = 0;
  for (int i = tid; i < n; i += THREADS) {
    const uint32_t key = float_to_key(row[i]);
    kmax = key > kmax ? key : kmax;
  }
  kmax = wave_max_u32(kmax);
  if (lane == 0) sh.ured[wave] = kmax;
  __syncthreads();
  kmax = sh.ured[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) kmax = sh.ured[w] > kmax ? sh.ured[w] : kmax;
  const float m = key_to_float(kmax);
  __syncthreads();

  uint32_t thr_key = 0;               // below every key: keep all
  const bool filter = a.top_k > 0 && a.top_k < n;
  if (filter) {
    uint32_t need = static_cast<uint32_t>(a.top_k), dgt;
    radix_pass<12>(row, n, 0u, 20, need, dgt, sh);
    thr_key = dgt << 20;
    radix_pass<10>(row, n, thr_key, 10, need, dgt, sh);
    thr_key |= dgt << 10;
    radix_pass<10>(row, n, thr_key, 0, need, dgt, sh);
    thr_key |= dgt;
  }

  // membership is the FLOAT comparison z >= thr (so -0 and +0 tie, as in the
  // definition of the kept set)
  const float thr = filter ? key_to_float(thr_key) : -INFINITY;
  float sum = 0.f;
  int cnt = 0;
  for (int i = tid; i < n; i += THREADS) {
    const float z = row[i];
    if (z >= thr) {
      sum += expf(z - m);
      ++cnt;
    }
  }
  sum = wave_sum(sum);
  cnt = wave_sum_i32(cnt);
  if (lane == 0) {
    sh.fred[wave] = sum;
    sh.ired[wave] = cnt;
  }
  __syncthreads();
  if (tid == 0) {
    float S = 0.f;
    int Cn = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      S += sh.fred[w];
      Cn += sh.ired[w];
    }
    const float lse = m + logf(S);
    a.thr[oidx] = thr;
    a.lse[oidx] = lse;
    a.nkept[oidx] = Cn;
    if (a.flags && !(lse == lse && fabsf(lse) < INFINITY)) atomicOr(a.flags, 1);
  }
}

}  // namespace

hipError_t launch_select(const SelectArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(select_kernel, dim3(a.rows), dim3(THREADS), 0, s, a);
  return hipGetLastError();
}

}  // namespace scd
