// Vectorised Modified Rejection Sampling: one MRS(p, q, x) call per window
// position, no break (Alg. 1; appendix "Algorithms", Alg. SCD(pi_MC),
// "Verify & Drafting with Vectorized MRS").  Left of the first rejection the
// call is the speculative verification, at it the residual resample, right of
// it the maximal-coupling redraft of the next iteration's draft (Sec. 4.1,
// Thm 4.3): the same kernel serves all three.
//
//   u ~ U(0,1) keyed on (seed, b, position, iteration)
//   accept  iff  fl(u * q(x)) <= p(x)         (no division; u in (0,1))
//   else    y = argmin over { v : r_v > 0 } of  -ln(U_v) / r_v,
//           r_v = p_v - q_v, U_v keyed additionally on v  (exponential race:
//           picks v with probability r_v / sum r, needs no normaliser and no
//           ordered scan; ties go to the lowest id)
//   p_v = [z_v >= thr] * exp(z_v - lse)  from this iteration's processed logits,
//   q_v likewise from the previous iteration's, or 1/n for a position that was
//   never evaluated.
//
// One workgroup per window position.  Accepting rows exit after two gathered
// loads; rejected rows stream the two logit rows once with 16-byte loads.
#include "scd_device.h"
#include "scd_kernels.h"

namespace scd {
namespace {

constexpr int THREADS = 1024;
constexpr int NW = THREADS / kWave;

__device__ __forceinline__ float prob(float z, float thr, float lse) {
  return z >= thr ? expf(z - lse) : 0.f;
}

__global__ __launch_bounds__(THREADS) void mrs_kernel(const MrsArgs a) {
  __shared__ float s_score[NW];
  __shared__ int s_id[NW];
  const int tid = threadIdx.x;
  const int b = blockIdx.x / a.L, s = blockIdx.x % a.L;
  const int p0 = a.pos[b];
  const int live = min(a.L, a.N - p0);
  const size_t widx = static_cast<size_t>(b) * a.L + s;   // window-order index
  if (s >= live) {
    if (tid == 0) {
      a.y[widx] = -1;
      a.k[widx] = 1;
      if (a.px) a.px[widx] = 0.f;
      if (a.qx) a.qx[widx] = 0.f;
    }
    return;
  }
  const int j = p0 + s;
  const int n = a.n;
  int it, x;
  bool fresh;
  const float *zc, *zp;
  float thr_c, lse_c, thr_p = 0.f, lse_p = 0.f;
  if (a.ring) {
    it = a.iter[b];
    const int par = it & 1;
    const size_t sidx = static_cast<size_t>(b) * a.L + (j % a.L);
    const size_t half = static_cast<size_t>(a.B) * a.L;
    x = a.x[sidx];
    fresh = a.age[sidx] == 0;
    zc = a.z_cur + static_cast<size_t>(par) * a.parity_stride + sidx * n;
    zp = a.z_cur + static_cast<size_t>(par ^ 1) * a.parity_stride + sidx * n;
    thr_c = a.thr_cur[par * half + sidx];
    lse_c = a.lse_cur[par * half + sidx];
    if (!fresh) {
      thr_p = a.thr_cur[(par ^ 1) * half + sidx];
      lse_p = a.lse_cur[(par ^ 1) * half + sidx];
    }
  } else {
    it = a.iter_scalar;
    x = a.x[widx];
    fresh = a.fresh ? a.fresh[widx] != 0 : false;
    zc = a.z_cur + widx * n;
    zp = a.z_prev + widx * n;
    thr_c = a.thr_cur[widx];
    lse_c = a.lse_cur[widx];
    if (!fresh) {
      thr_p = a.thr_prev[widx];
      lse_p = a.lse_prev[widx];
    }
  }
  const float q_uniform = __fdiv_rn(1.0f, static_cast<float>(n));
  const uint2 key = seed_key(a.seed);
  const uint32_t w3 = static_cast<uint32_t>(b) << 8;

  // ---- accept test (every thread computes the same values) ----------------
  const bool x_ok = x >= 0 && x < n;
  const float px = x_ok ? prob(zc[x], thr_c, lse_c) : 0.f;
  const float qx = fresh ? q_uniform : (x_ok ? prob(zp[x], thr_p, lse_p) : 0.f);
  const uint4 ra = philox4x32_10(make_uint4(0u, static_cast<uint32_t>(j), static_cast<uint32_t>(it),
                                            w3 | kStreamAccept), key);
  const float u = u01(ra.x);
  const bool accept = __fmul_rn(u, qx) <= px;
  if (tid == 0) {
    if (a.px) a.px[widx] = px;
    if (a.qx) a.qx[widx] = qx;
  }
  if (accept) {
    if (tid == 0) {
      a.y[widx] = x;
      a.k[widx] = 1;
    }
    return;
  }

  // ---- residual resample: exponential race over r = max(0, p - q) ----------
  float best = INFINITY;
  int best_id = 0x7FFFFFFF;
  const bool vec_ok = (n & 3) == 0;    // rows are 16-byte aligned iff n % 4 == 0
  const int ngroups = (n + 3) >> 2;
  for (int g = tid; g < ngroups; g += THREADS) {
    const int v0 = g << 2;
    float c4[4], p4[4] = {0.f, 0.f, 0.f, 0.f};
    if (vec_ok) {
      const float4 t = *reinterpret_cast<const float4*>(zc + v0);
      c4[0] = t.x; c4[1] = t.y; c4[2] = t.z; c4[3] = t.w;
      if (!fresh) {
        const float4 t2 = *reinterpret_cast<const float4*>(zp + v0);
        p4[0] = t2.x; p4[1] = t2.y; p4[2] = t2.z; p4[3] = t2.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool in = v0 + e < n;
        c4[e] = in ? zc[v0 + e] : -INFINITY;
        if (!fresh) p4[e] = in ? zp[v0 + e] : -INFINITY;
      }
    }
    float r4[4];
    bool any = false;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float pv = (v0 + e < n) ? prob(c4[e], thr_c, lse_c) : 0.f;
      const float qv = fresh ? q_uniform : prob(p4[e], thr_p, lse_p);
      r4[e] = __fsub_rn(pv, qv);
      any |= r4[e] > 0.f;
    }
    if (!any) continue;
    const uint4 rr = philox4x32_10(make_uint4(static_cast<uint32_t>(g), static_cast<uint32_t>(j),
                                              static_cast<uint32_t>(it), w3 | kStreamResid), key);
    const uint32_t bits[4] = {rr.x, rr.y, rr.z, rr.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (r4[e] > 0.f) {
        const float sc = __fdiv_rn(-logf(u01(bits[e])), r4[e]);
        // ids increase within a thread, so strict '<' keeps the lowest id on ties
        if (sc < best) {
          best = sc;
          best_id = v0 + e;
        }
      }
    }
  }
  // lexicographic (score, id) minimum over the workgroup
  wave_min_score_id(best, best_id);
  if ((tid & 63) == 0) {
    s_score[tid >> 6] = best;
    s_id[tid >> 6] = best_id;
  }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < NW; ++w) {
      if (s_score[w] < best || (s_score[w] == best && s_id[w] < best_id)) {
        best = s_score[w];
        best_id = s_id[w];
      }
    }
    if (best_id == 0x7FFFFFFF) {     // empty residual (rounding only): counts as accept
      a.y[widx] = x;
      a.k[widx] = 1;
    } else {
      a.y[widx] = best_id;
      a.k[widx] = 0;
    }
  }
}

}  // namespace

hipError_t launch_mrs(const MrsArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(mrs_kernel, dim3(a.B * a.L), dim3(THREADS), 0, s, a);
  return hipGetLastError();
}

}  // namespace scd
