// Fused per-row kernel of the SCD step: top-k threshold, softmax normaliser,
// Modified Rejection Sampling (accept test + residual resample) and -- through
// a last-arriver ticket per sequence -- first rejection, emission and window
// slide.  (Alg. 1; Sec. 4.3 "vectorizing verification loop without break and
// saving the index where the first rejection occurs"; appendix "Algorithms",
// Alg. SCD(pi_MC); top-k / temperature from the appendix "Experimental
// Details".)
//
//   thr  = K-th largest z (exact),  kept = { v : z_v >= thr }
//   lse  = m + log sum_kept exp(z_v - m),  p_v = [z_v >= thr] exp(z_v - lse)
//   accept iff fl(u * q(x)) <= p(x);  else y = argmin_{r_v > 0} -ln(U_v) / r_v
//
// gfx950 mapping.  One workgroup (16 wavefronts) per window position.  The row
// is read from memory ONCE, coalesced: the upper 16 bits of each logit's
// order-preserving key are parked in LDS (2 bytes per id, 128 KB for 65536
// ids).  Everything after that works on the LDS copy:
//   * the K-th largest 16-bit prefix by counting in an LDS histogram whose bins
//     are (prefix - min) >> s, i.e. spread over the row's actual range, so that
//     lanes rarely collide on a bin;
//   * the low 16 bits of the threshold, the sum of exponentials and the
//     residual race touch memory only for ids whose prefix is >= the
//     threshold's (about K of n ids).
// All counting is integer, all floating-point sums use a fixed assignment of
// ids to threads and a fixed reduction tree: results are run-to-run identical.
#include "scd_device.h"
#include "scd_kernels.h"

namespace scd {
namespace {

constexpr int THREADS = 1024;
constexpr int NW = THREADS / kWave;
constexpr int NBINS = 4096;
constexpr int kListCap = 6144;     // candidate ids kept in LDS (uint16 each)

struct Small {
  float fred[NW];
  uint32_t ured[NW];
  uint32_t umin[NW];
  uint32_t umax[NW];
  int ired[NW];
  uint32_t wtot[NW];
  uint32_t sel_bin, sel_above;
  float s_score[NW];
  int s_id[NW];
  int last;
  int first_rej;
};

// key with -0 folded onto +0, so that key order == float order for non-NaNs
__device__ __forceinline__ uint32_t zkey(float f) { return float_to_key(f == 0.f ? 0.f : f); }

// hist[0..NBINS): find the bin holding the `need`-th largest element counting
// from the top bin; lowers `need` by the population of the bins above it.
__device__ __forceinline__ uint32_t find_bin(const uint32_t* hist, uint32_t& need, Small& sm) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int PER = NBINS / THREADS;   // 4 consecutive bins per thread, top bins in thread 0
  uint32_t c[PER], local = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    c[j] = hist[NBINS - 1 - (tid * PER + j)];
    local += c[j];
  }
  uint32_t incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = static_cast<uint32_t>(__shfl_up(static_cast<int>(incl), o, kWave));
    if (lane >= o) incl += t;
  }
  if (lane == 63) sm.wtot[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += sm.wtot[w];
  incl += base;
  const uint32_t excl = incl - local;
  if (excl < need && need <= incl) {     // exactly one thread
    uint32_t above = excl;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (above + c[j] >= need) {
        sm.sel_bin = static_cast<uint32_t>(NBINS - 1 - (tid * PER + j));
        sm.sel_above = above;
        break;
      }
      above += c[j];
    }
  }
  __syncthreads();
  const uint32_t bin = sm.sel_bin;
  need -= sm.sel_above;
  __syncthreads();
  return bin;
}

__device__ __forceinline__ void zero_hist(uint32_t* hist) {
#pragma unroll
  for (int j = 0; j < NBINS / THREADS; ++j) hist[threadIdx.x + j * THREADS] = 0u;
}

__device__ __forceinline__ float prob(float z, float thr, float lse) {
  return z >= thr ? expf(z - lse) : 0.f;
}

__global__ __launch_bounds__(THREADS) void row_kernel(const RowArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ Small sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = a.n;
  const int n8 = (n + 7) & ~7;                       // prefix array padded to 8 entries
  uint16_t* k16 = reinterpret_cast<uint16_t*>(smem);
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + static_cast<size_t>(n8) * 2);
  uint16_t* list = reinterpret_cast<uint16_t*>(smem + static_cast<size_t>(n8) * 2 + NBINS * 4);

  // ---- which row ---------------------------------------------------------
  const int r = blockIdx.x;
  int b = 0, s = 0, p0 = 0, live = 0, it = a.iter_scalar;
  size_t widx = r, oidx = r;
  const float* zc;
  const float* zp = nullptr;
  float thr_p = 0.f, lse_p = 0.f;
  bool fresh = false;
  int x = -1;
  if (a.mode == kRowSelectOnly) {
    zc = a.z_cur + static_cast<size_t>(r) * n;
  } else {
    b = r / a.L;
    s = r % a.L;
    p0 = a.pos[b];
    live = max(0, min(a.L, a.N - p0));
    widx = static_cast<size_t>(b) * a.L + s;
    if (s >= live) {
      if (tid == 0) {
        a.y[widx] = -1;
        a.k[widx] = 1;
        if (a.px) a.px[widx] = 0.f;
        if (a.qx) a.qx[widx] = 0.f;
        if (a.mode == kRowRing && s == 0) a.accept_len[b] = 0;   // finished sequence
      }
      return;
    }
    if (a.mode == kRowRing) {
      it = a.iter[b];
      const int par = it & 1;
      const size_t sidx = static_cast<size_t>(b) * a.L + (p0 + s) % a.L;
      const size_t half = static_cast<size_t>(a.B) * a.L;
      oidx = par * half + sidx;
      x = a.x[sidx];
      fresh = a.age[sidx] == 0;
      zc = a.z_cur + static_cast<size_t>(par) * a.parity_stride + sidx * n;
      zp = a.z_cur + static_cast<size_t>(par ^ 1) * a.parity_stride + sidx * n;
      if (!fresh) {
        thr_p = a.thr[(par ^ 1) * half + sidx];
        lse_p = a.lse[(par ^ 1) * half + sidx];
      }
    } else {
      oidx = widx;
      x = a.x[widx];
      fresh = a.fresh ? a.fresh[widx] != 0 : false;
      zc = a.z_cur + widx * n;
      zp = a.z_prev + widx * n;
      if (!fresh) {
        thr_p = a.thr_prev[widx];
        lse_p = a.lse_prev[widx];
      }
    }
  }

  // Prefetch the two logits of the draft token so that their latency hides
  // behind the row pass.
  const bool x_ok = a.mode != kRowSelectOnly && x >= 0 && x < n;
  const float zcx = x_ok ? zc[x] : 0.f;
  const float zpx = (x_ok && !fresh) ? zp[x] : 0.f;

  // ---- pass 1: the only full read of the row ------------------------------
  // Batches of 8 independent 16-byte loads per thread keep 128 KB in flight.
  const bool vec_ok = (n & 3) == 0;
  const int ngroups = (n + 3) >> 2;          // groups of 4 ids holding at least one id
  const int ngroups8 = n8 >> 2;              // groups covering the padded LDS array
  uint32_t kmax = 0, p16min = 0xFFFFu, p16max = 0u;
  constexpr int UNR = 8;
  for (int g0 = tid; g0 < ngroups8; g0 += THREADS * UNR) {
    float f[UNR][4];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int g = g0 + u * THREADS;
      const int v0 = g << 2;
      if (vec_ok && g < ngroups) {
        const float4 t = *reinterpret_cast<const float4*>(zc + v0);
        f[u][0] = t.x; f[u][1] = t.y; f[u][2] = t.z; f[u][3] = t.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) f[u][e] = (v0 + e < n) ? zc[v0 + e] : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int g = g0 + u * THREADS;
      if (g < ngroups8) {
        const int v0 = g << 2;
        uint32_t h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t key = zkey(f[u][e]);
          h[e] = key >> 16;
          if (v0 + e < n) {
            kmax = key > kmax ? key : kmax;
            p16min = h[e] < p16min ? h[e] : p16min;
            p16max = h[e] > p16max ? h[e] : p16max;
          }
        }
        *reinterpret_cast<uint2*>(&k16[v0]) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
      }
    }
  }
  kmax = wave_max_u32(kmax);
  p16max = wave_max_u32(p16max);
  p16min = ~wave_max_u32(~p16min);
  if (lane == 0) {
    sm.ured[wave] = kmax;
    sm.umax[wave] = p16max;
    sm.umin[wave] = p16min;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    kmax = sm.ured[w] > kmax ? sm.ured[w] : kmax;
    p16max = sm.umax[w] > p16max ? sm.umax[w] : p16max;
    p16min = sm.umin[w] < p16min ? sm.umin[w] : p16min;
  }
  const float m = key_to_float(kmax);

  // Each thread owns the 8-id chunks c = tid, tid + THREADS, ... of the LDS copy.
  const int nchunks = n8 >> 3;
  const bool filter = a.top_k > 0 && a.top_k < n;
  const uint32_t K = static_cast<uint32_t>(a.top_k);

  // prefix histogram over chunks [0, upto): bins = (prefix - min) >> sh, optionally
  // only the prefixes that fall into bin `only` (then the bins are the sh low bits)
  const uint32_t range = p16max - p16min;
  int sh = 0;
  while ((range >> sh) >= static_cast<uint32_t>(NBINS)) ++sh;
  auto prefix_hist = [&](int upto, bool low_bits, uint32_t only) {
    zero_hist(hist);
    __syncthreads();
    const uint32_t mask = (1u << sh) - 1u;
    for (int c = tid; c < upto; c += THREADS) {
      const uint4 raw = *reinterpret_cast<const uint4*>(&k16[c << 3]);
      const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if ((c << 3) + e < n) {
          const uint32_t p = ((w4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu) - p16min;
          if (!low_bits) atomicAdd(&hist[p >> sh], 1u);
          else if ((p >> sh) == only) atomicAdd(&hist[p & mask], 1u);
        }
      }
    }
    __syncthreads();
  };
  // number of ids whose prefix is >= lowp: this thread's share, its exclusive
  // offset in a fixed order, and the total
  int my_cnt = 0, my_off = 0, ncand = 0;
  auto count_ge = [&](uint32_t lowp) {
    my_cnt = 0;
    for (int c = tid; c < nchunks; c += THREADS) {
      const uint4 raw = *reinterpret_cast<const uint4*>(&k16[c << 3]);
      const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t p = (w4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
        my_cnt += ((c << 3) + e < n && p >= lowp) ? 1 : 0;
      }
    }
    int incl = my_cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o, kWave);
      if (lane >= o) incl += t;
    }
    if (lane == 63) sm.ired[wave] = incl;
    __syncthreads();
    int base = 0;
    ncand = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      base += w < wave ? sm.ired[w] : 0;
      ncand += sm.ired[w];
    }
    my_off = base + incl - my_cnt;
    __syncthreads();
  };

  // ---- a prefix bound `lowp` with K <= #{prefix >= lowp} -----------------------
  uint32_t t16 = 0;         // exact 16-bit prefix of the threshold key (when computed)
  uint32_t need_ab = K;     // rank still to resolve below t16's bin (in-place path)
  bool exact16 = false;
  uint32_t lowp = 0;
  auto exact_prefix = [&]() {   // full histogram: exact 16-bit prefix of the K-th largest
    need_ab = K;
    prefix_hist(nchunks, false, 0u);
    const uint32_t binA = find_bin(hist, need_ab, sm);
    uint32_t low = 0;
    if (sh > 0) {
      prefix_hist(nchunks, true, binA);
      low = find_bin(hist, need_ab, sm);
    }
    t16 = p16min + (binA << sh) + low;
    exact16 = true;
  };
  bool use_list = false;
  if (filter) {
    if (nchunks <= THREADS) {
      exact_prefix();
      lowp = t16;
      count_ge(lowp);
    } else {
      // The first THREADS chunks (8192 ids) act as a sample: the prefix bin of the
      // sample's element of rank ~2K * 8192 / n is, almost always, a lower bound of
      // the K-th largest of the row with about 2K ids above it.  The bound is
      // verified by counting; if it fails the full histogram decides.
      prefix_hist(THREADS, false, 0u);
      const uint64_t target = min(static_cast<uint64_t>(2) * K, (static_cast<uint64_t>(K) + kListCap) / 2);
      uint32_t ks = static_cast<uint32_t>(target * (THREADS * 8) / n);
      ks = ks < 1 ? 1 : ks;
      const uint32_t bs = find_bin(hist, ks, sm);
      lowp = p16min + (bs << sh);
      count_ge(lowp);
      if (ncand < static_cast<int>(K) || ncand > kListCap) {
        exact_prefix();
        lowp = t16;
        count_ge(lowp);
      }
    }
    use_list = ncand <= kListCap;
  }

  float thr = -INFINITY;
  float sum = 0.f;
  int cnt = 0;
  float best = INFINITY;        // residual race
  int best_id = 0x7FFFFFFF;
  const int j = p0 + s;
  const float q_uniform = __fdiv_rn(1.0f, static_cast<float>(n));
  const uint2 key = seed_key(a.seed);
  const uint32_t w3 = static_cast<uint32_t>(b) << 8;
  bool accept = true;
  float px = 0.f, qx = 0.f;
  auto race_one = [&](int v, float rv) {   // exponential race entry of id v with residual rv > 0
    const uint4 rr = philox4x32_10(make_uint4(static_cast<uint32_t>(v >> 2), static_cast<uint32_t>(j),
                                              static_cast<uint32_t>(it), w3 | kStreamResid), key);
    const uint32_t lanes[4] = {rr.x, rr.y, rr.z, rr.w};
    const float sc = __fdiv_rn(-logf(u01(lanes[v & 3])), rv);
    if (sc < best || (sc == best && v < best_id)) {
      best = sc;
      best_id = v;
    }
  };
  auto accept_test = [&](float thr_c, float lse_c) {
    px = x_ok ? prob(zcx, thr_c, lse_c) : 0.f;
    qx = fresh ? q_uniform : (x_ok ? prob(zpx, thr_p, lse_p) : 0.f);
    const uint4 ra = philox4x32_10(make_uint4(0u, static_cast<uint32_t>(j), static_cast<uint32_t>(it),
                                              w3 | kStreamAccept), key);
    accept = __fmul_rn(u01(ra.x), qx) <= px;
  };
  float lse_c;

  if (use_list) {
    // ======== candidates in registers: at most kListCap / THREADS = 6 per thread ====
    constexpr int PER = kListCap / THREADS;
    {
      int o = my_off;
      for (int c = tid; c < nchunks; c += THREADS) {
        const uint4 raw = *reinterpret_cast<const uint4*>(&k16[c << 3]);
        const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t p = (w4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
          if ((c << 3) + e < n && p >= lowp) list[o++] = static_cast<uint16_t>((c << 3) + e);
        }
      }
    }
    __syncthreads();
    int vid[PER];
    float zv[PER];
    uint32_t kv[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int i = tid + e * THREADS;
      vid[e] = i < ncand ? static_cast<int>(list[i]) : -1;
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) zv[e] = vid[e] >= 0 ? zc[vid[e]] : 0.f;
#pragma unroll
    for (int e = 0; e < PER; ++e) kv[e] = zkey(zv[e]);
    // K-th largest key among the candidates: range-adaptive radix levels
    uint32_t lo = lowp << 16;
    uint64_t width = static_cast<uint64_t>(kmax) - lo + 1;
    uint32_t need = K;
    for (;;) {
      int s2 = 0;
      while (((width - 1) >> s2) >= static_cast<uint64_t>(NBINS)) ++s2;
      zero_hist(hist);
      __syncthreads();
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        if (vid[e] >= 0 && kv[e] >= lo && static_cast<uint64_t>(kv[e] - lo) < width)
          atomicAdd(&hist[(kv[e] - lo) >> s2], 1u);
      }
      __syncthreads();
      const uint32_t dgt = find_bin(hist, need, sm);
      lo += dgt << s2;
      width = 1ull << s2;
      if (s2 == 0) break;
    }
    thr = key_to_float(lo);
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (vid[e] >= 0 && zv[e] >= thr) {
        sum += expf(zv[e] - m);
        ++cnt;
      }
    }
    sum = wave_sum(sum);
    cnt = wave_sum_i32(cnt);
    if (lane == 0) {
      sm.fred[wave] = sum;
      sm.ired[wave] = cnt;
    }
    __syncthreads();
    float S = 0.f;
    int Cn = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      S += sm.fred[w];
      Cn += sm.ired[w];
    }
    lse_c = m + logf(S);
    if (tid == 0) {
      a.thr[oidx] = thr;
      a.lse[oidx] = lse_c;
      a.nkept[oidx] = Cn;
      if (a.flags && !(lse_c == lse_c && fabsf(lse_c) < INFINITY)) atomicOr(a.flags, 1);
    }
    if (a.mode == kRowSelectOnly) return;
    accept_test(thr, lse_c);
    if (!accept) {     // uniform over the workgroup
      float zq[PER];
#pragma unroll
      for (int e = 0; e < PER; ++e)
        zq[e] = (!fresh && vid[e] >= 0 && zv[e] >= thr) ? zp[vid[e]] : 0.f;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        if (vid[e] >= 0 && zv[e] >= thr) {
          const float pv = expf(zv[e] - lse_c);
          const float qv = fresh ? q_uniform : prob(zq[e], thr_p, lse_p);
          const float rv = __fsub_rn(pv, qv);
          if (rv > 0.f) race_one(vid[e], rv);
        }
      }
    }
  } else {
    // ======== in place: no filter, or the candidates do not fit (massive ties) ======
    if (filter && !exact16) exact_prefix();
    auto for_each_candidate = [&](auto&& f) {
      for (int c = tid; c < nchunks; c += THREADS) {
        const uint4 raw = *reinterpret_cast<const uint4*>(&k16[c << 3]);
        const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int v = (c << 3) + e;
          const uint32_t p = (w4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
          if (v < n && (!filter || p >= t16)) f(v, p);
        }
      }
    };
    if (filter) {
      // low 16 bits of the threshold key: two 8-bit digits over the ids whose prefix is t16
      uint32_t lowkey = 0;
#pragma unroll
      for (int pass = 0; pass < 2; ++pass) {
        zero_hist(hist);
        __syncthreads();
        const int shift = pass == 0 ? 8 : 0;
        for_each_candidate([&](int v, uint32_t p) {
          if (p == t16) {
            const uint32_t kk = zkey(zc[v]) & 0xFFFFu;
            if (pass == 0 || (kk >> 8) == (lowkey >> 8)) atomicAdd(&hist[(kk >> shift) & 0xFFu], 1u);
          }
        });
        __syncthreads();
        lowkey |= find_bin(hist, need_ab, sm) << shift;
      }
      thr = key_to_float((t16 << 16) | lowkey);
    }
    for_each_candidate([&](int v, uint32_t) {
      const float z = zc[v];
      if (z >= thr) {
        sum += expf(z - m);
        ++cnt;
      }
    });
    sum = wave_sum(sum);
    cnt = wave_sum_i32(cnt);
    if (lane == 0) {
      sm.fred[wave] = sum;
      sm.ired[wave] = cnt;
    }
    __syncthreads();
    float S = 0.f;
    int Cn = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      S += sm.fred[w];
      Cn += sm.ired[w];
    }
    lse_c = m + logf(S);
    if (tid == 0) {
      a.thr[oidx] = thr;
      a.lse[oidx] = lse_c;
      a.nkept[oidx] = Cn;
      if (a.flags && !(lse_c == lse_c && fabsf(lse_c) < INFINITY)) atomicOr(a.flags, 1);
    }
    if (a.mode == kRowSelectOnly) return;
    accept_test(thr, lse_c);
    if (!accept) {
      for_each_candidate([&](int v, uint32_t) {
        const float pv = prob(zc[v], thr, lse_c);
        if (pv > 0.f) {
          const float qv = fresh ? q_uniform : prob(zp[v], thr_p, lse_p);
          const float rv = __fsub_rn(pv, qv);
          if (rv > 0.f) race_one(v, rv);
        }
      });
    }
  }

  // ---- winner of the race (lexicographic (score, id) minimum) -------------------
  int y_out = x;
  int k_out = 1;
  if (!accept) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float os = __shfl_xor(best, o, kWave);
      const int oi = __shfl_xor(best_id, o, kWave);
      if (os < best || (os == best && oi < best_id)) {
        best = os;
        best_id = oi;
      }
    }
    if (lane == 0) {
      sm.s_score[wave] = best;
      sm.s_id[wave] = best_id;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      if (sm.s_score[w] < best || (sm.s_score[w] == best && sm.s_id[w] < best_id)) {
        best = sm.s_score[w];
        best_id = sm.s_id[w];
      }
    }
    if (best_id != 0x7FFFFFFF) {   // else: empty residual (rounding only) counts as accept
      y_out = best_id;
      k_out = 0;
    }
  }
  if (tid == 0) {
    a.y[widx] = y_out;
    a.k[widx] = static_cast<uint8_t>(k_out);
    if (a.px) a.px[widx] = px;
    if (a.qx) a.qx[widx] = qx;
  }
  if (a.mode != kRowRing) return;

  // ---- last workgroup of the sequence: first rejection, emit, slide -----------
  if (tid == 0) {
    __threadfence();
    sm.last = atomicAdd(&a.ticket[b], 1) == live - 1;
    sm.first_rej = live;
  }
  __syncthreads();
  if (!sm.last) return;
  __threadfence();
  const volatile int32_t* vy = a.y + static_cast<size_t>(b) * a.L;
  const volatile uint8_t* vk = a.k + static_cast<size_t>(b) * a.L;
  int yy = -1;
  if (tid < live) {
    yy = vy[tid];
    if (vk[tid] == 0) atomicMin(&sm.first_rej, tid);
  }
  __syncthreads();
  const int acc = min(sm.first_rej + 1, live);
  if (tid < acc) a.out[static_cast<size_t>(b) * a.N + p0 + tid] = a.v_lo + yy;
  if (tid < live) {
    const size_t sidx = static_cast<size_t>(b) * a.L + (p0 + tid) % a.L;
    if (tid >= acc) {
      a.X[sidx] = yy;
      a.age_w[sidx] += 1;
    } else {
      const int np = p0 + a.L + tid;
      a.X[sidx] = np < a.N ? init_token(a.seed, b, np, n) : -1;
      a.age_w[sidx] = 0;
    }
  }
  if (tid == 0) {
    a.accept_len[b] = acc;
    a.pos[b] = p0 + acc;
    a.iter[b] = it + 1;
    a.verified[b] += live;
    a.ticket[b] = 0;
  }
}

}  // namespace

size_t row_kernel_lds_bytes(int n) {
  return static_cast<size_t>((n + 7) & ~7) * 2 + NBINS * sizeof(uint32_t) + kListCap * sizeof(uint16_t);
}

hipError_t launch_row(const RowArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  const size_t lds = row_kernel_lds_bytes(a.n);
  static size_t configured = 0;          // grows monotonically; benign if raced (idempotent call)
  if (lds > configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(row_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(lds));
    if (e != hipSuccess) return e;
    configured = lds;
  }
  hipLaunchKernelGGL(row_kernel, dim3(a.rows), dim3(THREADS), lds, s, a);
  return hipGetLastError();
}

}  // namespace scd
