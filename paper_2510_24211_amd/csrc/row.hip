// Per-row part of the SCD step: top-k threshold, softmax normaliser, Modified
// Rejection Sampling (accept test + residual resample) and -- through a
// last-arriver ticket per sequence -- first rejection, emission and window
// slide.  (Alg. 1; Sec. 4.3 "Implementation Details": every window position is
// verified, none is skipped after a rejection, and only the offset of the first
// rejection is kept; appendix "Algorithms", Alg. SCD(pi_MC); top-k / temperature
// from the appendix "Experimental Details".)
//
//   thr  = K-th largest z (exact),  kept = { v : z_v >= thr }
//   lse  = m + log sum_kept exp(z_v - m),  p_v = [z_v >= thr] exp(z_v - lse)
//   accept iff fl(u * q(x)) <= p(x);  else y = argmin_{r_v > 0} -ln(U_v) / r_v
//
// gfx950 mapping.  A row of up to 65536 logits is far more than one CU should
// chew through alone (a CU retires 64 lane-operations per clock), and with few
// sequences there are few rows, so the work is cut in two:
//   slice_kernel  rows x P workgroups.  Each holds 1/P of a row in registers
//                 (8 logits per thread), finds the slice's r-th largest key
//                 exactly (r ~ 2K/P) and emits the (id, logit) pairs above it.
//                 The union of the emitted sets contains the row's top K unless
//                 one slice holds more than r of them.
//   row_kernel    one workgroup per row.  Loads the <= 6144 candidates into
//                 registers (6 per thread), selects the K-th largest key among
//                 them, and accepts the answer only if it is >= every slice's
//                 cut (then no unseen logit can be >= it): exact, verified.
//                 Sum of exponentials, accept test, residual race and the
//                 commit follow from the same registers.
// Rows of <= 16384 logits need no candidates (the whole row fits the row
// kernel's registers); on longer ones the lists come from the LM head's
// epilogue, one per 256-column tile, when that kernel emits them.  If the verification fails (massive ties, adversarial
// layouts) or top-k is off, the row kernel falls back to a complete in-place
// path: one coalesced read of the row, 16-bit key prefixes parked in LDS,
// histogram select, candidate list or in-place scans.
// The K-th largest key is always found by integer counting (LDS histograms
// whose bins adapt to the key range, so lanes rarely collide); all
// floating-point sums use a fixed assignment of ids to threads and a fixed
// reduction tree, so results are run-to-run identical.
//
// This file is compiled twice.  The second time (row_batched.hip defines
// SCD_ROW_BATCHED) with 512 threads per row and rows of at most 8192 ids: such a
// workgroup takes 122 registers per lane and 64 KB of LDS, so two of them share a
// CU, and when there are more rows than CUs the barrier-separated phases of one
// row overlap with another's instead of the rows queueing in rounds.  With few
// rows the 1024-thread form is faster (half the work per lane).
#include "scd_device.h"
#include "scd_kernels.h"

#ifdef SCD_ROW_BATCHED
#define SCD_ROW_THREADS 512
#define SCD_ROW_DIRECT_MAX 8192
#define row_kernel row_kernel_batched        // distinct names in traces
#define slice_kernel slice_kernel_batched
#define LAUNCH_ROW launch_row_batched
#else
#define LAUNCH_ROW launch_row
#endif

namespace scd {
namespace {

#ifndef SCD_ROW_THREADS
#define SCD_ROW_THREADS 1024
#endif
// Few, fat threads: the per-wavefront bookkeeping (scans, reductions, the accept draw)
// costs issue slots per wavefront, the per-logit work does not care how it is cut.
constexpr int THREADS = SCD_ROW_THREADS;
constexpr int NW = THREADS / kWave;
constexpr int NBINS = 4096;
constexpr int kListCap = kRowListCap;         // candidate ids per row (LDS list / slice or tile output)
constexpr int PER_LIST = kListCap / THREADS; // candidates per thread
#ifndef SCD_ROW_DIRECT_MAX
#define SCD_ROW_DIRECT_MAX 16384
#endif
constexpr int kDirectMaxN = SCD_ROW_DIRECT_MAX;   // whole row in registers up to this many ids
constexpr int PER_DIRECT = kDirectMaxN / THREADS;   // (rows of half that size take half of them)
constexpr int kSliceMax = 8192;              // logits per slice workgroup
constexpr int PER_SLICE = kSliceMax / THREADS;
static_assert(THREADS >= 256 && kListCap % THREADS == 0 && PER_DIRECT % 8 == 0 && PER_SLICE % 4 == 0,
              "row kernels: unsupported workgroup size");
constexpr int kKeptCap = 4096;               // kept ids compacted in LDS

struct Small {
  float fred[NW];
  uint32_t ured[NW];
  uint32_t umin[NW];
  uint32_t umax[NW];
  int ired[NW];
  uint32_t wtot[NW];
  uint32_t sel_bin, sel_above;
  uint32_t cursor;        // append cursor of select_regs
  int ired2[NW];          // second slot of block_offsets
  float s_score[NW];
  int s_id[NW];
  int last;
  int first_rej;
  unsigned long long mtot[NW];   // nucleus: per-wavefront masses
  unsigned long long sel_mass;
  float dred[3][NW];             // statistics: per-wavefront sums
  int hamm[6];                   // (differing, compared) drafts 1, 2, 3 iterations apart
  int xnew[256];                 // the sequence's new drafts by ring slot
};

// Lexicographic (score, id) minimum over the per-wavefront entries in LDS.  All entries are read
// first and folded with selects: a chain of compare-and-branch steps waits for one LDS round
// trip per entry (about a microsecond for 16 wavefronts).
__device__ __forceinline__ void block_min_score_id(const Small& sm, float& best, int& best_id) {
  float ss[NW];
  int si[NW];
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    ss[w] = sm.s_score[w];
    si[w] = sm.s_id[w];
  }
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const bool better = (ss[w] < best) | ((ss[w] == best) & (si[w] < best_id));
    best = better ? ss[w] : best;
    best_id = better ? si[w] : best_id;
  }
}

// hist[0..NBINS): find the bin holding the `need`-th largest element counting
// from the top bin; lowers `need` by the population of the bins above it.
// The trailing barrier keeps a later writer of sel_bin / sel_above / wtot away from slow
// readers; a caller whose next such write comes after another barrier anyway may drop it.
// T: threads of the workgroup (the row kernel's, or the slice kernel's smaller one).
template <int T = THREADS>
__device__ __forceinline__ uint32_t find_bin(const uint32_t* hist, uint32_t& need, Small& sm,
                                             bool trailing = true) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int PER = NBINS / T;         // consecutive bins per thread, top bins in thread 0
  uint32_t c[PER], local = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    c[j] = hist[NBINS - 1 - (tid * PER + j)];
    local += c[j];
  }
  uint32_t incl = static_cast<uint32_t>(wave_inclusive_sum_i32(static_cast<int>(local), lane));
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
  if (trailing) __syncthreads();
  return bin;
}

template <int T = THREADS>
__device__ __forceinline__ void zero_hist(uint32_t* hist) {
#pragma unroll
  for (int j = 0; j < NBINS / T; ++j) hist[threadIdx.x + j * T] = 0u;
}

__device__ __forceinline__ float prob(float z, float thr, float lse) {
  return z >= thr ? expf(z - lse) : 0.f;
}

// Exclusive offset of this thread's `cnt` in a fixed thread order, and the total.
// `slot` picks one of two exchange arrays; without the trailing barrier the caller must
// have another barrier between this call and the next one on the same slot.
template <int T = THREADS>
__device__ __forceinline__ int block_offsets(int cnt, int& total, Small& sm, int slot = 0,
                                             bool trailing = true) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int incl = wave_inclusive_sum_i32(cnt, lane);
  int* const ex = slot ? sm.ired2 : sm.ired;
  if (lane == 63) ex[wave] = incl;
  __syncthreads();
  int base = 0;
  total = 0;
#pragma unroll
  for (int w = 0; w < T / kWave; ++w) {
    base += w < wave ? ex[w] : 0;
    total += ex[w];
  }
  if (trailing) __syncthreads();
  return base + incl - cnt;
}

// max / min of keys over the workgroup
template <int T = THREADS>
__device__ __forceinline__ void block_minmax(uint32_t& kmin, uint32_t& kmax, Small& sm,
                                             bool trailing = true) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  kmax = wave_max_u32(kmax);
  kmin = ~wave_max_u32(~kmin);
  if (lane == 0) {
    sm.umax[wave] = kmax;
    sm.umin[wave] = kmin;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < T / kWave; ++w) {
    kmax = sm.umax[w] > kmax ? sm.umax[w] : kmax;
    kmin = sm.umin[w] < kmin ? sm.umin[w] : kmin;
  }
  if (trailing) __syncthreads();
}

// `need`-th largest key among the register-resident logits zv[e] (keys kv[e], valid
// where ok[e]).  kmin_in is the smallest key among the valid logits above -1e30,
// kmax the largest key (both from block_minmax).
//   Level 1 bins the logits LINEARLY in value between those two (any monotone map
//   of the value preserves the order statistic; a linear one spreads a bell-shaped
//   row over all bins, where the float bit pattern would pile it into a few
//   exponent bins and serialise the LDS atomics).
//   Level 2 ranks the handful of members of the selected bin against each other.
//   Should that bin hold more than NBINS members (massive ties), radix levels over
//   the key bits finish the job.
constexpr float kRangeFloor = -1.0e30f;
template <int PER, int T = THREADS>
__device__ __forceinline__ uint32_t select_regs(const float (&zv)[PER], const uint32_t (&kv)[PER],
                                                const bool (&ok)[PER], uint32_t kmin_in,
                                                uint32_t kmax, uint32_t need, uint32_t* hist,
                                                uint32_t* arr, Small& sm) {
  // hist was zeroed by the caller before the barrier of block_minmax; arr (NBINS entries,
  // disjoint from hist) takes the members of the selected bin.
  const float zlo = key_to_float(kmin_in), zhi = key_to_float(kmax);
  const float scale = (zhi > zlo) ? __fdiv_rn(static_cast<float>(NBINS - 1), zhi - zlo) : 0.f;
  int bin[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    int bb = 0;
    if (ok[e] && zv[e] > kRangeFloor) {
      const float t = (zv[e] - zlo) * scale;
      bb = t >= 0.f ? (t >= static_cast<float>(NBINS - 1) ? NBINS - 1 : static_cast<int>(t)) : 0;
    }
    bin[e] = bb;
  }
  if (threadIdx.x == 0) sm.cursor = 0u;          // append cursor, published by the next barrier
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (ok[e]) atomicAdd(&hist[bin[e]], 1u);
  __syncthreads();
  // no trailing barrier: sel_bin is next written after the barrier that follows the append
  const int b1 = static_cast<int>(find_bin<T>(hist, need, sm, false));
  const uint32_t members = hist[b1];
  if (members <= static_cast<uint32_t>(NBINS)) {
#pragma unroll
    for (int e = 0; e < PER; ++e)
      if (ok[e] && bin[e] == b1) arr[atomicAdd(&sm.cursor, 1u)] = kv[e];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (ok[e] && bin[e] == b1) {
        uint32_t gt = 0, ge = 0;
        for (uint32_t i = 0; i < members; ++i) {
          const uint32_t k = arr[i];
          gt += k > kv[e] ? 1u : 0u;
          ge += k >= kv[e] ? 1u : 0u;
        }
        if (gt < need && need <= ge) sm.sel_bin = kv[e];   // equal keys write the same value
      }
    }
    __syncthreads();
    return sm.sel_bin;      // its next writer sits behind the barriers of the caller's next step
  }
  __syncthreads();          // every thread has read hist[b1] before the histogram is reused
  // radix levels over the key bits of the members, range [lo, lo + width)
  uint32_t lo = 0;
  uint64_t width = 1ull << 32;
  for (;;) {
    int s2 = 0;
    while (((width - 1) >> s2) >= static_cast<uint64_t>(NBINS)) ++s2;
    zero_hist<T>(hist);
    __syncthreads();
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (ok[e] && bin[e] == b1 && kv[e] >= lo && static_cast<uint64_t>(kv[e] - lo) < width)
        atomicAdd(&hist[(kv[e] - lo) >> s2], 1u);
    }
    __syncthreads();
    const uint32_t dgt = find_bin<T>(hist, need, sm);
    lo += dgt << s2;
    width = 1ull << s2;
    if (s2 == 0) return lo;
  }
}

// ---------------------------------------------------------------------------------
// Nucleus (top-p) filter (appendix "Experimental Details", video setting p = 0.8), applied
// to the set K1 that top-k left:  keep v  iff  the mass of the ids with a LARGER logit is
// below top_p times the mass of K1 -- the shortest most-probable prefix reaching top_p, ids
// tied with its last member included.  Like top-k the result is a threshold on the logit.
//   Masses are 64-bit fixed point, w_v = trunc(expf(z_v - m) * 2^40): integer sums do not
//   depend on the order of the LDS atomics, so the decision is run-to-run identical, and it
//   is taken exactly:  above(v) * 2^24 < P24 * S  with P24 = round(top_p * 2^24).
//   Search: one histogram of masses over bins LINEAR in the logit (spreads a bell-shaped row
//   over the bins), then radix levels over the key bits of the selected bin's members.
// `each(f)` must call f(key, z) for every element of K1.  After the first level
// `prepare(klo, khi)` is called once and then `near(f)` must call f for at least the elements of
// K1 whose key lies in [klo, khi] (a path that can find them without reading the whole row again
// does so; extra elements are filtered here).
// mh: NBINS_P 64-bit bins (the space of the count histogram).  Uniform over the workgroup.
constexpr int NBINS_P = NBINS / 2;
static_assert(NBINS_P % THREADS == 0 || THREADS % NBINS_P == 0, "nucleus: bins per thread");

__device__ __forceinline__ unsigned long long mass_of(float z, float m) {
  return static_cast<unsigned long long>(expf(z - m) * 1099511627776.0f);   // <= 2^40
}

__device__ __forceinline__ unsigned long long wave_inclusive_sum_u64(unsigned long long v, int lane) {
  // three 24-bit limbs: 64 lanes x 2^24 stays inside an int
  const int l0 = wave_inclusive_sum_i32(static_cast<int>(v & 0xFFFFFFull), lane);
  const int l1 = wave_inclusive_sum_i32(static_cast<int>((v >> 24) & 0xFFFFFFull), lane);
  const int l2 = wave_inclusive_sum_i32(static_cast<int>(v >> 48), lane);
  return static_cast<unsigned long long>(static_cast<uint32_t>(l0)) +
         (static_cast<unsigned long long>(static_cast<uint32_t>(l1)) << 24) +
         (static_cast<unsigned long long>(static_cast<uint32_t>(l2)) << 48);
}

// ceil(P24 * S / 2^24) for S < 2^58
__device__ __forceinline__ unsigned long long nucleus_target(unsigned long long S, uint32_t p24) {
  const unsigned long long hi = (S >> 32) * p24, lo = (S & 0xFFFFFFFFull) * p24;
  return (hi << 8) + ((lo + 0xFFFFFFull) >> 24);
}

// The bin b with  above + mass(bins > b) < target <= above + mass(bins >= b);  `above` grows
// by mass(bins > b).  FIRST: target is derived here from the total mass of the histogram.
template <bool FIRST>
__device__ __forceinline__ uint32_t find_bin_mass(const unsigned long long* mh, unsigned long long& target,
                                                  unsigned long long& above, uint32_t p24, Small& sm) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int PER = NBINS_P >= THREADS ? NBINS_P / THREADS : 1;
  unsigned long long c[PER], local = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int idx = tid * PER + j;                 // top bins first
    c[j] = idx < NBINS_P ? mh[NBINS_P - 1 - idx] : 0ull;
    local += c[j];
  }
  unsigned long long incl = wave_inclusive_sum_u64(local, lane);
  if (lane == 63) sm.mtot[wave] = incl;
  __syncthreads();
  unsigned long long base = above, total = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    base += w < wave ? sm.mtot[w] : 0ull;
    total += sm.mtot[w];
  }
  if (FIRST) target = nucleus_target(total, p24);
  incl += base;
  const unsigned long long excl = incl - local;
  if (excl < target && target <= incl) {           // exactly one thread
    unsigned long long ab = excl;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (ab + c[j] >= target) {
        sm.sel_bin = static_cast<uint32_t>(NBINS_P - 1 - (tid * PER + j));
        sm.sel_mass = ab;
        break;
      }
      ab += c[j];
    }
  }
  __syncthreads();
  const uint32_t bin = sm.sel_bin;
  above = sm.sel_mass;
  __syncthreads();
  return bin;
}

template <class Each, class Prepare, class Near>
__device__ __forceinline__ uint32_t nucleus_key(Each&& each, Prepare&& prepare, Near&& near, float m, float zmin, uint32_t p24,
                                                unsigned long long* mh, Small& sm) {
  const int tid = threadIdx.x;
  // logits more than 110 below the maximum weigh nothing: they all go to bin 0
  const float zlo = fmaxf(zmin, m - 110.f);
  const float scale = (m > zlo) ? __fdiv_rn(static_cast<float>(NBINS_P - 1), m - zlo) : 0.f;
  auto lin_bin = [&](float z) {
    const float t = (z - zlo) * scale;
    return t >= 0.f ? (t >= static_cast<float>(NBINS_P - 1) ? NBINS_P - 1 : static_cast<int>(t)) : 0;
  };
  auto zero = [&]() {
    for (int i = tid; i < NBINS_P; i += THREADS) mh[i] = 0ull;
  };
  __syncthreads();                                  // earlier users of the histogram space are done
  zero();
  __syncthreads();
  each([&](uint32_t key, float z) { atomicAdd(&mh[lin_bin(z)], mass_of(z, m)); });
  __syncthreads();
  unsigned long long target = 0, above = 0;
  const int b1 = static_cast<int>(find_bin_mass<true>(mh, target, above, p24, sm));
  // keys that can fall into bin b1: its interval of logits widened by a bin on either side
  // (the rounding of lin_bin's arithmetic moves a logit by far less than a bin)
  uint32_t near_lo = 0u, near_hi = 0xFFFFFFFFu;
  if (scale > 0.f) {
    const float inv = __fdiv_rn(m - zlo, static_cast<float>(NBINS_P - 1));
    if (b1 > 1) near_lo = zkey(zlo + static_cast<float>(b1 - 1) * inv);
    if (b1 < NBINS_P - 2) near_hi = zkey(zlo + static_cast<float>(b1 + 2) * inv);
  }
  prepare(near_lo, near_hi);
  // radix levels over the key bits of the members of bin b1
  uint32_t lo = 0;
  int s2 = 32;
  while (s2 > 0) {
    const int width_bits = s2;                      // candidates: keys in [lo, lo + 2^width_bits)
    s2 = width_bits > 11 ? width_bits - 11 : 0;
    zero();
    __syncthreads();
    near([&](uint32_t key, float z) {
      if (lin_bin(z) == b1 && key >= lo &&
          (width_bits == 32 || (key - lo) >> width_bits == 0u))
        atomicAdd(&mh[(key - lo) >> s2], mass_of(z, m));
    });
    __syncthreads();
    lo += find_bin_mass<false>(mh, target, above, p24, sm) << s2;
  }
  return lo;
}

// Where a kernel instance finds its row.
struct RowRef {
  const float* zc;
  const float* zp;
  float thr_p, lse_p;
  bool fresh, active;
  int x, b, s, p0, live, it;
  size_t widx, oidx;
  size_t pidx;    // where the previous evaluation of the slot left its per-slot results (ring mode)
};

// pos, iter, mode, L, N repeat a.pos, a.iter, mode, L, N: the kernels receive them as plain
// leading arguments, which the hardware preloads into SGPRs at wavefront launch, so that the first
// dependent load (pos[b]) does not wait for a fetch of the kernel-argument segment.
__device__ __forceinline__ RowRef locate_row(const RowArgs& a, int r, const int32_t* pos,
                                             const int32_t* iter, int mode, int L, int N) {
  RowRef R{};
  R.widx = r;
  R.oidx = r;
  R.it = a.iter_scalar;
  R.x = -1;
  R.active = true;
  const int n = a.n;
  if (mode == kRowSelectOnly) {
    R.zc = a.z_cur + static_cast<size_t>(r) * n;
    return R;
  }
  R.b = r / L;
  R.s = r % L;
  R.p0 = pos[R.b];
  R.live = max(0, min(L, N - R.p0));
  R.widx = static_cast<size_t>(R.b) * L + R.s;
  if (R.s >= R.live) {
    R.active = false;
    return R;
  }
  if (mode == kRowRing) {
    R.it = iter[R.b];
    const int par = R.it & 1;
    const size_t sidx = static_cast<size_t>(R.b) * L + (R.p0 + R.s) % L;
    const size_t half = static_cast<size_t>(a.B) * L;
    R.oidx = par * half + sidx;
    R.pidx = (par ^ 1) * half + sidx;
    R.x = a.x[sidx];
    R.fresh = a.age[sidx] == 0;
    R.zc = a.z_cur + static_cast<size_t>(par) * a.parity_stride + sidx * n;
    R.zp = a.z_cur + static_cast<size_t>(par ^ 1) * a.parity_stride + sidx * n;
    if (!R.fresh) {
      R.thr_p = a.thr[(par ^ 1) * half + sidx];
      R.lse_p = a.lse[(par ^ 1) * half + sidx];
    }
  } else {
    R.oidx = R.widx;
    R.x = a.x[R.widx];
    R.fresh = a.fresh ? a.fresh[R.widx] != 0 : false;
    R.zc = a.z_cur + R.widx * n;
    R.zp = a.z_prev + R.widx * n;
    if (!R.fresh) {
      R.thr_p = a.thr_prev[R.widx];
      R.lse_p = a.lse_prev[R.widx];
    }
  }
  return R;
}

// ---------------------------------------------------------------------------------
// slice kernel
// ---------------------------------------------------------------------------------
// ST threads: 1024, or 512 when there are more slices than two per CU (four such workgroups
// fit a CU by LDS and wavefronts, so that all of them run at once: C4 192 -> 186 us per step)
template <int ST>
__global__ __launch_bounds__(ST) void slice_kernel(const int32_t* const pos_, const int32_t* const iter_,
                                                        const int mode_, const int L_, const int N_,
                                                        const int P, const int capE, const int rank,
                                                        const RowArgs a) {
  __shared__ uint32_t hist[NBINS];
  __shared__ uint32_t arr[NBINS];
  __shared__ Small sm;
  constexpr int PS = kSliceMax / ST;   // logits per thread
  const int tid = threadIdx.x;
  const int r = blockIdx.x / P, p = blockIdx.x % P;
  const RowRef R = locate_row(a, r, pos_, iter_, mode_, L_, N_);
  if (!R.active) return;
  const int n = a.n;
  const int slice_len = (((n + P - 1) / P) + 3) & ~3;
  const int lo_id = p * slice_len;
  const int hi_id = min(n, lo_id + slice_len);
  uint32_t* const cnt_out = a.cand_cnt + static_cast<size_t>(r) * P;
  uint32_t* const cut_out = a.cand_cut + static_cast<size_t>(r) * P;
  if (lo_id >= hi_id) {
    if (tid == 0) {
      cnt_out[p] = 0;
      cut_out[p] = 0;
    }
    return;
  }
  const bool vec_ok = (n & 3) == 0;
  float zv[PS];
  int vid[PS];
  bool ok[PS];
#pragma unroll
  for (int u = 0; u < PS / 4; ++u) {
    const int v0 = lo_id + ((tid + u * ST) << 2);
    if (vec_ok && v0 + 3 < hi_id) {
      const float4 t = *reinterpret_cast<const float4*>(R.zc + v0);
      zv[u * 4 + 0] = t.x; zv[u * 4 + 1] = t.y; zv[u * 4 + 2] = t.z; zv[u * 4 + 3] = t.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) zv[u * 4 + e] = (v0 + e < hi_id) ? R.zc[v0 + e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vid[u * 4 + e] = v0 + e;
      ok[u * 4 + e] = v0 + e < hi_id;
    }
  }
  uint32_t kv[PS], kmax = 0, kmin = 0xFFFFFFFFu;
#pragma unroll
  for (int e = 0; e < PS; ++e) {
    kv[e] = zkey(zv[e]);
    if (ok[e]) {
      kmax = kv[e] > kmax ? kv[e] : kmax;
      if (zv[e] > kRangeFloor) kmin = kv[e] < kmin ? kv[e] : kmin;
      if (zv[e] != zv[e] && a.flags) atomicOr(a.flags, 1);     // NaN of either sign
    }
  }
  zero_hist<ST>(hist);                        // published by the barrier inside block_minmax
  block_minmax<ST>(kmin, kmax, sm, false);
  const int nvalid = hi_id - lo_id;
  uint32_t cut = 0;                       // 0: the whole slice is emitted
  if (nvalid > rank)
    cut = select_regs<PS, ST>(zv, kv, ok, kmin, kmax, static_cast<uint32_t>(rank), hist, arr, sm);
  int mine = 0;
#pragma unroll
  for (int e = 0; e < PS; ++e) mine += (ok[e] && kv[e] >= cut) ? 1 : 0;
  int total;
  int off = block_offsets<ST>(mine, total, sm, 0, false);
  uint2* const dst = a.cand + (static_cast<size_t>(r) * kListCap + static_cast<size_t>(p) * capE);
#pragma unroll
  for (int e = 0; e < PS; ++e) {
    if (ok[e] && kv[e] >= cut) {
      if (off < capE) dst[off] = make_uint2(static_cast<uint32_t>(vid[e]), __float_as_uint(zv[e]));
      ++off;
    }
  }
  if (tid == 0) {
    cnt_out[p] = static_cast<uint32_t>(total);   // > capE signals overflow
    cut_out[p] = cut;
  }
}

// Per-position statistics of the iteration (Sec. 3: acceptance rate beta = 1 - D_TV(p, q) =
// sum_v min(p_v, q_v); Prop. "SJD Collision Probability": C = sum_v p_v q_v and its bound
// sqrt(sum p^2 * sum q^2) = exp(-(H_2(p) + H_2(q)) / 2)).  d0..d2: this thread's share of
// sum min(p, q), sum p q, sum p^2 over the kept ids.  sum q^2 is what the slot's previous
// evaluation stored (1/n for a never-evaluated position).  Uniform over the workgroup.
__device__ __forceinline__ void row_statistics_out(const RowArgs& a, const RowRef& R, float d0, float d1,
                                                   float d2, float q_uniform, Small& sm) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  d0 = wave_sum(d0);
  d1 = wave_sum(d1);
  d2 = wave_sum(d2);
  if (lane == 0) {
    sm.dred[0][wave] = d0;
    sm.dred[1][wave] = d1;
    sm.dred[2][wave] = d2;
  }
  __syncthreads();
  if (tid == 0) {
    float s0 = 0.f, s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      s0 += sm.dred[0][w];
      s1 += sm.dred[1][w];
      s2 += sm.dred[2][w];
    }
    const float s2q = R.fresh ? q_uniform : a.s2[R.pidx];
    *reinterpret_cast<float4*>(a.diag + R.widx * 4) = make_float4(s0, s1, s2, s2q);
    a.s2[R.oidx] = s2;
  }
}

// ---------------------------------------------------------------------------------
// row kernel
// ---------------------------------------------------------------------------------
struct RowOut {      // what a path hands to the common tail
  bool accept;
  bool prace;         // the row makes a Gumbel-max draw from p (GS kernels only)
  float px, qx;
  float best;         // residual race (on rejection)
  int best_id;
  float gbest;        // Gumbel-sharing draft (GS kernels only)
  int gbest_id;
};

// Entry of id v, probability pv > 0, in the shared-noise Gumbel-max draw of position j
// (Alg. GS / Alg. SCD(pi_GS)): argmax_v(log p_v + G_v) with G_v = -ln(-ln U_v) is the
// argmin of -ln(U_v) / p_v (appendix proof of the Gumbel-coupling theorem).  U_v is keyed by
// (seed, sequence, position, id) only -- not by the iteration -- so that every iteration
// redraws the position with the same noise (w3s = stream 3, it = 0).  The independent redraft
// of the alpha-coupling is the same draw with fresh noise (stream 5, it = the iteration).
// Ties go to the lowest id.
__device__ __forceinline__ void gumbel_entry(RowOut& out, uint2 key, uint32_t w3s, int j, int it,
                                             int v, float pv) {
  const uint4 rr = philox4x32_10(make_uint4(static_cast<uint32_t>(v >> 2), static_cast<uint32_t>(j),
                                            static_cast<uint32_t>(it), w3s), key);
  const uint32_t lanes[4] = {rr.x, rr.y, rr.z, rr.w};
  const float sc = __fdiv_rn(-logf(u01(lanes[v & 3])), pv);
  if (sc < out.gbest || (sc == out.gbest && v < out.gbest_id)) {
    out.gbest = sc;
    out.gbest_id = v;
  }
}

// Which Gumbel-max draw from p the row makes for its next draft, if any (uniform over the
// workgroup).  alpha-coupling (Sec. 5.3): with probability 1 - alpha the redraft is independent:
// fresh noise.  Otherwise the shared-noise draw under pi_GS, and none under pi_MC (the MRS output
// is the redraft).
struct PRace {
  bool on;
  uint32_t w3s;
  int it;
};
__device__ __forceinline__ PRace p_race_of_row(const RowArgs& a, uint2 key, uint32_t w3, int j, int it) {
  if (a.alpha < 1.0f) {
    const uint4 rs = philox4x32_10(make_uint4(0u, static_cast<uint32_t>(j), static_cast<uint32_t>(it),
                                              w3 | kStreamAlpha), key);
    if (!(u01(rs.x) <= a.alpha)) return {true, w3 | kStreamIndep, it};
  }
  return {a.gumbel != 0, w3 | kStreamGumbel, 0};
}

// Everything after the candidates sit in registers: threshold (if top-k filters),
// normaliser, accept test, residual race.  Returns false if the threshold could not
// be certified against `cut_max` (the caller then takes the complete path).
// PREQ: zq[e] is the previous iteration's logit of id vid[e], read by the caller together
// with zv (coalesced, long before a rejection may need it; unused for a fresh position).
// Otherwise (ids scattered over the row) the previous logits of the KEPT ids are gathered
// here, right after the compaction, so that the round trip hides behind the normaliser and
// the accept draw.  The LDS arrays cid / cz / cq hold ccap entries each.
template <int PER, bool PREQ, bool GS, bool EXTRA>
__device__ __forceinline__ bool finish_regs(const RowArgs& a, const RowRef& R, const int (&vid)[PER],
                                            const float (&zv)[PER], const float (&zq)[PER],
                                            const bool (&ok)[PER], bool filter, uint32_t cut_max,
                                            float zcx, float zpx, uint32_t* hist, uint32_t* cid,
                                            float* cz, float* cq, int ccap, Small& sm, RowOut& out,
                                            bool have_thr = false, float thr_given = 0.f) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = a.n;
  uint32_t kv[PER], kmax = 0, kmin = 0xFFFFFFFFu;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    kv[e] = zkey(zv[e]);
    if (ok[e]) {
      kmax = kv[e] > kmax ? kv[e] : kmax;
      if (zv[e] > kRangeFloor) kmin = kv[e] < kmin ? kv[e] : kmin;
      if (zv[e] != zv[e] && a.flags) atomicOr(a.flags, 1);     // NaN of either sign
    }
  }
  if (filter) zero_hist(hist);            // published by the barrier inside block_minmax
  block_minmax(kmin, kmax, sm, false);
  const float m = key_to_float(kmax);
  float thr = have_thr ? thr_given : -INFINITY;   // given: the caller has applied the filters
  if (filter) {
    // cid (ccap entries, all of them free until the compaction) takes the selected bin's members
    const uint32_t tkey = select_regs<PER>(zv, kv, ok, kmin, kmax, static_cast<uint32_t>(a.top_k), hist,
                                           cid, sm);
    if (tkey < cut_max) return false;     // an unseen logit could be >= the K-th candidate
    thr = key_to_float(tkey);
  }
  if (EXTRA && a.top_p24 != 0u && !have_thr) {   // nucleus filter on what top-k left
    const float thr_k = thr;
    const float zmin = filter ? thr_k : (kmin <= kmax ? key_to_float(kmin) : m);
    auto each = [&](auto&& f) {
#pragma unroll
      for (int e = 0; e < PER; ++e)
        if (ok[e] && zv[e] >= thr_k) f(kv[e], zv[e]);
    };
    const uint32_t pkey = nucleus_key(each, [](uint32_t, uint32_t) {}, each, m, zmin, a.top_p24,
                                      reinterpret_cast<unsigned long long*>(hist), sm);
    thr = key_to_float(pkey);
  }
  // Kept ids are a random ~K/n of each thread's logits; compacting them into LDS (count /
  // scan / write: a fixed order) lets the expensive per-id work that follows be dealt out
  // evenly, kKeptPer per thread, instead of at the pace of the unluckiest lane.
  bool kept[PER];
  int mine = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    kept[e] = ok[e] && zv[e] >= thr;
    mine += kept[e] ? 1 : 0;
  }
  int Cn;
  int off = block_offsets(mine, Cn, sm, 0, false);   // next barrier: after the compaction / in the sum
  const bool compact = Cn <= ccap;
  const bool want_q = a.mode != kRowSelectOnly && !R.fresh;
  constexpr int KPT = kKeptCap / THREADS;   // ccap <= KPT * THREADS
  int rid[KPT];
  float rz[KPT], rq[KPT];
  if (compact) {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (kept[e]) {
        cid[off] = static_cast<uint32_t>(vid[e]);
        cz[off] = zv[e];
        if (PREQ) cq[off] = zq[e];
        ++off;
      }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      const int i = tid + q * THREADS;
      rid[q] = i < Cn ? static_cast<int>(cid[i]) : -1;
      rz[q] = i < Cn ? cz[i] : 0.f;
      rq[q] = (PREQ && i < Cn) ? cq[i] : 0.f;
    }
    if (!PREQ && want_q) {                    // unpredicated gathers (id 0 where there is none)
#pragma unroll
      for (int q = 0; q < KPT; ++q) rq[q] = R.zp[rid[q] >= 0 ? rid[q] : 0];
    }
  }
  float sum = 0.f;
  if (compact) {
#pragma unroll
    for (int q = 0; q < KPT; ++q)
      if (rid[q] >= 0) sum += expf(rz[q] - m);
  } else {
#pragma unroll
    for (int e = 0; e < PER; ++e)
      if (kept[e]) sum += expf(zv[e] - m);
  }
  sum = wave_sum(sum);
  if (lane == 0) sm.fred[wave] = sum;
  __syncthreads();
  float S = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) S += sm.fred[w];
  const float lse_c = m + logf(S);
  if (tid == 0) {
    a.thr[R.oidx] = thr;
    a.lse[R.oidx] = lse_c;
    a.nkept[R.oidx] = Cn;
    if (a.flags && !(lse_c == lse_c && fabsf(lse_c) < INFINITY)) atomicOr(a.flags, 1);
  }
  if (a.mode == kRowSelectOnly) return true;

  // Modified Rejection Sampling
  const int j = R.p0 + R.s;
  const float q_uniform = __fdiv_rn(1.0f, static_cast<float>(n));
  const uint2 key = seed_key(a.seed);
  const uint32_t w3 = static_cast<uint32_t>(R.b) << 8;
  const bool x_ok = R.x >= 0 && R.x < n;
  out.px = x_ok ? prob(zcx, thr, lse_c) : 0.f;
  out.qx = R.fresh ? q_uniform : (x_ok ? prob(zpx, R.thr_p, R.lse_p) : 0.f);
  const uint4 ra = philox4x32_10(make_uint4(0u, static_cast<uint32_t>(j), static_cast<uint32_t>(R.it),
                                            w3 | kStreamAccept), key);
  out.accept = __fmul_rn(u01(ra.x), out.qx) <= out.px;
  out.best = INFINITY;
  out.best_id = 0x7FFFFFFF;
  out.gbest = INFINITY;
  out.gbest_id = 0x7FFFFFFF;
  if (EXTRA && a.diag != nullptr && a.mode == kRowRing) {
    float d0 = 0.f, d1 = 0.f, d2 = 0.f;
    auto add = [&](float zc_v, float zq_v) {
      const float pv = expf(zc_v - lse_c);
      const float qv = R.fresh ? q_uniform : prob(zq_v, R.thr_p, R.lse_p);
      d0 += fminf(pv, qv);
      d1 += pv * qv;
      d2 += pv * pv;
    };
    if (compact) {
#pragma unroll
      for (int q = 0; q < KPT; ++q)
        if (rid[q] >= 0) add(rz[q], rq[q]);
    } else {
#pragma unroll
      for (int e = 0; e < PER; ++e)
        if (kept[e]) add(zv[e], PREQ ? zq[e] : (want_q ? R.zp[vid[e]] : 0.f));
    }
    row_statistics_out(a, R, d0, d1, d2, q_uniform, sm);
  }
  if (GS) {                        // next draft should the row survive
    const PRace pr = p_race_of_row(a, key, w3, j, R.it);
    out.prace = pr.on;
    if (pr.on) {
      if (compact) {
#pragma unroll
        for (int q = 0; q < KPT; ++q)
          if (rid[q] >= 0) {
            const float pv = expf(rz[q] - lse_c);
            if (pv > 0.f) gumbel_entry(out, key, pr.w3s, j, pr.it, rid[q], pv);
          }
      } else {
#pragma unroll
        for (int e = 0; e < PER; ++e)
          if (kept[e]) {
            const float pv = expf(zv[e] - lse_c);
            if (pv > 0.f) gumbel_entry(out, key, pr.w3s, j, pr.it, vid[e], pv);
          }
      }
    }
  }
  if (out.accept) return true;     // uniform over the workgroup

  auto race_one = [&](int v, float rv) {   // exponential-race entry of id v, residual rv > 0
    const uint4 rr = philox4x32_10(make_uint4(static_cast<uint32_t>(v >> 2), static_cast<uint32_t>(j),
                                              static_cast<uint32_t>(R.it), w3 | kStreamResid), key);
    const uint32_t lanes[4] = {rr.x, rr.y, rr.z, rr.w};
    const float sc = __fdiv_rn(-logf(u01(lanes[v & 3])), rv);
    if (sc < out.best || (sc == out.best && v < out.best_id)) {
      out.best = sc;
      out.best_id = v;
    }
  };
  if (compact) {
    // residuals r = p - q of the kept ids, then a second compaction of the positive ones
    int npos = 0;
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      float rv = 0.f;
      if (rid[q] >= 0) {
        const float pv = expf(rz[q] - lse_c);
        const float qv = R.fresh ? q_uniform : prob(rq[q], R.thr_p, R.lse_p);
        rv = __fsub_rn(pv, qv);
      }
      rz[q] = rv;
      npos += rv > 0.f ? 1 : 0;
    }
    int ntot;
    int o2 = block_offsets(npos, ntot, sm, 1, false);   // cid / cz were read before the sum's barrier
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      if (rz[q] > 0.f) {
        cid[o2] = static_cast<uint32_t>(rid[q]);
        cz[o2] = rz[q];
        ++o2;
      }
    }
    __syncthreads();
    for (int i = tid; i < ntot; i += THREADS) race_one(static_cast<int>(cid[i]), cz[i]);
  } else {
    float zq2[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) zq2[e] = PREQ ? zq[e] : ((want_q && kept[e]) ? R.zp[vid[e]] : 0.f);
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (kept[e]) {
        const float pv = expf(zv[e] - lse_c);
        const float qv = R.fresh ? q_uniform : prob(zq2[e], R.thr_p, R.lse_p);
        const float rv = __fsub_rn(pv, qv);
        if (rv > 0.f) race_one(vid[e], rv);
      }
    }
  }
  return true;
}

// The complete in-place path: one coalesced read of the row, 16-bit key prefixes in
// LDS, histogram select; then a candidate list in registers, or in-place scans when
// top-k is off or the candidates do not fit.
template <bool GS, bool EXTRA>
__device__ __forceinline__ void full_path(const RowArgs& a, const RowRef& R, unsigned char* smem,
                                          float zcx, float zpx, Small& sm, RowOut& out) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = a.n;
  const int n8 = (n + 7) & ~7;
  uint16_t* k16 = reinterpret_cast<uint16_t*>(smem);
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + static_cast<size_t>(n8) * 2);
  uint16_t* list = reinterpret_cast<uint16_t*>(smem + static_cast<size_t>(n8) * 2 + NBINS * 4);
  const float* zc = R.zc;
  const float* zp = R.zp;

  // pass 1: batches of 8 independent 16-byte loads per thread
  const bool vec_ok = (n & 3) == 0;
  const int ngroups = (n + 3) >> 2;
  const int ngroups8 = n8 >> 2;
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
            if (f[u][e] != f[u][e] && a.flags) atomicOr(a.flags, 1);   // NaN of either sign
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
  if (lane == 0) sm.ured[wave] = kmax;
  block_minmax(p16min, p16max, sm);      // its barriers also publish ured and the LDS prefixes
#pragma unroll
  for (int w = 0; w < NW; ++w) kmax = sm.ured[w] > kmax ? sm.ured[w] : kmax;
  const float m = key_to_float(kmax);

  const int nchunks = n8 >> 3;           // thread owns the 8-id chunks tid, tid + THREADS, ...
  const bool filter = a.top_k > 0 && a.top_k < n;
  const uint32_t K = static_cast<uint32_t>(a.top_k);
  const uint32_t range = p16max - p16min;
  int sh = 0;
  while ((range >> sh) >= static_cast<uint32_t>(NBINS)) ++sh;
  auto prefix_hist = [&](bool low_bits, uint32_t only) {
    zero_hist(hist);
    __syncthreads();
    const uint32_t mask = (1u << sh) - 1u;
    for (int c = tid; c < nchunks; c += THREADS) {
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
  uint32_t t16 = 0, need_ab = K;
  int ncand = 0, my_off = 0;
  // ids whose 16-bit key prefix is >= t16: this thread's offset in a fixed order, and the total
  auto count_candidates = [&]() {
    int my_cnt = 0;
    for (int c = tid; c < nchunks; c += THREADS) {
      const uint4 raw = *reinterpret_cast<const uint4*>(&k16[c << 3]);
      const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t p = (w4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
        my_cnt += ((c << 3) + e < n && p >= t16) ? 1 : 0;
      }
    }
    my_off = block_offsets(my_cnt, ncand, sm);
  };
  // those ids (at most kListCap) as a list, their logits in registers, and the common tail;
  // have_thr: the filters have been applied already and thr_given is their threshold
  auto run_list = [&](bool have_thr, float thr_given) {
    int o = my_off;
    for (int c = tid; c < nchunks; c += THREADS) {
      const uint4 raw = *reinterpret_cast<const uint4*>(&k16[c << 3]);
      const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t p = (w4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
        if ((c << 3) + e < n && p >= t16) list[o++] = static_cast<uint16_t>((c << 3) + e);
      }
    }
    __syncthreads();
    int vid[PER_LIST];
    float zv[PER_LIST];
    bool ok[PER_LIST];
#pragma unroll
    for (int e = 0; e < PER_LIST; ++e) {
      const int i = tid + e * THREADS;
      ok[e] = i < ncand;
      vid[e] = ok[e] ? static_cast<int>(list[i]) : 0;
    }
#pragma unroll
    for (int e = 0; e < PER_LIST; ++e) zv[e] = ok[e] ? zc[vid[e]] : 0.f;
    float zq[PER_LIST];                        // unused: finish_regs gathers what it needs
#pragma unroll
    for (int e = 0; e < PER_LIST; ++e) zq[e] = 0.f;
    // the prefixes in LDS are spent: their space takes the compaction arrays
    const int ccap = min(kKeptCap, static_cast<int>(static_cast<size_t>(n8) * 2 / 12));
    finish_regs<PER_LIST, false, GS, EXTRA>(a, R, vid, zv, zq, ok, !have_thr, 0u, zcx, zpx, hist,
                          reinterpret_cast<uint32_t*>(smem), reinterpret_cast<float*>(smem) + ccap,
                          reinterpret_cast<float*>(smem) + 2 * ccap, ccap, sm, out, have_thr, thr_given);
  };
  if (filter) {
    prefix_hist(false, 0u);
    const uint32_t binA = find_bin(hist, need_ab, sm);
    uint32_t low = 0;
    if (sh > 0) {
      prefix_hist(true, binA);
      low = find_bin(hist, need_ab, sm);
    }
    t16 = p16min + (binA << sh) + low;
    count_candidates();
    if (ncand <= kListCap) {
      run_list(false, 0.f);
      return;
    }
  }

  // in place: no filter, or the candidates do not fit (massive ties)
  bool pfilter = filter;                 // candidates = ids whose 16-bit key prefix is >= t16
  auto for_each_candidate = [&](auto&& f) {
    for (int c = tid; c < nchunks; c += THREADS) {
      const uint4 raw = *reinterpret_cast<const uint4*>(&k16[c << 3]);
      const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int v = (c << 3) + e;
        const uint32_t p = (w4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
        if (v < n && (!pfilter || p >= t16)) f(v, p);
      }
    }
  };
  // The same candidates with their logits: f(v, z).  Without a filter every id is a candidate
  // and the row is read in coalesced 32-byte pieces, two chunks per thread in flight; with one
  // the few ids that pass the prefix test are gathered.
  auto for_each_logit = [&](auto&& f) {
    if (!pfilter && vec_ok) {
      for (int c0 = tid; c0 < nchunks; c0 += 2 * THREADS) {
        float zz[2][8];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int c = c0 + u * THREADS;
          if (c < nchunks && (c << 3) + 7 < n) {
            const float4 lo4 = *reinterpret_cast<const float4*>(zc + (c << 3));
            const float4 hi4 = *reinterpret_cast<const float4*>(zc + (c << 3) + 4);
            zz[u][0] = lo4.x; zz[u][1] = lo4.y; zz[u][2] = lo4.z; zz[u][3] = lo4.w;
            zz[u][4] = hi4.x; zz[u][5] = hi4.y; zz[u][6] = hi4.z; zz[u][7] = hi4.w;
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) zz[u][e] = (c < nchunks && (c << 3) + e < n) ? zc[(c << 3) + e] : 0.f;
          }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int c = c0 + u * THREADS;
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (c < nchunks && (c << 3) + e < n) f((c << 3) + e, zz[u][e]);
        }
      }
    } else {
      for_each_candidate([&](int v, uint32_t) { f(v, zc[v]); });
    }
  };
  float thr = -INFINITY;
  if (filter) {
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
  if (EXTRA && a.top_p24 != 0u) {          // nucleus filter on what top-k left
    const float thr_k = thr;
    const float zmin = filter ? thr_k : key_to_float(p16min << 16);
    // members of the selected bin: ids found by the prefixes in LDS (appended in any order:
    // the masses are integers), their logits gathered once and kept for the three radix levels
    int near_cnt = 0;
    bool near_dense = false;
    float nz[PER_LIST];
    const uint32_t pkey = nucleus_key(
        [&](auto&& f) {
          for_each_logit([&](int, float z) {
            if (z >= thr_k) f(zkey(z), z);
          });
        },
        [&](uint32_t klo, uint32_t khi) {
          const uint32_t pa = klo >> 16, pb = khi >> 16;
          if (tid == 0) sm.cursor = 0u;
          __syncthreads();
          for_each_candidate([&](int v, uint32_t p) {
            if (p >= pa && p <= pb) {
              const uint32_t slot = atomicAdd(&sm.cursor, 1u);
              if (slot < static_cast<uint32_t>(kListCap)) list[slot] = static_cast<uint16_t>(v);
            }
          });
          __syncthreads();
          const uint32_t found = sm.cursor;
          near_dense = found > static_cast<uint32_t>(kListCap);
          near_cnt = near_dense ? 0 : static_cast<int>(found);
#pragma unroll
          for (int e = 0; e < PER_LIST; ++e) {
            const int i = tid + e * THREADS;
            nz[e] = i < near_cnt ? zc[list[i]] : 0.f;
          }
        },
        [&](auto&& f) {
          if (near_dense) {
            for_each_logit([&](int, float z) {
              if (z >= thr_k) f(zkey(z), z);
            });
          } else {
#pragma unroll
            for (int e = 0; e < PER_LIST; ++e)
              if (tid + e * THREADS < near_cnt && nz[e] >= thr_k) f(zkey(nz[e]), nz[e]);
          }
        },
        m, zmin, a.top_p24, reinterpret_cast<unsigned long long*>(hist), sm);
    thr = key_to_float(pkey);
    // the kept ids sit at or above the threshold's prefix: a short list takes the common tail
    t16 = max(t16, pkey >> 16);
    count_candidates();
    if (ncand <= kListCap) {
      run_list(true, thr);
      return;
    }
  }
  float sum = 0.f;
  int cnt = 0;
  for_each_logit([&](int, float z) {
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
  const float lse_c = m + logf(S);
  if (tid == 0) {
    a.thr[R.oidx] = thr;
    a.lse[R.oidx] = lse_c;
    a.nkept[R.oidx] = Cn;
    if (a.flags && !(lse_c == lse_c && fabsf(lse_c) < INFINITY)) atomicOr(a.flags, 1);
  }
  if (a.mode == kRowSelectOnly) return;
  const int j = R.p0 + R.s;
  const float q_uniform = __fdiv_rn(1.0f, static_cast<float>(n));
  const uint2 key = seed_key(a.seed);
  const uint32_t w3 = static_cast<uint32_t>(R.b) << 8;
  const bool x_ok = R.x >= 0 && R.x < n;
  out.px = x_ok ? prob(zcx, thr, lse_c) : 0.f;
  out.qx = R.fresh ? q_uniform : (x_ok ? prob(zpx, R.thr_p, R.lse_p) : 0.f);
  const uint4 ra = philox4x32_10(make_uint4(0u, static_cast<uint32_t>(j), static_cast<uint32_t>(R.it),
                                            w3 | kStreamAccept), key);
  out.accept = __fmul_rn(u01(ra.x), out.qx) <= out.px;
  out.best = INFINITY;
  out.best_id = 0x7FFFFFFF;
  out.gbest = INFINITY;
  out.gbest_id = 0x7FFFFFFF;
  if (EXTRA && a.diag != nullptr && a.mode == kRowRing) {
    float d0 = 0.f, d1 = 0.f, d2 = 0.f;
    for_each_logit([&](int v, float z) {
      const float pv = prob(z, thr, lse_c);
      if (pv > 0.f) {
        const float qv = R.fresh ? q_uniform : prob(zp[v], R.thr_p, R.lse_p);
        d0 += fminf(pv, qv);
        d1 += pv * qv;
        d2 += pv * pv;
      }
    });
    row_statistics_out(a, R, d0, d1, d2, q_uniform, sm);
  }
  if (GS) {
    const PRace pr = p_race_of_row(a, key, w3, j, R.it);
    out.prace = pr.on;
    if (pr.on) {
      for_each_logit([&](int v, float z) {
        const float pv = prob(z, thr, lse_c);
        if (pv > 0.f) gumbel_entry(out, key, pr.w3s, j, pr.it, v, pv);
      });
    }
  }
  if (!out.accept) {
    for_each_logit([&](int v, float z) {
      const float pv = prob(z, thr, lse_c);
      if (pv > 0.f) {
        const float qv = R.fresh ? q_uniform : prob(zp[v], R.thr_p, R.lse_p);
        const float rv = __fsub_rn(pv, qv);
        if (rv > 0.f) {
          const uint4 rr = philox4x32_10(make_uint4(static_cast<uint32_t>(v >> 2), static_cast<uint32_t>(j),
                                                    static_cast<uint32_t>(R.it), w3 | kStreamResid), key);
          const uint32_t lanes[4] = {rr.x, rr.y, rr.z, rr.w};
          const float sc = __fdiv_rn(-logf(u01(lanes[v & 3])), rv);
          if (sc < out.best || (sc == out.best && v < out.best_id)) {
            out.best = sc;
            out.best_id = v;
          }
        }
      }
    });
  }
}

// The whole row in registers, PER logits per thread (n <= PER * THREADS).
template <int PER, bool GS, bool EXTRA>
__device__ __forceinline__ void direct_path(const RowArgs& a, const RowRef& R, unsigned char* smem,
                                            bool filter, float zcx, float zpx, Small& sm, RowOut& out) {
  const int tid = threadIdx.x, n = a.n;
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem);
  const bool vec_ok = (n & 3) == 0;
  const bool want_q = a.mode != kRowSelectOnly && !R.fresh;   // previous logits, for a rejection
  int vid[PER];
  float zv[PER], zq[PER];
  bool ok[PER];
#pragma unroll
  for (int u = 0; u < PER / 4; ++u) {
    const int v0 = (tid + u * THREADS) << 2;
    if (vec_ok && v0 + 3 < n) {
      const float4 t = *reinterpret_cast<const float4*>(R.zc + v0);
      zv[u * 4 + 0] = t.x; zv[u * 4 + 1] = t.y; zv[u * 4 + 2] = t.z; zv[u * 4 + 3] = t.w;
      float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
      if (want_q) q = *reinterpret_cast<const float4*>(R.zp + v0);
      zq[u * 4 + 0] = q.x; zq[u * 4 + 1] = q.y; zq[u * 4 + 2] = q.z; zq[u * 4 + 3] = q.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        zv[u * 4 + e] = (v0 + e < n) ? R.zc[v0 + e] : 0.f;
        zq[u * 4 + e] = (want_q && v0 + e < n) ? R.zp[v0 + e] : 0.f;
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vid[u * 4 + e] = v0 + e;
      ok[u * 4 + e] = v0 + e < n;
    }
  }
  uint32_t* cid = hist + NBINS;
  finish_regs<PER, true, GS, EXTRA>(a, R, vid, zv, zq, ok, filter, 0u, zcx, zpx, hist, cid,
                   reinterpret_cast<float*>(cid + kKeptCap),
                   reinterpret_cast<float*>(cid + 2 * kKeptCap), kKeptCap, sm, out);
}

// GS: the row also makes a Gumbel-max draw from p; EXTRA: the optional parts are compiled in
// (nucleus filter, per-position statistics; kept out of the other instances: their live ranges
// cost the hot kernels registers)
template <bool GS, bool EXTRA>
__global__ __launch_bounds__(THREADS) void row_kernel(const int32_t* const pos_, const int32_t* const iter_,
                                                      const int mode_, const int L_, const int N_,
                                                      const int P, const int capE, const RowArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ Small sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = a.n;
  const int r = blockIdx.x;
  const RowRef R = locate_row(a, r, pos_, iter_, mode_, L_, N_);
  if (!R.active) {
    if (tid == 0) {
      a.y[R.widx] = -1;
      a.k[R.widx] = 1;
      if (GS) a.g[R.widx] = -1;
      if (a.px) a.px[R.widx] = 0.f;
      if (a.qx) a.qx[R.widx] = 0.f;
      if (a.mode == kRowRing && R.s == 0) a.accept_len[R.b] = 0;   // finished sequence
      if (EXTRA && a.diag != nullptr && a.mode == kRowRing) {
        *reinterpret_cast<float4*>(a.diag + R.widx * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
        if (R.s == 0)
          for (int i = 0; i < 6; ++i) a.hamm[6 * R.b + i] = 0;
      }
    }
    return;
  }
  // the two logits of the draft token: their latency hides behind the selection
  const bool x_ok = a.mode != kRowSelectOnly && R.x >= 0 && R.x < n;
  const float zcx = x_ok ? R.zc[R.x] : 0.f;
  const float zpx = (x_ok && !R.fresh) ? R.zp[R.x] : 0.f;
  const bool filter = a.top_k > 0 && a.top_k < n;

  RowOut out{};
  out.accept = true;
  bool done = false;
  if (n <= kDirectMaxN) {
    // ---- the whole row in registers ------------------------------------------------
    if (n <= kDirectMaxN / 2) direct_path<PER_DIRECT / 2, GS, EXTRA>(a, R, smem, filter, zcx, zpx, sm, out);
    else direct_path<PER_DIRECT, GS, EXTRA>(a, R, smem, filter, zcx, zpx, sm, out);
    done = true;
  } else if (filter && a.cand && P > 0) {
    // ---- candidates emitted by the slice kernel ----------------------------------
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem + static_cast<size_t>((n + 7) & ~7) * 2);
    // The P counts and cuts of the row's lists (P slices of the slice kernel, or P column tiles
    // of the LM head's epilogue; thread t holds those of list t), the count that governs each
    // of this thread's candidate slots, and the slots themselves are fetched in ONE round trip:
    // slots are read whether filled or not (always inside the row's kListCap pairs) and masked
    // by the counts afterwards.
    const uint32_t* const cntp = a.cand_cnt + static_cast<size_t>(r) * P;
    const uint32_t* const cutp = a.cand_cut + static_cast<size_t>(r) * P;
    uint32_t tc = 0, tq = 0;
    if (tid < P) {
      tc = cntp[tid];
      tq = cutp[tid];
    }
    const uint2* src = a.cand + static_cast<size_t>(r) * kListCap;
    uint2 raw[PER_LIST];
    uint32_t slot_cnt[PER_LIST];
    int slot_off[PER_LIST];
#pragma unroll
    for (int e = 0; e < PER_LIST; ++e) {
      const int i = tid + e * THREADS;
      const int p = static_cast<int>(__umulhi(static_cast<uint32_t>(i), a.cand_recip));   // i / capE
      slot_off[e] = i - p * capE;
      raw[e] = src[i];
      slot_cnt[e] = cntp[p < P ? p : 0];
      if (p >= P) slot_cnt[e] = 0;
    }
    // every list fits its capacity, how many candidates there are, the largest cut
    {
      const int tot = wave_sum_i32(static_cast<int>(tc <= static_cast<uint32_t>(capE) ? tc : 0u));
      const uint32_t cm = wave_max_u32(tq);
      const bool anybad = __ballot(tc > static_cast<uint32_t>(capE)) != 0ull;
      if (lane == 0) {
        sm.ired2[wave] = tot;
        sm.wtot[wave] = cm;
        sm.ired[wave] = anybad ? 1 : 0;
      }
    }
    __syncthreads();                // their next writers sit behind the barrier of block_minmax
    bool fits = true;
    uint32_t cut_max = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      fits &= sm.ired[w] == 0;
      total += static_cast<uint32_t>(sm.ired2[w]);
      cut_max = sm.wtot[w] > cut_max ? sm.wtot[w] : cut_max;
    }
    if (fits && total >= static_cast<uint32_t>(a.top_k)) {
      int vid[PER_LIST];
      float zv[PER_LIST];
      bool ok[PER_LIST];
#pragma unroll
      for (int e = 0; e < PER_LIST; ++e) {
        ok[e] = static_cast<uint32_t>(slot_off[e]) < slot_cnt[e] && raw[e].x < static_cast<uint32_t>(n);
        vid[e] = ok[e] ? static_cast<int>(raw[e].x) : 0;
        zv[e] = ok[e] ? __uint_as_float(raw[e].y) : 0.f;
      }
      float zq[PER_LIST];                      // unused: finish_regs gathers what it needs
#pragma unroll
      for (int e = 0; e < PER_LIST; ++e) zq[e] = 0.f;
      const int ccap = min(kKeptCap, static_cast<int>(static_cast<size_t>((n + 7) & ~7) * 2 / 12));
      done = finish_regs<PER_LIST, false, GS, EXTRA>(a, R, vid, zv, zq, ok, true, cut_max, zcx, zpx, hist,
                                   reinterpret_cast<uint32_t*>(smem), reinterpret_cast<float*>(smem) + ccap,
                                   reinterpret_cast<float*>(smem) + 2 * ccap, ccap, sm, out);
    }
  }
  if (!done) full_path<GS, EXTRA>(a, R, smem, zcx, zpx, sm, out);
  if (a.mode == kRowSelectOnly) return;

  // ---- winner of the race (lexicographic (score, id) minimum) -------------------
  int y_out = R.x;
  int k_out = 1;
  if (!out.accept) {
    float best = out.best;
    int best_id = out.best_id;
    wave_min_score_id(best, best_id);
    if (lane == 0) {
      sm.s_score[wave] = best;
      sm.s_id[wave] = best_id;
    }
    __syncthreads();
    block_min_score_id(sm, best, best_id);
    if (best_id != 0x7FFFFFFF) {   // else: empty residual (rounding only) counts as accept
      y_out = best_id;
      k_out = 0;
    }
  }
  // ---- Gumbel-sharing draft of the row: the same reduction over (score, id) ---------
  int g_out = -1;
  if (GS) {
    float gb = out.gbest;
    int gi = out.gbest_id;
    wave_min_score_id(gb, gi);
    __syncthreads();               // the exchange arrays may still be read by the race above
    if (lane == 0) {
      sm.s_score[wave] = gb;
      sm.s_id[wave] = gi;
    }
    __syncthreads();
    block_min_score_id(sm, gb, gi);
    // empty support cannot happen (the maximum is kept); -1: the row made no such draw
    g_out = out.prace ? (gi != 0x7FFFFFFF ? gi : R.x) : -1;
  }
  if (a.mode != kRowRing) {
    if (tid == 0) {
      a.y[R.widx] = y_out;
      a.k[R.widx] = static_cast<uint8_t>(k_out);
      if (a.px) a.px[R.widx] = out.px;
      if (a.qx) a.qx[R.widx] = out.qx;
      if (GS) a.g[R.widx] = g_out;
    }
    return;
  }

  // ---- last workgroup of the sequence: first rejection, emit, slide -----------
  // Hand-off between workgroups WITHOUT an agent-scope fence (on this chip such a fence
  // writes back the whole L2 and costs tens of microseconds per launch).  The few bytes that
  // travel (y, k, g) are stored with agent-scope atomic stores, which are written through
  // to the device-coherent level.  The storing wavefront then WAITS until those stores have
  // been acknowledged (s_waitcnt vmcnt(0): the vector-memory counter of a wavefront covers
  // its stores on gfx950) and only then bumps the sequence's ticket with an agent-scope
  // atomic; a workgroup-scope fence alone does not make the compiler emit that wait.  The
  // last arriver (the one that reads live - 1 from the ticket) reads y, k, g back with
  // agent-scope atomic loads, which bypass the non-coherent cache levels.
  // Assumption about gfx950 stated here on purpose: an agent-scope atomic store is complete
  // at the device-coherent level when the issuing wavefront's vmcnt reaches zero, and
  // agent-scope atomic RMWs on one address are totally ordered, so every store of a row that
  // took an earlier ticket is visible to the workgroup that takes the last one.
  const int b = R.b, p0 = R.p0, live = R.live;
  if (tid == 0) {
    __hip_atomic_store(&a.y[R.widx], y_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&a.k[R.widx], static_cast<uint8_t>(k_out), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (GS) __hip_atomic_store(&a.g[R.widx], g_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (a.px) a.px[R.widx] = out.px;
    if (a.qx) a.qx[R.widx] = out.qx;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the stores above have completed
    sm.last = __hip_atomic_fetch_add(&a.ticket[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == live - 1;
    sm.first_rej = live;
  }
  __syncthreads();
  if (!sm.last) return;
  // nothing below may be moved above the ticket read (the barrier orders the other threads)
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  int yy = -1, gg = -1;
  if (tid < live) {
    yy = __hip_atomic_load(&a.y[static_cast<size_t>(b) * a.L + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (GS)
      gg = __hip_atomic_load(&a.g[static_cast<size_t>(b) * a.L + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint8_t kk = __hip_atomic_load(&a.k[static_cast<size_t>(b) * a.L + tid], __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    if (kk == 0) atomicMin(&sm.first_rej, tid);
  }
  __syncthreads();
  const int acc = min(sm.first_rej + 1, live);
  if (tid < acc) a.out[static_cast<size_t>(b) * a.N + p0 + tid] = a.v_lo + yy;
  const bool stats = EXTRA && a.diag != nullptr;
  const int ring = R.it % 3;
  if (stats) {
    // the drafts this iteration started with, by ring slot, and where its window started
    if (tid < a.L) a.xhist[(static_cast<size_t>(ring) * a.B + b) * a.L + tid] = a.X[static_cast<size_t>(b) * a.L + tid];
    if (tid == 0) a.phist[ring * a.B + b] = p0;
    if (tid < 6) sm.hamm[tid] = 0;
    __syncthreads();                 // slot tid is rewritten by another thread below
  }
  if (tid < live) {
    const int slot = (p0 + tid) % a.L;
    const size_t sidx = static_cast<size_t>(b) * a.L + slot;
    int next;
    if (tid >= acc) {
      // survivors: the MRS output is the coupled redraft (pi_MC); under pi_GS, or when the
      // alpha-coupling switch chose the independent redraft, it is the row's Gumbel-max draw
      next = (GS && gg >= 0) ? gg : yy;
      a.age_w[sidx] += 1;
    } else {
      const int np = p0 + a.L + tid;
      next = np < a.N ? init_token(a.seed, b, np, n) : -1;
      a.age_w[sidx] = 0;
    }
    a.X[sidx] = next;
    if (stats) sm.xnew[slot] = next;
  }
  if (tid == 0) {
    a.accept_len[b] = acc;
    a.pos[b] = p0 + acc;
    a.iter[b] = R.it + 1;
    a.verified[b] += live;
    a.ticket[b] = 0;
  }
  if (stats) {
    // Hamm(t + 1 - n, t + 1), n = 1..3 (Sec. 5.3 "Multi-Step Behavior"): the new drafts against
    // those of n iterations earlier over the positions that sit in both windows.  The thread of
    // ring slot tid owns the position j of the new window with j % L == tid.
    __syncthreads();
    const int pnew = p0 + acc;
    if (tid < a.L) {
      const int j = pnew + (tid - pnew % a.L + a.L) % a.L;
      if (j < a.N && j < p0 + a.L) {               // a position the step left in the window
        const int xn = sm.xnew[tid];
#pragma unroll
        for (int back = 0; back < 3; ++back) {
          const int ri = (ring + 3 - back) % 3;
          const int ph = back == 0 ? p0 : a.phist[ri * a.B + b];
          if (j >= ph && j < ph + a.L) {
            const int xo = a.xhist[(static_cast<size_t>(ri) * a.B + b) * a.L + tid];
            atomicAdd(&sm.hamm[2 * back + 1], 1);
            if (xo != xn) atomicAdd(&sm.hamm[2 * back], 1);
          }
        }
      }
    }
    __syncthreads();
    if (tid < 6) a.hamm[6 * b + tid] = sm.hamm[tid];
  }
}

size_t lds_bytes_for(int n) {
  if (n <= kDirectMaxN) return NBINS * sizeof(uint32_t) + kKeptCap * 12;
  return static_cast<size_t>((n + 7) & ~7) * 2 + NBINS * sizeof(uint32_t) + kListCap * sizeof(uint16_t);
}

inline size_t small_block(int rows) {
  return (static_cast<size_t>(rows) * kRowMaxTiles * 4 + 255) / 256 * 256;
}

}  // namespace

#ifndef SCD_ROW_BATCHED
size_t row_candidate_bytes(int rows) {
  // per row: kListCap (id, logit) pairs, kRowMaxTiles list counts, kRowMaxTiles list cuts
  return static_cast<size_t>(rows) * kListCap * sizeof(uint2) + 2 * small_block(rows);
}

void row_candidate_layout(void* base_, int rows, uint2** cand, uint32_t** cnt, uint32_t** cut) {
  char* base = static_cast<char*>(base_);
  const size_t pairs = static_cast<size_t>(rows) * kListCap * sizeof(uint2);
  *cand = reinterpret_cast<uint2*>(base);
  *cnt = reinterpret_cast<uint32_t*>(base + pairs);
  *cut = reinterpret_cast<uint32_t*>(base + pairs + small_block(rows));
}

bool row_uses_candidates(int n, int top_k) {
  const bool filter = top_k > 0 && top_k < n;
  return n > kDirectMaxN && n <= kRowKernelMaxN && filter && top_k <= kListCap / 2;
}

#endif  // !SCD_ROW_BATCHED

hipError_t LAUNCH_ROW(const RowArgs& a_in, hipStream_t s, size_t* lds_configured) {
  if (a_in.rows <= 0) return hipSuccess;
#ifdef SCD_ROW_BATCHED
  if (a_in.n > kDirectMaxN) return hipErrorInvalidValue;     // this build holds whole rows in registers only
#else
  // more rows than compute units (256 on this chip), short rows, the hot instances: the build
  // of this file whose workgroups pair up on a CU
  if (a_in.rows > 256 && a_in.n <= kRowBatchedMaxN && a_in.top_p24 == 0u && a_in.diag == nullptr)
    return launch_row_batched(a_in, s, lds_configured ? lds_configured + 1 : nullptr);
#endif
  RowArgs a = a_in;
  int P = 0, capE = 0;
  a.cand = nullptr;
  if (a.cand_base && row_uses_candidates(a.n, a.top_k)) {
    row_candidate_layout(a.cand_base, a.rows, &a.cand, &a.cand_cnt, &a.cand_cut);
    if (a.tiles > 0) {
      // the LM head's epilogue has filled the lists: one per 256-column tile
      P = a.tiles;
      capE = kListCap / P;
    } else {
      P = (a.n + kSliceMax - 1) / kSliceMax;                     // <= 8 for n <= 65536
      capE = kListCap / P;
      int rank = (2 * a.top_k + P - 1) / P;
      rank = rank < 64 ? 64 : rank;
      if (rank > capE * 4 / 5) rank = capE * 4 / 5;
      if (a.rows * P > 512)
        hipLaunchKernelGGL(slice_kernel<512>, dim3(a.rows * P), dim3(512), 0, s, a.pos, a.iter, a.mode, a.L, a.N, P,
                           capE, rank, a);
      else
        hipLaunchKernelGGL(slice_kernel<THREADS>, dim3(a.rows * P), dim3(THREADS), 0, s, a.pos, a.iter, a.mode, a.L,
                           a.N, P, capE, rank, a);
      if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
  }
  const size_t lds = lds_bytes_for(a.n);
  // The dynamic-LDS limit is an attribute of the function on a device.  Every context asks
  // for the same value, the largest any row needs, once (a context has one stream, hence one
  // device), so contexts of different row lengths cannot lower each other's limit.
  size_t none = 0;
  size_t& configured = lds_configured ? *lds_configured : none;
  if (configured == 0) {
    const size_t most = lds_bytes_for(kRowKernelMaxN);
    for (const void* f : {reinterpret_cast<const void*>(row_kernel<false, false>),
                          reinterpret_cast<const void*>(row_kernel<true, false>),
                          reinterpret_cast<const void*>(row_kernel<false, true>),
                          reinterpret_cast<const void*>(row_kernel<true, true>)}) {
      hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(most));
      if (e != hipSuccess) return e;
    }
    configured = most;
  }
  const bool gs = (a.gumbel || a.alpha < 1.0f) && a.g && a.mode != kRowSelectOnly;
  const bool topp = a.top_p24 != 0u || a.diag != nullptr;   // the instances with the optional parts
  auto* const kernel = gs ? (topp ? row_kernel<true, true> : row_kernel<true, false>)
                          : (topp ? row_kernel<false, true> : row_kernel<false, false>);
  a.cand_recip = capE > 0 ? static_cast<uint32_t>(((1ull << 32) + capE - 1) / capE) : 0u;
  hipLaunchKernelGGL(kernel, dim3(a.rows), dim3(THREADS), lds, s, a.pos, a.iter, a.mode, a.L, a.N, P, capE, a);
  return hipGetLastError();
}

}  // namespace scd
