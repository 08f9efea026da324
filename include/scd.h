/*
 * scd.h -- C ABI of the MI355X (gfx950) library for the per-iteration
 * draft-and-verify pass of Speculative Coupled Decoding (SCD).
 *
 * What one iteration computes (appendix "Algorithms", Alg. SCD(pi_MC); Sec. 4.3
 * "Implementation Details"; Alg. 1 "Modified Rejection Sampling"):
 *   1. Evaluate: LM-head logits of the L window positions,
 *        logit[m, v] = sum_k h[m, k] * W[v, k]           (bf16 in, fp32 accumulate)
 *   2. logit post-processing, which defines p^(t) (Sec. 4.3, last sentence;
 *      Sec. 5.1 "Effect on CFG"; appendix "Experimental Details"):
 *        z = (1 + lambda) * c - lambda * u   (classifier-free guidance, C = 2 rows)
 *        ids outside [v_lo, v_hi) are masked out;  z <- z / tau
 *        keep the ids with z >= (K-th largest z);  p = softmax over the kept ids
 *   3. one Modified-Rejection-Sampling call per window position, no break:
 *        u ~ U(0,1);  accept iff  u * q(x) <= p(x)              (k = 1, y = x)
 *        else y ~ norm(max(0, p - q))                             (k = 0)
 *      q is the position's distribution from the previous iteration (uniform
 *      over the allowed ids if it was never evaluated), x its current draft.
 *   4. first rejection r: emit y[0..a), a = min(r + 1, Lw) (a = Lw if none);
 *      the y right of r are the coupled redraft = next iteration's drafts;
 *      slide the window by a and give the entering positions uniform drafts.
 * With coupling = SCD_COUPLING_GS (Alg. "GS(P, Q, G)", appendix Alg. SCD(pi_GS)) steps 1-3
 * and the emission are the same; the redraft of the positions right of r is instead the
 * shared-noise Gumbel-max draw from the position's new distribution,
 *        g = argmax_v (log p(v) + G_j(v)),  G_j(v) = -ln(-ln U_j(v)),
 * with noise that depends on the position j (and the id v) only, not on the iteration,
 * decided as the equivalent exponential race argmin_v -ln(U_j(v)) / p(v) in fp32.
 * With sjd_mix > 0 (alpha-coupling, Sec. 5.3 and appendix Alg. "alpha-Coupling
 * Implementation", alpha = 1 - sjd_mix): per redraft one uniform u (stream 4); if
 * u <= alpha (fp32, alpha = fl(1 - sjd_mix)) the coupled redraft above is taken, otherwise an
 * independent draw from p: the same race with noise keyed by position AND iteration (stream 5).
 *
 * Conventions
 *   - Every pointer named d_* is a DEVICE pointer owned by the caller.  The
 *     library allocates no device memory, frees nothing of the caller's and
 *     never synchronises the stream (scd_status is the one exception).
 *   - Every call returns SCD_OK (0) or a negative scd_error.  No exceptions,
 *     no errno, no global state (the one exception: the library remembers, per
 *     GPU, the address of the static scratch of scd_couple_draft_static).  Kernels are launched asynchronously on the
 *     HIP stream given to scd_create.
 *   - A context is not thread-safe; distinct contexts are independent.
 *   - "Allowed ids" A = [v_lo, v_hi), n = |A|.  Tokens in x / y / the state are
 *     OFFSETS into A (0..n-1); emitted tokens (out) are real ids v_lo + offset.
 *     Processed logits z hold only the n allowed columns.
 *   - Rows of up to 65536 allowed ids run through one fused kernel per row (plus the LM
 *     head).  Longer rows are supported with top-k and the maximal coupling only (one kernel
 *     per stage: select, MRS, commit); Gumbel sharing, sjd_mix > 0, top_p and diagnostics on
 *     such rows are refused by scd_create with SCD_EUNSUPPORTED.
 *   - Window order: row s of a [B, L, ...] array belongs to position pos0[b]+s.
 *     Lw_b = min(L, N - pos0[b]) rows are live; the rest are ignored on input
 *     and written as y = -1, k = 1 on output.
 *   - Random numbers: Philox4x32-10, key = (seed low 32, seed high 32),
 *     counter = (vocab offset >> 2 or 0, position, iteration, b << 8 | stream),
 *     lane = vocab offset & 3 (lane 0 for scalar draws); streams 0 = initial
 *     draft, 1 = accept uniform, 2 = residual race, 3 = Gumbel noise (iteration
 *     word 0), 4 = alpha-coupling switch, 5 = independent redraft.
 *     u = ((bits >> 9) + 0.5) * 2^-23.
 */
#ifndef SCD_H
#define SCD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct scd_ctx scd_ctx; /* opaque, host memory, owned by the library */

typedef struct scd_config {
  int32_t B;           /* sequences decoded together, >= 1                         */
  int32_t L;           /* Jacobi window length, 1..256                              */
  int32_t N;           /* tokens to generate per sequence, >= 1                     */
  int32_t V;           /* vocabulary size = rows of W                               */
  int32_t d;           /* hidden size, multiple of 8; 0 => no LM head (logits given) */
  int32_t v_lo, v_hi;  /* allowed ids [v_lo, v_hi), 0 <= v_lo < v_hi <= V;
                          L * (v_hi - v_lo) must stay below 2^31                    */
  int32_t top_k;       /* 0 => off; K = min(top_k, n)                               */
  float temperature;   /* tau > 0                                                   */
  float cfg_lambda;    /* 0 => no guidance (C = 1); else C = 2, z = (1+l)c - l u    */
  int32_t coupling;    /* scd_coupling: 0 = maximal coupling (MRS), 1 = Gumbel sharing */
  float sjd_mix;       /* 1 - alpha of the alpha-coupling (Sec. 5.3): probability that a
                          redraft is an independent draw from p instead of the coupled one;
                          0 = SCD (default), 1 = vanilla SJD; must be in [0, 1]          */
  float top_p;         /* nucleus filter (appendix "Experimental Details", video setting
                          p = 0.8), applied to the distribution that top-k leaves: of the ids
                          in order of decreasing probability the shortest prefix whose mass
                          reaches top_p is kept, ids tied with its last member included;
                          0 or 1 => off; must be in [0, 1]; needs v_hi - v_lo <= 65536.
                          Decided on 2^-40 fixed-point masses of expf(z - max), exactly:
                          mass above an id * 2^24 < round(top_p * 2^24) * total mass          */
  int32_t diagnostics; /* 1 => every scd_step also writes the per-position statistics of the
                          paper's analysis (Sec. 3: acceptance rate beta = 1 - D_TV(p, q),
                          Prop. "SJD Collision Probability": C = sum_v p_v q_v and the two
                          sums its Renyi-2 bound needs) to SCD_F_DIAG and the number of changed
                          drafts (Hamming distance between the drafts 1, 2 and 3 iterations
                          apart, Sec. 5.3 "Multi-Step Behavior") to SCD_F_HAMM;
                          0 => off; needs v_hi - v_lo <= 65536                               */
  uint64_t seed;
} scd_config;

typedef enum scd_coupling {
  SCD_COUPLING_MC = 0,   /* survivors' next drafts = their MRS outputs (Sec. 4.1)            */
  SCD_COUPLING_GS = 1    /* survivors' next drafts = shared-noise Gumbel-max draws; needs
                            v_hi - v_lo <= 65536                                             */
} scd_coupling;

typedef enum scd_error {
  SCD_OK = 0,
  SCD_EINVAL = -1,       /* bad argument or configuration                       */
  SCD_EWORKSPACE = -2,   /* workspace pointer null / misaligned / too small      */
  SCD_EHIP = -3,         /* a HIP runtime call or kernel launch failed           */
  SCD_ENUMERIC = -4,     /* a logit row had no finite value or a NaN (scd_status) */
  SCD_EUNSUPPORTED = -5, /* valid request this build does not implement          */
  SCD_ESCRATCH = -6      /* scd_couple_draft_static: the configuration needs more than
                            SCD_STATIC_SCRATCH_BYTES of scratch                   */
} scd_error;

/* Fields of the device-resident decode state, for scd_state_field. */
typedef enum scd_field {
  SCD_F_POS = 0,      /* int32 [B]       accepted-prefix pointer i_b                   */
  SCD_F_ITER = 1,     /* int32 [B]       iterations done t_b (= NFE)                   */
  SCD_F_X = 2,        /* int32 [B, L]    draft token offsets, ring slot = position % L */
  SCD_F_AGE = 3,      /* int32 [B, L]    earlier evaluations of the slot's position    */
  SCD_F_OUT = 4,      /* int32 [B, N]    emitted token ids, -1 where not yet emitted   */
  SCD_F_ACCEPT = 5,   /* int32 [B]       tokens emitted by the last step               */
  SCD_F_Y = 6,        /* int32 [B, L]    last step's MRS outputs, window order         */
  SCD_F_K = 7,        /* uint8 [B, L]    last step's accept bits, window order         */
  SCD_F_PX = 8,       /* float [B, L]    last step's p(x), window order                */
  SCD_F_QX = 9,       /* float [B, L]    last step's q(x), window order                */
  SCD_F_THR = 10,     /* float [2, B, L] smallest kept logit (top-k / nucleus threshold; -inf when
                                         neither filters) per parity (t & 1) and slot  */
  SCD_F_LSE = 11,     /* float [2, B, L] log normaliser per parity and slot            */
  SCD_F_NKEPT = 12,   /* int32 [2, B, L] size of the kept set per parity and slot      */
  SCD_F_Z = 13,       /* float [2, B, L, n] processed logits per parity and slot       */
  SCD_F_FLAGS = 14,   /* int32 [4]       [0] numeric-fault bits                        */
  SCD_F_VERIFIED = 15,/* int32 [B]       window positions verified so far (sum of Lw)  */
  SCD_F_TICKET = 16,  /* int32 [B]       internal arrival counters, zero between steps */
  SCD_F_G = 17,       /* int32 [B, L]    last step's Gumbel-sharing / independent redraft draws,
                                         window order; -1 where the row drew none (written
                                         under SCD_COUPLING_GS or sjd_mix > 0 only)      */
  SCD_F_DIAG = 18,    /* float [B, L, 4] last step, window order (diagnostics = 1 only):
                                         [0] beta = sum_v min(p_v, q_v) = 1 - D_TV(p, q)
                                         [1] C = sum_v p_v q_v
                                         [2] sum_v p_v^2 = exp(-H_2(p))   [3] sum_v q_v^2
                                         (C <= sqrt([2] * [3])); p = this iteration's
                                         distribution of the position, q = the one its draft
                                         came from (uniform for a first evaluation); rows that
                                         are not live hold zeros                             */
  SCD_F_S2 = 19,      /* float [2, B, L] internal: sum_v p_v^2 per parity and slot            */
  SCD_F_HAMM = 20,    /* int32 [B, 6]    last step (diagnostics = 1 only): for n = 1, 2, 3 the pair
                                         (differing, compared) of Hamm(t + 1 - n, t + 1): the
                                         window's drafts after the step against the drafts n
                                         iterations earlier, over the positions in both windows
                                         (n = 1: the surviving positions whose draft changed)  */
  SCD_F_XHIST = 21,   /* int32 [3, B, L] internal: drafts at the start of the last 3 iterations */
  SCD_F_PHIST = 22,   /* int32 [3, B]    internal: window starts of those iterations            */
  SCD_F_COUNT = 23
} scd_field;

/* Bytes of caller-provided device scratch a context needs; 0 on a bad config. */
size_t scd_workspace_bytes(const scd_config* cfg);

/* Bytes of the device-resident decode state; 0 on a bad config. */
size_t scd_state_bytes(const scd_config* cfg);

/* Validates cfg, copies it, remembers the workspace (256-byte aligned device
 * memory of >= scd_workspace_bytes, kept by the caller until scd_destroy) and
 * the HIP stream (a hipStream_t passed as void*, NULL = default stream).
 * *out is set only on SCD_OK. */
int scd_create(scd_ctx** out, const scd_config* cfg, void* d_workspace, size_t workspace_bytes,
               void* hip_stream);

/* Frees the host-side context.  Touches no device memory. */
int scd_destroy(scd_ctx* ctx);

/* Initialises a state buffer (256-byte aligned, >= scd_state_bytes): i_b = 0,
 * t_b = 0, the first min(L, N) positions get uniform initial drafts, out = -1.
 * Asynchronous. */
int scd_reset(scd_ctx* ctx, void* d_state);

/* Host-only address arithmetic: pointer and size of one field inside d_state. */
int scd_state_field(const scd_ctx* ctx, void* d_state, int field, void** d_ptr, size_t* bytes);

/* Step 1+2a (Evaluate + CFG + mask + temperature) for all B*L window rows.
 *   d_h  bf16 bits [B, C, L, d] row-major (C = 2: cond rows then uncond rows of
 *        each sequence);  d_W bf16 bits [V, d] row-major; only rows
 *        [v_lo, v_hi) are read;  d_z fp32 [B, L, n] window order, written.
 * Requires cfg.d > 0. */
int scd_lm_head(scd_ctx* ctx, const uint16_t* d_h, const uint16_t* d_W, float* d_z);

/* Step 2b (top-k threshold + softmax normaliser) for rows of processed logits.
 *   d_z fp32 [rows, n];  outputs per row: d_thr (K-th largest value, -inf if
 *   top-k is off or K >= n), d_lse (log of the sum of exp over the kept ids),
 *   d_nkept (size of the kept set).  p_v = [z_v >= thr] * exp(z_v - lse). */
int scd_select(scd_ctx* ctx, const float* d_z, int32_t rows, float* d_thr, float* d_lse,
               int32_t* d_nkept);

/* Step 3: vectorised MRS = speculative verification and maximal-coupling
 * redraft in one call (Alg. 1; Alg. SCD(pi_MC) parallel-for).
 *   d_z_cur, d_z_prev fp32 [B, L, n] processed logits of this / the previous
 *   iteration, window order;  d_x int32 [B, L] draft token offsets;
 *   d_fresh uint8 [B, L], nonzero = never evaluated (q uniform; d_z_prev row
 *   unread), may be NULL = none fresh;  d_pos0 int32 [B];  iter = iteration
 *   index used in the random-number counters;
 *   outputs d_y int32 [B, L], d_k uint8 [B, L]. */
int scd_couple_draft(scd_ctx* ctx, const float* d_z_cur, const float* d_z_prev,
                     const int32_t* d_x, const uint8_t* d_fresh, const int32_t* d_pos0,
                     int32_t iter, int32_t* d_y, uint8_t* d_k);

/* scd_couple_draft for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels,
 * same results; the scratch that scd_couple_draft keeps in the context's workspace (per-row
 * thresholds / normalisers / kept counts of both logit arrays and the slice kernel's candidate
 * lists) lives in a static device array of SCD_STATIC_SCRATCH_BYTES inside the library instead
 * (one copy per GPU, held until the process ends).  The call allocates and frees nothing and
 * does not touch the context's workspace.  Returns SCD_ESCRATCH when the configuration needs
 * more: 24 bytes per window row (B * L rows, each of the six arrays rounded up to 256 bytes),
 * plus 51200 bytes per window row when top-k filters rows of 16385..65536 ids with
 * top_k <= 3072 (the slice kernel's candidate lists), i.e. up to 163 such rows.
 * All calls on one GPU share that array and it keeps the last call's contents (nothing in it has
 * to start at zero): calls that overlap in time on one GPU -- different streams or contexts --
 * race.  The array's address is looked up once per GPU, in scd_create when a GPU is present,
 * else in the first call. */
#define SCD_STATIC_SCRATCH_BYTES (8u << 20)
int scd_couple_draft_static(scd_ctx* ctx, const float* d_z_cur, const float* d_z_prev,
                            const int32_t* d_x, const uint8_t* d_fresh, const int32_t* d_pos0,
                            int32_t iter, int32_t* d_y, uint8_t* d_k);

/* Step 4 without the slide: first rejection per sequence, accept length and
 * emitted tokens (Alg. SCD(pi_MC), "find first rejection index").
 *   d_k, d_y [B, L] from scd_couple_draft; d_pos0 [B];
 *   d_accept_len int32 [B] written; d_out int32 [B, N]: entries
 *   [pos0, pos0 + accept_len) written with v_lo + y. */
int scd_verify(scd_ctx* ctx, const uint8_t* d_k, const int32_t* d_y, const int32_t* d_pos0,
               int32_t* d_accept_len, int32_t* d_out);

/* One whole iteration (steps 1-4 incl. window slide) on the device-resident
 * state.  d_h as in scd_lm_head for the CURRENT windows (row s <-> position
 * i_b + s; rows past the sequence end are ignored but must be readable).
 * Finished sequences cost nothing and change nothing.  Requires cfg.d > 0. */
int scd_step(scd_ctx* ctx, const uint16_t* d_h, const uint16_t* d_W, void* d_state);

/* Optional instrumentation for benchmarks: while both events are non-NULL,
 * scd_step launches the LM-head kernel with the two events attached to the
 * dispatch (hipExtLaunchKernel): ev_start takes the kernel's start time, ev_stop
 * its stop time, on the context's stream; no other packet enters the stream
 * (hipEvent_t passed as void*, owned by the caller).  NULL, NULL turns it off.
 * Host-only call. */
int scd_set_lm_head_events(scd_ctx* ctx, void* ev_start, void* ev_stop);

/* For reports: writes the name of the LM-head kernel that scd_step / scd_lm_head launch
 * for this context's sizes, e.g. "lm_head_splitk_kernel<1, 2, 8>" (template arguments:
 * row blocks per workgroup, 1 + CFG, wavefronts), NUL-terminated, into host_buf[0..cap).
 * Returns SCD_OK, or SCD_EINVAL (NULL argument, cfg.d == 0, or cap too small).
 * Host-only call. */
int scd_lm_head_kernel_name(scd_ctx* ctx, char* host_buf, size_t cap);

/* The same iteration with the processed logits supplied by the caller
 * (d_z fp32 [B, L, n], window order) instead of computed by the LM head. */
int scd_step_logits(scd_ctx* ctx, const float* d_z, void* d_state);

/* Synchronises the stream and reports: host_flags[0] = numeric-fault bits,
 * host_flags[1] = 1 if every sequence has emitted N tokens, host_flags[2] =
 * largest t_b, host_flags[3] = 0.  Returns SCD_ENUMERIC if a fault bit is set. */
int scd_status(scd_ctx* ctx, void* d_state, int32_t host_flags[4]);

const char* scd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SCD_H */
