/*
 * scd_workload.h -- device-side plumbing for the synthetic benchmark inputs.
 * Not part of the decoding method: a pure index gather (no arithmetic) that
 * assembles the hidden-state rows of the current Jacobi windows from a
 * pre-generated table, so that a benchmark loop never leaves the device.
 */
#ifndef SCD_WORKLOAD_H
#define SCD_WORKLOAD_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* d_h[b, c, s, :] = d_table[b, c, pos, min(age, age_cap), :] for pos = d_pos[b] + s < N,
 * age = d_age[b, pos % L]; rows with pos >= N are zero-filled.
 *   d_table bf16 bits [B, C, N, age_cap + 1, d];  d_pos int32 [B];  d_age int32 [B, L]
 *   (ring slots, as in the decode state);  d_h bf16 bits [B, C, L, d], written.
 * d must be a multiple of 8 and all pointers 16-byte aligned.  Asynchronous on
 * hip_stream (a hipStream_t as void*).  Returns 0, -1 (bad argument) or -3
 * (launch failed). */
int scdw_gather_hidden(void* hip_stream, const uint16_t* d_table, int32_t B, int32_t C, int32_t L,
                       int32_t N, int32_t d, int32_t age_cap, const int32_t* d_pos,
                       const int32_t* d_age, uint16_t* d_h);

/* Plain device copy d_dst[0 .. bytes) = d_src[0 .. bytes) by one kernel (copy_kernel) that
 * reads and writes every byte exactly once with 16-byte accesses.  It exists so that a
 * profiler's HBM byte counters can be scaled by what they report for a transfer of known
 * size.  bytes must be a multiple of 16, both pointers 16-byte aligned and the ranges
 * disjoint.  Asynchronous on hip_stream.  Returns 0, -1 (bad argument) or -3. */
int scdw_copy(void* hip_stream, const void* d_src, void* d_dst, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif
