/*
 * chunk_plan.h -- C ABI of the host-side sequence processor that feeds the chunk-attention library.
 *
 * It turns the lengths of the sequences of one training batch into chunks {C, S} (paper section 3.1):
 * long sequences are split along a workload-balanced "mesh" into split chunks plus a tail slice, and
 * tail slices and short sequences are packed into hybrid and batched chunks of balanced time and
 * token count (paper section 3.3, Algorithm 1, "Workload-Balanced Sequence Processing for
 * Heterogeneous Chunks").  Times come from the paper's cost model (section 3.2.1, Eq. 1 plus the
 * all-to-all term of Eq. 3, summed as in Eq. 4).  Everything here runs on the host; no GPU is touched.
 *
 * Where the paper's sketch leaves a step open, this is what is implemented:
 *   - "K workload-balanced slices" (the mesh step): the mesh whose largest slice time T_tot is as small as it can be, slices
 *     being multiples of `align` except the last;
 *   - the token threshold T_m (the paper refers to its repository): min(capacity, first mesh slice);
 *   - time of a bucket with one more sequence (the fit test of the packing loop): T_tot of the combined chunk, i.e. the per-chunk constants of
 *     Eq. 1 and Eq. 3 are paid once; buckets are tried in ascending tot_time / tot_tokens, ties in order of creation;
 *   - relaxing T_t (when no bucket accepts the sequence): the smallest combined time among the buckets that have room for the sequence's tokens
 *     (the minimum over all buckets would not terminate when the cheapest bucket is full).
 *
 * All pointers are HOST pointers owned by the caller.  Functions return CHUNK_ATTN_OK (0) or a negative
 * code of chunk_attn.h (INVALID_ARG for null pointers, non-positive sizes or an output array that is
 * too small) and never throw or abort.
 */
#ifndef CHUNK_PLAN_H_
#define CHUNK_PLAN_H_

#include <stddef.h>
#include <stdint.h>

#include "chunk_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Cost model of one chunk (seconds or any other unit):
 *   T_tot(C, S) = ( alpha1 ((C + s0)^2 - C^2) + alpha2 s0 + sum_{s in S - {s0}} (alpha1 s^2 + alpha2 s) ) / n_devices
 *                 + beta1 / dp + a2a_per_token * sum_{s in S} s + a2a_const
 * (Eq. 1: quadratic attention term, linear term, constant; Eq. 3 contributes a term linear in the tokens and a
 * constant).  alpha1 > 0; the other coefficients >= 0; n_devices, dp >= 1.
 */
typedef struct {
  double alpha1, alpha2, beta1;
  double a2a_per_token, a2a_const;
  int32_t n_devices, dp;
} chunk_cost_model;

/* One slice: tokens [start, start + len) of input sequence `seq`. */
typedef struct {
  int32_t seq, start, len;
} chunk_plan_slice;

/* One chunk {C, S}: slices[first_slice .. first_slice + num_slices); `context` is C, the number of
 * tokens of slices[first_slice].seq that precede the chunk's first slice (0 for a batched chunk);
 * is_split is the paper's indicator I (1 only for a chunk that is one non-final slice of a long sequence). */
typedef struct {
  int64_t context;
  int32_t first_slice, num_slices;
  int32_t is_split;
  int32_t tokens;
  double time; /* T_tot(C, S) */
} chunk_plan_chunk;

/* T_tot of a chunk with context C and slice lengths S[0..n). */
double chunk_plan_time(const chunk_cost_model* model, int64_t context, const int32_t* slice_lens, int32_t n);

/*
 * Mesh (the first step of Algorithm 1): split a sequence of max_len tokens into K slices of (nearly) equal T_tot, slice
 * k having the slices before it as context.  Slice lengths are multiples of `align` (>= 1) except the last,
 * which takes the remainder; every slice has at least one token (K is lowered if max_len < K * align; the
 * number of slices actually produced is returned in *k_out).  Also returns the initial time threshold T_t
 * (the largest slice time of the mesh) and the token threshold T_m = min(capacity, mesh[0]).
 */
int chunk_plan_mesh(const chunk_cost_model* model, int32_t max_len, int32_t K, int32_t align, int64_t capacity,
                    int32_t* mesh, int32_t* k_out, double* time_threshold, int64_t* token_threshold);

/*
 * Algorithm 1.  lengths[0..n_seqs): tokens per sequence (>= 1).  Outputs: chunks[0..*n_chunks) (split chunks
 * first, in sequence order, then the packed chunks) and slices[0..*n_slices).  Array capacities max_chunks,
 * max_slices: n_seqs * (K + 1) each always suffices.  *time_threshold receives the final (possibly relaxed) T_t,
 * *token_threshold T_m.
 */
int chunk_plan_build(const chunk_cost_model* model, int64_t capacity, const int32_t* lengths, int32_t n_seqs, int32_t K,
                     int32_t align, chunk_plan_chunk* chunks, int32_t max_chunks, int32_t* n_chunks,
                     chunk_plan_slice* slices, int32_t max_slices, int32_t* n_slices, double* time_threshold,
                     int64_t* token_threshold);

/*
 * Segment table of one chunk for chunk_attn_fwd / chunk_attn_bwd: the first slice attends to its context
 * (its key/value rows are [context rows | own rows]), every further slice is an independent sequence.
 * segs must hold chunk->num_slices entries.  *total_q, *total_kv receive the row counts of the chunk's
 * Q and K/V tensors.
 */
int chunk_plan_segments(const chunk_plan_chunk* chunk, const chunk_plan_slice* slices, chunk_attn_seg* segs,
                        int32_t* total_q, int32_t* total_kv);

#ifdef __cplusplus
}
#endif
#endif /* CHUNK_PLAN_H_ */
