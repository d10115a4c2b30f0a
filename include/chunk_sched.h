/*
 * chunk_sched.h -- C ABI of the host-side chunk scheduler that sits between the sequence processor
 * (chunk_plan.h) and the chunk-attention kernels (chunk_attn.h).
 *
 * It decides how the chunks of one training batch are run (paper section 3.4, "Chunk Scheduler"):
 *   - the sequences are grouped by the number of chunks they were cut into, each group running as one 1F1B
 *     pipeline (section 3.4.2, "Sequence Grouping": dynamic programme over dp[i], the cheapest way to run all
 *     sequences of at most i chunks, a pipeline costing delta + T_ckpt(P));
 *   - inside a pipeline, every chunk gets a number of checkpointed layers per stage, ckpt(p, k) =
 *     C[f2b[k] + d_p - p], the n + d_p - 1 integers C chosen with the smallest sum such that every chunk window
 *     of every stage fits the memory capacity (section 3.4.3, "Stage-Aware Chunk-Level Adaptive Checkpointing",
 *     Algorithm 2; memory model of sections 3.2.2 and 3.2.3).  The paper hands this integer programme to a
 *     solver library; here it is solved by best-first branch and bound over linear relaxations (dense simplex,
 *     rounding cuts at the root), to optimality or to a relative gap the caller gives;
 *   - a 1F1B timeline of a pipeline (makespan, busy time and peak memory per stage) to check a plan.
 * Everything runs on the host; no GPU is touched.
 *
 * Stages are numbered p = 1 .. d_p as in the paper, chunks 0 .. n - 1 in forward order.
 * Where the paper leaves a step open, this is what is implemented:
 *   - N (devices an activation is spread over) = d_p * d_s, the value for which the footprint of section 3.2.3
 *     and the coefficients of Algorithm 2 agree;
 *   - forward order of a pipeline: sequences with more chunks first (then more tokens, then input order), the
 *     chunks of a sequence in order; backward order: same order of sequences, chunks of a sequence last to first;
 *   - stage p runs min(n, d_p - p + N_split) forward passes, then alternates backward / forward, then the remaining
 *     backward passes; a chunk window is taken after each forward pass;
 *   - delta is passed in by the caller ((d_p - 1) * average chunk time in the paper);
 *   - a range of chunk counts that holds no sequence costs nothing.
 *
 * All pointers are HOST pointers owned by the caller.  Functions return CHUNK_ATTN_OK (0) or a negative code of
 * chunk_attn.h (INVALID_ARG for null pointers, sizes out of range or an output array that is too small) and
 * never throw or abort.  "Does not fit" is not an error: it is reported through *feasible.
 */
#ifndef CHUNK_SCHED_H_
#define CHUNK_SCHED_H_

#include <stddef.h>
#include <stdint.h>

#include "chunk_attn.h"
#include "chunk_plan.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Memory model of sections 3.2.2 / 3.2.3.  Bytes, tokens and layers; m_ms[p - 1] is the model-state footprint
 * of stage p.  layers must be a positive multiple of d_p. */
typedef struct {
  int32_t d_p, d_s, layers;
  double m_token;   /* activation bytes per token, all layers (M_token) */
  double m_logits;  /* logits bytes per token (M_logits) */
  double e;         /* bytes per activation element */
  double hidden;    /* D */
  double kv_hidden; /* D_kv */
  double capacity;  /* G */
  const double* m_ms; /* [d_p] */
} chunk_sched_mem_model;

/* One chunk as the scheduler sees it: its tokens (sum of its slices) and the paper's indicator I. */
typedef struct {
  int32_t tokens;
  int32_t is_split;
} chunk_sched_chunk;

#define CHUNK_SCHED_MAX_CHUNKS 1024 /* chunks per pipeline */
#define CHUNK_SCHED_MAX_STAGES 64

/* Activation bytes of one chunk at stage p with l_ckpt checkpointed layers (section 3.2.3). Returns a negative
 * number on invalid arguments. */
double chunk_sched_act_bytes(const chunk_sched_mem_model* model, int32_t p, int32_t tokens, int32_t is_split,
                             int32_t l_ckpt);

/* Backward position of every chunk.  unit_of_chunk[0..n): the sequence each chunk belongs to, chunks in forward
 * order, the chunks of a sequence adjacent.  f2b[0..n) receives the positions. */
int chunk_sched_f2b(const int32_t* unit_of_chunk, int32_t n, int32_t* f2b);

/* Chunk windows of stage p: windows[i * (*width) + j], i < *n_windows, lists (ascending) the chunks of the i-th
 * steady-phase window; *width = min(n, d_p - p + n_split); *n_windows = n - *width + 1.  windows must hold
 * n * n entries at most ((*n_windows) * (*width)). */
int chunk_sched_windows(int32_t d_p, int32_t p, int32_t n, int32_t n_split, const int32_t* f2b, int32_t* windows,
                        int32_t* n_windows, int32_t* width);

/*
 * Algorithm 2: checkpointing of one pipeline.  chunks[0..n) in forward order, unit_of_chunk as above, n_split the
 * number of chunks of the pipeline's longest sequence.  C[0 .. n + d_p - 1) receives the solution, *sum its sum
 * (T_ckpt = F_hat * sum), *feasible 0 if even full checkpointing does not fit (then C and *sum are not written).
 * gap >= 0 is the relative optimality gap at which the search stops: the returned sum is at most (1 + gap) times
 * the smallest one (0: the smallest one; the paper runs its solver at 0.02, section 5.5).
 * *nodes (may be null) receives the number of branch-and-bound nodes solved, negated if the search was cut short at
 * its node limit (then C is the best configuration found, not proven to be within the gap); *lower_bound (may be
 * null) a proven lower bound of the smallest sum (equal to *sum when the search ran to the end).  Every chunk must
 * free memory when a layer is checkpointed (F[k] of Algorithm 2 positive), else INVALID_ARG.
 */
int chunk_sched_solve_ckpt(const chunk_sched_mem_model* model, const chunk_sched_chunk* chunks,
                           const int32_t* unit_of_chunk, int32_t n, int32_t n_split, double gap, int32_t* C,
                           int64_t* sum, int32_t* feasible, int64_t* nodes, int64_t* lower_bound);

/*
 * Sequence grouping.  Units (sequences) u = 0 .. n_units - 1 own chunks[unit_first[u] .. unit_first[u + 1]) in
 * order.  Outputs: group_of_unit[u] (groups numbered from 0 in ascending chunk count), *n_groups, *cost =
 * sum over groups of (delta + layer_fwd_time * sum of the group's C), and per group g the forward order of its
 * chunks order[order_first[g] .. order_first[g + 1]) (indices into chunks) and its C at
 * C[c_first[g] .. c_first[g + 1]).  Capacities: order n_chunks, order_first and c_first n_units + 1,
 * C n_chunks + n_units * (d_p - 1).  *feasible is 0 if some sequence fits in no grouping.  gap as in
 * chunk_sched_solve_ckpt, applied to every pipeline tried.
 */
int chunk_sched_group(const chunk_sched_mem_model* model, const chunk_sched_chunk* chunks, const int32_t* unit_first,
                      int32_t n_units, double layer_fwd_time, double delta, double gap, int32_t* group_of_unit,
                      int32_t* n_groups, double* cost, int32_t* order, int32_t* order_first, int32_t* C, int32_t* c_first,
                      int32_t* feasible);

/*
 * 1F1B timeline of one pipeline.  t_fwd[k], t_bwd[k]: time of chunk k's forward / backward pass on one stage;
 * t_recomp (may be null): [d_p][n], added to the backward pass of chunk k at stage p (index (p - 1) * n + k);
 * mem (may be null): [d_p][n] bytes held from a chunk's forward pass to the end of its backward pass; p2p: delay
 * between a pass and the same chunk's pass on the next stage.  Outputs (each may be null): *makespan,
 * busy[d_p], peak_mem[d_p], peak_held[d_p] (largest number of chunks held).
 */
int chunk_sched_simulate(int32_t d_p, int32_t n, int32_t n_split, const int32_t* f2b, const double* t_fwd,
                         const double* t_bwd, const double* t_recomp, const double* mem, double p2p, double* makespan,
                         double* busy, double* peak_mem, int32_t* peak_held);

/*
 * The whole solve for one batch (section 3.3 with the tuning of K of section 3.3 / 3.4.1, then section 3.4): for every
 * slice number K in [k_min, k_max] (the paper tunes it in [1, d_p + 4]) the sequence processor of chunk_plan.h cuts
 * the batch into chunks, the chunks are grouped into 1F1B pipelines and given their checkpointing; the K with the
 * smallest estimated time wins (ties: the smaller K).  Estimated time of a plan:
 *     sum over chunks of T_tot(chunk) * layers / d_p  +  sum over pipelines of (delta + F_hat * sum of the pipeline's C)
 * with delta = (d_p - 1) * mean over the chunks of T_tot * layers / d_p and F_hat = fwd_fraction * mean T_tot (the
 * forward share of one layer's time for an average chunk).  The cost model gives T_tot of one layer, forward +
 * backward; `cost->n_devices` and `cost->dp` are used as given.
 * A sequence, for the scheduler, is the split chunks of one long sequence in order followed by the chunk that holds
 * its tail slice; every other chunk is a sequence of its own.
 *
 * Outputs: *best_k, *est_time; the chunks and slices of the winning plan (as chunk_plan_build; capacities max_chunks,
 * max_slices: n_seqs * (k_max + 1) each always suffices); for every chunk its pipeline (pipelines numbered from 0)
 * and its position in that pipeline's forward order; *n_pipelines; C of pipeline g at C[c_first[g] .. c_first[g + 1])
 * (capacities: pipeline_of_chunk, fwd_pos_of_chunk max_chunks; c_first max_chunks + 1; C max_chunks * d_p).
 * *feasible is 0 if no K in the range gives a plan that fits (then nothing else is written).
 */
int chunk_sched_plan_batch(const chunk_cost_model* cost, const chunk_sched_mem_model* mem, int64_t token_capacity,
                           const int32_t* lengths, int32_t n_seqs, int32_t k_min, int32_t k_max, int32_t align,
                           double fwd_fraction, double gap, int32_t* best_k, double* est_time, chunk_plan_chunk* chunks,
                           int32_t max_chunks, int32_t* n_chunks, chunk_plan_slice* slices, int32_t max_slices,
                           int32_t* n_slices, int32_t* pipeline_of_chunk, int32_t* fwd_pos_of_chunk,
                           int32_t* n_pipelines, int32_t* C, int32_t* c_first, int32_t* feasible);

#ifdef __cplusplus
}
#endif
#endif /* CHUNK_SCHED_H_ */
