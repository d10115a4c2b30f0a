/*
 * chunk_attn.h -- C ABI of the MI355X (gfx950) chunk-attention library.
 *
 * Chunk attention is the attention step of one pipeline stage over one "chunk" of the
 * paper's Dynamic Pipeline Parallelism (section 3.1, "Definition of Chunk").  A chunk
 * {C, S} is a set of slice lengths S and a context length C for its first slice:
 *
 *   batched (packed) chunk : several whole short sequences, C = 0;
 *   split chunk            : one slice of a long sequence; its queries also attend to the
 *                            keys/values of all earlier slices (the context, length C);
 *   hybrid chunk           : a tail slice with context C packed with whole short sequences.
 *
 * Here a chunk is a table of segments.  Segment t has q_len = s query rows and
 * kv_len = C + s key/value rows.  Query i of the segment (row q_start + i) sits at position
 * C + i of its sequence and attends to key/value rows kv_start + j for j = 0 .. C + i
 * (causal mask aligned to the end of the key range; section 2.1: a query accesses only the
 * keys and values of preceding tokens) and to nothing outside its own segment (section 2.2,
 * sequence packing: packed sequences do not attend to each other).  The result is exact
 * softmax attention, O = softmax(scale * Q K^T + mask) V, and its exact gradients; key and
 * value gradients of context rows are produced too, because the gradient of a token's key
 * and value depends on every later token (section 2.1; section 3.2.2 on the gradients of
 * keys and values of split sequences).
 *
 * Tensors (all DEVICE pointers, contiguous, bf16 unless noted; the caller owns them):
 *   q, o, d_o, dq : [total_q ][num_q_heads ][head_dim]
 *   k, v, dk, dv  : [total_kv][num_kv_heads][head_dim]
 *   lse           : [num_q_heads][total_q] float32, natural-log sum of exp of the scaled scores
 * Query head h uses key/value head h / (num_q_heads / num_kv_heads).
 *
 * All calls are asynchronous: they enqueue work on `stream` (a hipStream_t passed as
 * void*; NULL is the default stream) and return.  The segment table is a HOST pointer and
 * is only read during the call.  The library allocates no device memory: scratch space is
 * the caller's `workspace` (device memory, 256-byte aligned, at least the size reported by
 * chunk_attn_workspace_bytes; its contents need not survive between calls, and calls that
 * may run at the same time, on different streams, need a workspace each).  Every tensor pointer must be 16-byte aligned (lse: 4-byte),
 * else CHUNK_ATTN_INVALID_ARG.  Functions return CHUNK_ATTN_OK (0) or a negative code and
 * never throw or abort; argument errors are detected on the host before anything is
 * launched.
 *
 * The only state the library keeps between calls is a pool of pinned host buffers through
 * which the tile schedules of chunk_attn_fwd / chunk_attn_bwd are uploaded (it grows with
 * the schedules in flight, to 256 MB at most).  The library owns it; chunk_attn_shutdown
 * releases it.
 */
#ifndef CHUNK_ATTN_H_
#define CHUNK_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CHUNK_ATTN_OK = 0,
  CHUNK_ATTN_INVALID_ARG = -1,         /* null pointer, non-positive dimension, bad scale */
  CHUNK_ATTN_UNSUPPORTED = -2,         /* head_dim not 64, 96, 128 or 256, or num_q_heads % num_kv_heads != 0 */
  CHUNK_ATTN_BAD_SEGMENT = -3,         /* see chunk_attn_desc.segments */
  CHUNK_ATTN_WORKSPACE_TOO_SMALL = -4, /* workspace_bytes below chunk_attn_workspace_bytes */
  CHUNK_ATTN_HIP_ERROR = -5,           /* a HIP call or kernel launch failed */
  CHUNK_ATTN_TOO_LARGE = -6            /* chunk_attn_fwd_static: more than its fixed scratch buffer holds */
};

/* One segment, in rows.  Context length C = kv_len - q_len >= 0. */
typedef struct {
  int32_t q_start, q_len, kv_start, kv_len;
} chunk_attn_seg;

typedef struct {
  int32_t num_q_heads;  /* Hq > 0 */
  int32_t num_kv_heads; /* Hkv > 0, divides Hq */
  int32_t head_dim;     /* 64, 96, 128 or 256 (96 runs as 128 on zero-padded copies in the workspace) */
  int32_t total_q;      /* rows of q / o / d_o / dq */
  int32_t total_kv;     /* rows of k / v / dk / dv */
  int32_t num_segments; /* >= 1 */
  /* HOST array, borrowed for the call.  Requirements (else CHUNK_ATTN_BAD_SEGMENT):
   * q_len >= 1, kv_len >= q_len, ranges inside [0,total_q) resp. [0,total_kv); query
   * ranges in increasing order, back to back, covering [0,total_q) exactly; key ranges
   * in increasing order without overlap (gaps are allowed). */
  const chunk_attn_seg* segments;
  float softmax_scale; /* finite, > 0; normally 1/sqrt(head_dim) */
} chunk_attn_desc;

/*
 * Scratch sizes (bytes) for a descriptor: *fwd_bytes for chunk_attn_fwd, *bwd_bytes for
 * chunk_attn_bwd (the tile schedules, the row sums D_i = <dO_i, O_i>, and transposed
 * tile images of the operands; for head_dim 96 also zero-padded copies of the tensors, 128
 * wide).  Either output pointer may be NULL.  Validates the descriptor.
 */
int chunk_attn_workspace_bytes(const chunk_attn_desc* desc, size_t* fwd_bytes, size_t* bwd_bytes);

/*
 * Validates a descriptor on the host without touching the GPU (same checks every entry
 * point performs first).
 */
int chunk_attn_validate(const chunk_attn_desc* desc);

/*
 * Forward (paper section 3.1 mask; exact softmax attention, section 3.2.2 notes that
 * no O(S^2) score matrix is materialised).  Writes o (bf16) and lse (float32) for every
 * query row.  q, k, v are read only.
 */
int chunk_attn_fwd(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, void* o, float* lse,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * chunk_attn_fwd for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and
 * results as chunk_attn_fwd; the call allocates nothing, on the host side of the runtime or the
 * device (no hipMalloc / hipFree / pinned buffers: the schedule is built by a small kernel from the
 * segment table, which travels as a kernel argument).  Its scratch memory is a fixed array of
 * 16 MiB inside the library, one copy per GPU, held until the process ends.
 * Limits: at most 64 segments, and a forward scratch need (chunk_attn_workspace_bytes' *fwd_bytes:
 * the schedule plus one transposed copy of V) of at most 16 MiB, else CHUNK_ATTN_TOO_LARGE and
 * nothing is launched.  All calls on one GPU share that GPU's array: calls that may overlap on
 * one GPU (different streams, different threads) race and must be serialised by the caller.
 */
int chunk_attn_fwd_static(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, void* o, float* lse,
                          void* stream);

/*
 * Backward for the loss L = sum(o .* d_o): dq for every query row; dk, dv for every
 * key/value row including context rows (section 2.1: gradients of a token's key and value
 * come from the tokens after it).  o and lse must be the outputs of chunk_attn_fwd on the
 * same inputs.
 *
 * accumulate_dkv == 0: dk/dv rows inside some segment's key range are overwritten, all
 *   other rows are set to zero.
 * accumulate_dkv != 0: rows inside a key range get  dk[row] = bf16(float(dk[row]) + sum)
 *   (one rounding per call), other rows are left untouched.  This is how the slices of a
 *   split sequence, run in reverse order, add up the gradients of shared context rows
 *   (section 3.2.2: the key/value gradients of all slices stay alive until each slice's
 *   own backward has run).
 */
int chunk_attn_bwd(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, const void* o,
                   const void* d_o, const float* lse, void* dq, void* dk, void* dv, int accumulate_dkv,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * chunk_attn_bwd with the key/value gradients kept in float32: dk, dv are DEVICE arrays of
 * [total_kv, Hkv, head_dim] floats (16-byte aligned), everything else as in chunk_attn_bwd.  The rows of a
 * key range receive the call's fp32 sums unrounded (accumulate_dkv == 0) or have them added in fp32
 * (accumulate_dkv != 0), so the gradients of context rows that the slices of a split sequence build up over
 * several calls (section 3.2.2) are rounded to bf16 once, by the caller, instead of once per slice.  The paper
 * sizes these buffers at e bytes per element; this variant trades twice the memory for that accuracy.
 * Same workspace as chunk_attn_bwd.
 */
int chunk_attn_bwd_f32kv(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, const void* o,
                         const void* d_o, const float* lse, void* dq, float* dk, float* dv, int accumulate_dkv,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Number of unmasked (query, key) pairs per query head, sum_t (s C + s (s + 1) / 2): the
 * quantity behind the quadratic term of the paper's computation-time model (Eq. 1).
 * Forward costs 4 * head_dim flops per pair per query head, backward 10 * head_dim.
 * Returns a negative error code for an invalid descriptor.
 */
int64_t chunk_attn_pair_count(const chunk_attn_desc* desc);

/*
 * Measurement hook (not part of the method): arms one pair of hipEvent_t (passed as void*) for the
 * calling thread.  The next chunk_attn_fwd or chunk_attn_bwd call on this thread records `start`
 * immediately before and `stop` immediately after its main kernel (the forward kernel, resp. the
 * dK/dV/dQ kernel of the backward) on that call's stream, then disarms.  Pass NULLs to disarm.
 * The caller owns the events.  Always returns CHUNK_ATTN_OK.
 */
int chunk_attn_profile_events(void* start_event, void* stop_event);

/*
 * Releases the pinned host buffers the library has allocated for schedule uploads (waiting for the
 * uploads that still read them).  Optional: call it when no more work will be submitted, or to
 * return the memory between phases; later calls simply allocate again.  Must not run concurrently
 * with other calls of this library.  Returns CHUNK_ATTN_OK or CHUNK_ATTN_HIP_ERROR.
 */
int chunk_attn_shutdown(void);

/*
 * Test hook (not part of the method): the head_dim 128 forward keeps the softmax reference
 * maximum of a row fixed after its first key tile and recomputes, in a second pass with a moving
 * maximum, the rows whose later scores exceed it by more than 2^log2_growth (default 60; any
 * reference gives the same softmax).  A very negative value sends every row through the second
 * pass.  Process-wide.  Always returns CHUNK_ATTN_OK.
 */
int chunk_attn_test_set_fwd_rescale_limit(float log2_growth);

/*
 * Measurement hook (not part of the method): the bf16 matrix throughput this GPU sustains when a kernel issues nothing
 * but independent v_mfma_f32_32x32x16_bf16 instructions on random operands, one workgroup of four waves per CU, for
 * about `milliseconds` (1 .. 10000) of GPU time; the rate of the last launch goes to *tflops.  Under sustained matrix
 * load the chip runs below its 2.4 GHz peak clock, so this -- not the published 2516.6 TFLOP/s -- is the ceiling any
 * kernel sees.  `scratch`: DEVICE memory, 256-byte aligned, at least 1052672 bytes (else
 * CHUNK_ATTN_WORKSPACE_TOO_SMALL).  Synchronises `stream`.
 */
int chunk_attn_measure_mfma_rate(int milliseconds, void* scratch, size_t scratch_bytes, void* stream, double* tflops);

/*
 * The same measurement with `workgroups` workgroups (1 .. number of CUs) instead of one per CU, i.e. with only part
 * of the chip busy: the rate per busy CU rises as fewer are busy, which shows that the sustained matrix rate of the
 * whole chip is set by its power budget and not by a fixed clock.  CHUNK_ATTN_INVALID_ARG for a count out of range.
 */
int chunk_attn_measure_mfma_rate_on(int milliseconds, int workgroups, void* scratch, size_t scratch_bytes, void* stream,
                                    double* tflops);

/*
 * Measurement hook (not part of the method): the clock the three pipelined kernels (forward, dQ, dK/dV; head_dim 64,
 * 96 and 128) actually run at.  `device_buffer`: DEVICE memory, 8-byte aligned, at least CHUNK_ATTN_CLOCK_LOG_BYTES
 * (else CHUNK_ATTN_WORKSPACE_TOO_SMALL; CHUNK_ATTN_INVALID_ARG if misaligned), owned by the caller and kept alive until
 * the hook is switched off with a null pointer.  While it is set, every workgroup of those kernels writes four 64-bit
 * values when it starts and when it has run out of work: section k of the buffer (k = 0 forward, 1 dQ, 2 dK/dV; 4096
 * values each) holds, for workgroup b < 1024, at [4 b .. 4 b + 3] = {constant 100 MHz counter at the start, at the
 * end, shader-clock counter at the start, at the end}.  The ratio of the differences, times 100 MHz, is the clock.
 * Each launch overwrites its kernel's section; clear the buffer before a launch to tell entries apart.  Process-wide;
 * the kernels' results do not depend on it.
 */
#define CHUNK_ATTN_CLOCK_LOG_BYTES (3 * 4096 * 8)
int chunk_attn_measure_set_clock_log(void* device_buffer, size_t bytes);

/*
 * Test and measurement hook: which backward chunk_attn_bwd / chunk_attn_bwd_f32kv run for head_dim 128.
 * 0: the library's choice; 1: two kernels (dQ query-stationary, dK/dV key-stationary, P recomputed in both);
 * 2: one pass (the key-stationary kernel also forms dQ and adds it into float32 tiles in the workspace in a fixed
 * order).  Same results up to the order of float32 additions in dQ; both are bit-reproducible.  Process-wide; the
 * workspace size does not depend on it.  Returns CHUNK_ATTN_INVALID_ARG for any other value.
 */
int chunk_attn_test_set_bwd_mode(int mode);

/*
 * Test hook: byte offset, inside the backward workspace of `desc`, of the status word (uint32) of the one-pass
 * backward.  After a head_dim 128 backward in mode 2 has completed it is 0 unless something went wrong: bit 0 = a wave
 * gave up waiting for the workgroup before it in the dQ order (bounded wait; dQ is then wrong), bit 1 = an XCD
 * received more workgroups than the plan has for it (the grid was not dealt to the XCDs round robin; work is then
 * left undone).
 */
int chunk_attn_test_bwd_status_offset(const chunk_attn_desc* desc, size_t* offset);

/* Static description of an error code; for CHUNK_ATTN_HIP_ERROR includes the last HIP error text. */
const char* chunk_attn_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CHUNK_ATTN_H_ */
