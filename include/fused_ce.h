/*
 * fused_ce.h -- C ABI of the fused in-place cross-entropy of the chunk-attention library.
 *
 * The paper (section 4, "Fused In-Place Cross-Entropy") removes the peak of activation memory at the start of the
 * backward pass -- the gradient of the logits and the intermediates of the loss, at vocabularies of 128K and more
 * (section 3.2.2) -- by computing the loss and overwriting the logits with their gradient in one operator.  This is
 * that operator for one GPU's share of the tokens (the paper shards the logits along the sequence):
 *
 *   for every row i with target y_i >= 0:   lse_i  = log sum_j exp(z_ij)            (natural log, fp32 reductions)
 *                                            loss_i = lse_i - z_i[y_i]
 *                                            z_ij  <- grad_scale * (exp(z_ij - lse_i) - [j == y_i])     (bf16, RNE)
 *   for every row with y_i < 0 (ignored):   loss_i = 0,  z_ij <- 0
 *
 * One pass over HBM: every logit is read once and written once (4 bytes per element, the minimum for an in-place
 * result); a row stays in the registers of the workgroup that owns it between the two.
 *
 * logits:      DEVICE pointer, bf16 [rows][row_stride], the first `vocab` entries of a row are used; overwritten.
 * targets:     DEVICE pointer, int32 [rows]; values >= vocab are rejected by the kernel as ignored rows.
 * loss:        DEVICE pointer, fp32 [rows]; written.
 * rows >= 0, 8 <= vocab <= FUSED_CE_MAX_VOCAB, vocab % 8 == 0, row_stride >= vocab, row_stride % 8 == 0, logits
 * 16-byte aligned.  All buffers are the caller's; nothing is allocated; the call is asynchronous on `hip_stream`.
 * Returns CHUNK_ATTN_OK or a negative code of chunk_attn.h (INVALID_ARG, UNSUPPORTED for a vocabulary that is too
 * large or not a multiple of 8, HIP_ERROR); argument errors are found on the host before any launch.
 */
#ifndef FUSED_CE_H_
#define FUSED_CE_H_

#include <stddef.h>
#include <stdint.h>

#include "chunk_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

#define FUSED_CE_MAX_VOCAB 262144

int fused_ce_inplace(void* logits, const int32_t* targets, float* loss, int64_t rows, int32_t vocab, int64_t row_stride,
                     float grad_scale, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FUSED_CE_H_ */
