/*
 * flame_climber.h - C ABI of the stage above the block stacks in the paper's own model (Section 2.1).
 *
 * The paper describes the model in prose only: the user sequence is reorganised into N_b
 * sub-sequences, each processed by an independent Transformer block stack with an adaptive
 * temperature before the softmax; the candidate items are appended to the sub-sequence of every
 * block; the block outputs are joined by a "bit-wise gating fusion module"; task probabilities come
 * from the expert module of a top-level multi-layer perceptron.  The readings this library takes:
 *
 *   - block stack b is the GR forward of flame_gr.h with FLAME_GR_ATTN_SOFTMAX and its own weights,
 *     run on the contiguous history slice [floor(b L / N_b), floor((b+1) L / N_b)) of every request
 *     (flame_climber_block_range; positions restart at 0 inside a slice) plus all of the request's
 *     candidates; its output is the candidates' final residual rows H_b [sum M][d]
 *     (flame_gr_forward_hidden).  The caller runs the N_b stacks, e.g. on N_b handles and streams;
 *   - fusion, per feature ("bit-wise"): with C = [H_0 | ... | H_{N_b-1}],
 *         g_b = sigmoid(C Wg_b^T + cg_b),      F = sum_b g_b * H_b;
 *   - head: T tasks with an expert layer of width E each:
 *         p_t = sigmoid(<v_t, relu(F A_t^T + a_t)> + c_t).
 *
 * flame_climber_head computes the last two steps.  It is a plain function: no handle, no
 * allocation (the caller brings the [rows][d] workspace for F), fp32 throughout.
 * Conventions as in flame_gr.h (0 or a negative flame_gr_status).
 */
#ifndef FLAME_CLIMBER_H
#define FLAME_CLIMBER_H

#include <stdint.h>

#include "flame_gr.h"

#ifdef __cplusplus
extern "C" {
#endif

#define FLAME_CLIMBER_MAX_BLOCKS 8

typedef struct {
  int32_t n_blocks;     /* N_b: 1..FLAME_CLIMBER_MAX_BLOCKS */
  int32_t d_model;      /* d */
  int32_t n_tasks;      /* T: 1..64 */
  int32_t expert_width; /* E >= 1 */
} flame_climber_head_config;

/* Device pointers, fp32, caller-owned, row-major with the input feature contiguous. */
typedef struct {
  const float *wg;  /* [N_b][d][N_b*d]  gate of block b reads the concatenation of all blocks */
  const float *cg;  /* [N_b][d] */
  const float *a_w; /* [T][E][d] */
  const float *a_b; /* [T][E] */
  const float *v;   /* [T][E] */
  const float *c;   /* [T] */
} flame_climber_head_weights;

/* hidden   HOST array of N_b device pointers, each fp32 [n_rows][d] (one per block stack, same row order)
 * fused    device fp32 [n_rows][d]: workspace, holds F afterwards
 * probs    device fp32 [n_rows][T]
 * stream   hipStream_t or NULL.  The call enqueues two kernels and returns.
 * Errors: INVALID_ARGUMENT, HIP_ERROR (message: flame_climber_last_error). */
int flame_climber_head(const flame_climber_head_config *cfg, const flame_climber_head_weights *weights,
                       const float *const *hidden, int64_t n_rows, float *fused, float *probs, void *stream);

/* Host-only: history slice [*begin, *end) of block b out of n_blocks for a history of L items. */
int flame_climber_block_range(int32_t L, int32_t n_blocks, int32_t b, int32_t *begin, int32_t *end);

/* Message of the last failing flame_climber_* call on this thread ("" if none). */
const char *flame_climber_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FLAME_CLIMBER_H */
