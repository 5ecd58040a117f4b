/* What surrounds the decoder layers in the first and the last pipeline stage (arxiv 2504.14775, section 2.1):
 * the embedding layer (token ids -> hidden states), the projection of the final hidden states to logits over the
 * vocabulary, and the sampling strategy (greedy, top-k, nucleus) that selects the next token.
 *
 * Same conventions as gllm_stage.h: plain C, every pointer marked HOST or DEVICE, calls enqueue on `stream` and
 * return a gllm_status; there is no CPU fallback.  The caller owns every buffer passed in; the head object owns its
 * padded copy of the weights.
 */
#ifndef GLLM_HEAD_H
#define GLLM_HEAD_H

#include <stddef.h>
#include <stdint.h>

#include "gllm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Embedding layer (section 2.1): out[t][:] = table[ids[t]][:].
 *   ids    DEVICE int32 [num_tokens]
 *   table  DEVICE bf16 [vocab][hidden], row-major
 *   out    DEVICE bf16 [num_tokens][ld_out], ld_out >= hidden (e.g. the stage's hidden_in)
 * An id outside [0, vocab) gives a row of zeros (ids live on the device, so the call cannot report them).
 * hidden must be a multiple of 8. */
gllm_status gllm_op_embedding(const int32_t* ids, const void* table, void* out, int32_t num_tokens, int32_t hidden,
                              int32_t vocab, int64_t ld_out, void* stream);

typedef struct gllm_head gllm_head;

typedef struct gllm_head_config {
    int32_t hidden;    /* multiple of 64 */
    int32_t vocab;
    int32_t max_rows;  /* most rows projected by one call (sequences that receive a token in one micro-batch) */
    int32_t reserved;
    double rms_eps;
} gllm_head_config;

gllm_status gllm_head_create(const gllm_head_config* cfg /*HOST*/, gllm_head** out);
void gllm_head_destroy(gllm_head* head);
const char* gllm_head_last_error(const gllm_head* head);

/* Scratch the caller allocates (DEVICE) and binds before the first projection; freed by the caller after destroy. */
size_t gllm_head_workspace_bytes(const gllm_head* head);
gllm_status gllm_head_bind_workspace(gllm_head* head, void* workspace /*DEVICE*/, size_t bytes);

/* Copies the final norm's gain (bf16 [hidden]) and the projection matrix (bf16 [vocab][hidden], row-major) into
 * the head's own padded buffers (DEVICE inputs; the caller may free them once `stream` has passed this point). */
gllm_status gllm_head_load(gllm_head* head, const void* norm_gain, const void* w_vocab, void* stream);

/* Logits of selected rows (section 2.1: after the last layer a linear projection turns the final hidden states
 * into logits): logits[i][v] = sum_j h[j] * w_vocab[v][j] with h = bf16(x[rows[i]] * rsqrt(mean_j x^2 + eps) * gain),
 * fp32 accumulation on the matrix cores.
 *   x        DEVICE float [num_x_rows][hidden]: the fp32 residual stream the last stage returns
 *            (gllm_stage_forward's hidden_out_f32)
 *   rows     DEVICE int32 [num_rows]: which rows of x receive a next token (the last new token of each sequence
 *            whose prompt ends in this micro-batch, and every decode row); values outside [0, num_x_rows) are
 *            clamped into it
 *   logits   DEVICE float [num_rows][ld_logits], ld_logits >= gllm_head_padded_vocab(); columns vocab .. padded
 *            vocab - 1 receive 0
 * GLLM_E_CAPACITY if num_rows > max_rows, GLLM_E_STATE before load / bind_workspace. */
gllm_status gllm_head_logits(gllm_head* head, const float* x, int32_t num_x_rows, const int32_t* rows, int32_t num_rows,
                             float* logits, int64_t ld_logits, void* stream);
int32_t gllm_head_padded_vocab(const gllm_head* head);

/* gllm_head_logits for callers that cannot allocate device memory and have no workspace to bind (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels, same results bit for
 * bit, but the normalised bf16 rows between the two kernels live in a fixed array inside the library
 * (gllm_head_static_scratch_bytes() = 8 MiB per GPU, held until the process ends) instead of a bound workspace.  The
 * call allocates and frees nothing.  Limit: round_up(num_rows, 256) * hidden * 2 bytes must fit the array (512 rows
 * at hidden 8192, 1024 at 4096), else GLLM_E_CAPACITY and nothing is enqueued; max_rows and the bound workspace of
 * the head are not consulted.  GLLM_E_STATE before gllm_head_load.  All calls on one GPU share the one array, also
 * across head objects and streams: calls that may overlap in time on one GPU race on it (order them on one stream
 * or with events); nothing in it needs clearing between calls. */
gllm_status gllm_head_logits_static(gllm_head* head, const float* x, int32_t num_x_rows, const int32_t* rows,
                                    int32_t num_rows, float* logits, int64_t ld_logits, void* stream);
size_t gllm_head_static_scratch_bytes(void);

/* Sampling strategy (section 2.1: greedy, top-k, nucleus), one token per row of logits:
 *   temperature[i] <= 0: greedy, the lowest index among the largest logits.
 *   otherwise: z = logits / temperature; keep the top_k[i] largest z (top_k <= 0 or >= vocab keeps all; every z
 *   equal to the k-th largest stays); softmax over what is kept; keep the smallest set of most probable tokens
 *   whose mass reaches top_p[i] (top_p >= 1 keeps all; tokens as probable as the last one needed all stay);
 *   draw: the first token, in index order, at which the running sum of kept probabilities exceeds u[i] times their
 *   total, u[i] in [0, 1) supplied by the caller (the library draws no random numbers).
 *   logits DEVICE float [num_rows][ld_logits]; temperature, top_p, u DEVICE float [num_rows]; top_k DEVICE int32
 *   [num_rows]; out_ids DEVICE int32 [num_rows].  vocab <= 2^24. */
gllm_status gllm_op_sample(const float* logits, int64_t ld_logits, int32_t num_rows, int32_t vocab,
                           const float* temperature, const int32_t* top_k, const float* top_p, const float* u,
                           int32_t* out_ids, void* stream);

#ifdef __cplusplus
}
#endif
#endif
