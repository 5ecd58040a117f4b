/*
 * gllm_stage.h -- C ABI of the MI355X (gfx950) stage-forward library.
 *
 * The library runs ONE pipeline stage's forward pass over a hybrid micro-batch of
 * chunked-prefill and decode tokens, the computation that a pipeline-parallel serving
 * runtime with Token Throttling (arxiv 2504.14775) schedules:
 *   - a stage worker receives activations, runs its share of decoder layers, and hands
 *     activations on (paper section 3.3, description of the workers);
 *   - prefill and decode tokens are merged into a single batch (opening of section 3); a prompt may
 *     be prefilled in chunks that attend to the chunks already cached (section 2.2,
 *     "Scheduling Policies");
 *   - the KV cache is paged and every stage shares one set of page tables; pages for the
 *     new tokens are assigned before the micro-batch runs (section 3.3; caption of the
 *     prefill case-study figure in section 3.1), so this library never allocates KV pages:
 *     it only writes K/V into the pages the caller's tables name;
 *   - weights and activations are bf16 (section 4.1).
 * The layer arithmetic is the public Llama/Qwen decoder layer: pre-norm RMSNorm, QKV
 * projection (optional bias), rotate-half RoPE, grouped-query causal attention with scale
 * 1/sqrt(head_dim), output projection + residual, RMSNorm, SwiGLU MLP + residual.
 *
 * General rules
 *   - Every pointer is marked HOST or DEVICE.  Device pointers must belong to the HIP
 *     device that was current when the stage was created.
 *   - Every call returns a gllm_status (0 = success, negative = error).  After an error,
 *     gllm_last_error() gives a message.  Errors found by validation are reported before
 *     anything is enqueued, so a failed call has no side effects on device memory.
 *   - `stream` arguments are hipStream_t values passed as void* (NULL = the null stream).
 *     gllm_stage_forward only enqueues work; it does not synchronise.
 *   - A stage object is not thread safe; use one per stream.
 *   - There is no CPU fallback: without a usable HIP device create() fails.
 */
#ifndef GLLM_STAGE_H
#define GLLM_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t gllm_status;
enum {
    GLLM_OK = 0,
    GLLM_E_INVALID = -1,     /* null pointer, bad shape, new_tokens < 1, cached_len < 0, too many sequences */
    GLLM_E_CAPACITY = -2,    /* more tokens / positions / pages per sequence than the stage was created for */
    GLLM_E_BLOCK_RANGE = -3, /* a page id outside [0, num_blocks) */
    GLLM_E_BLOCK_ALIAS = -4, /* two (sequence, logical page) pairs that receive new tokens share a physical page */
    GLLM_E_STATE = -5,       /* weights, KV pool or workspace not bound yet */
    GLLM_E_HIP = -6,         /* a HIP runtime call failed */
    GLLM_E_UNSUPPORTED = -7  /* shape outside what the kernels implement */
};

typedef struct gllm_stage gllm_stage;

/* Shape and limits of a stage.  Supported: page_size == 16; head_dim in {64, 128};
 * n_q_heads a multiple of n_kv_heads with at most 16 query heads per KV head; hidden a multiple of 128;
 * n_q_heads*head_dim a multiple of 64; intermediate a multiple of 8.  Anything else gives GLLM_E_UNSUPPORTED. */
typedef struct {
    int32_t num_layers;
    int32_t hidden;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t intermediate;
    int32_t page_size;
    int32_t has_qkv_bias;
    int32_t max_tokens;          /* most new tokens in one batch */
    int32_t max_seqs;            /* most sequences in one batch */
    int32_t max_blocks_per_seq;  /* most pages one sequence may own */
    int32_t max_position;        /* largest cached_len + new_tokens of any sequence */
    double rms_eps;
    double rope_theta;
} gllm_stage_config;

/* One layer's parameters.  DEVICE pointers, bf16, row-major [out_features][in_features]:
 *   wq [n_q*d][hidden]  wk, wv [n_kv*d][hidden]  wo [hidden][n_q*d]
 *   wgate, wup [intermediate][hidden]  wdown [hidden][intermediate]
 *   norm1, norm2 [hidden] (RMSNorm gains before attention / before the MLP)
 *   bq [n_q*d], bk, bv [n_kv*d]: required iff has_qkv_bias, else ignored (may be NULL). */
typedef struct {
    const void *wq, *wk, *wv, *wo, *wgate, *wup, *wdown, *norm1, *norm2, *bq, *bk, *bv;
} gllm_layer_weights;

/* A micro-batch (HOST memory, read completely before gllm_stage_forward returns).
 * Sequence s contributes new_tokens[s] >= 1 rows at positions cached_len[s] ..
 * cached_len[s]+new_tokens[s]-1; row i of it attends to positions 0 .. cached_len[s]+i.
 * A decode step is new_tokens == 1.  Rows are packed in sequence order: the first row of
 * sequence s is row sum_{r<s} new_tokens[r].  block_tables[s*block_table_stride + b] is
 * the physical page holding positions 16b .. 16b+15 of sequence s; entries are read for
 * b < ceil((cached_len+new_tokens)/16) only. */
typedef struct {
    int32_t num_seqs;
    int32_t block_table_stride;
    const int32_t* new_tokens;
    const int32_t* cached_len;
    const int32_t* block_tables;
} gllm_batch;

/* Creates a stage on the current HIP device: allocates the RoPE table and the metadata staging.  The
 * library-owned copies of a layer's weights are allocated when gllm_stage_load_layer first fills them. */
gllm_status gllm_stage_create(const gllm_stage_config* cfg /*HOST*/, gllm_stage** out /*HOST*/);
void gllm_stage_destroy(gllm_stage* stage);

/* Message of the last failed call on this stage (or of the last failed create when stage
 * is NULL).  The string is owned by the library and valid until the next call. */
const char* gllm_last_error(const gllm_stage* stage);
const char* gllm_status_name(gllm_status s);

/* Activation workspace: the caller allocates workspace_bytes() of device memory (256-byte
 * aligned) and binds it; the library never frees it.  Contents need not survive between
 * forward calls. */
size_t gllm_stage_workspace_bytes(const gllm_stage* stage);
gllm_status gllm_stage_bind_workspace(gllm_stage* stage, void* workspace /*DEVICE*/, size_t bytes);

/* Copies and repacks one layer's parameters into library-owned device buffers (QKV rows
 * concatenated, gate/up rows interleaved in groups of 32, rows and columns padded to tile
 * multiples).  The copy is enqueued on `stream`; the caller's tensors may be released once
 * the stream has passed this point. */
gllm_status gllm_stage_load_layer(gllm_stage* stage, int32_t layer, const gllm_layer_weights* w /*HOST struct of DEVICE ptrs*/,
                                  void* stream);

/* Binds the caller-owned paged KV pool (DEVICE, bf16), page_size = 16 slots per page:
 *   k_pool [num_layers][num_blocks][n_kv][head_dim/8][16][8]
 *   v_pool [num_layers][num_blocks][n_kv][head_dim][16]
 * i.e. K keeps each 8-element group of a head vector contiguous per slot, V keeps the 16
 * slots of one head-dimension contiguous.  The forward pass writes the K/V of the new
 * tokens (K after RoPE), rounded to bf16 (nearest even), to
 *   page = block_tables[s][pos / 16], slot = pos % 16
 * of every layer, and reads all earlier positions from the pool. */
gllm_status gllm_stage_bind_kv_pool(gllm_stage* stage, void* k_pool /*DEVICE*/, void* v_pool /*DEVICE*/,
                                    int64_t num_blocks);

/* Several stage objects over one set of weights: `stage` gives up its own (repacked) weight buffers and uses those
 * of `owner` from now on -- for running micro-batches on several streams, one stage object per stream (each has its
 * own workspace, metadata buffers and internal streams; calls on one object are still not thread-safe), without a
 * copy of the weights per stream.  Both must have been created with the same layer shapes; every layer of `owner`
 * must be loaded; `owner` must stay alive, and its weights unchanged, as long as `stage` is used.  Synchronises the
 * device.  GLLM_E_INVALID for differing shapes or an owner that borrows itself, GLLM_E_STATE for an owner with
 * unloaded layers; afterwards gllm_stage_load_layer on `stage` gives GLLM_E_STATE. */
gllm_status gllm_stage_share_weights(gllm_stage* stage, const gllm_stage* owner);

/* Debug option: when nonzero, forward() also rejects batches in which two different
 * (sequence, logical page) pairs that receive new tokens name the same physical page. */
gllm_status gllm_stage_set_alias_check(gllm_stage* stage, int32_t on);

/* Tuning knobs (defaults are chosen for MI355X).  Known names:
 *   "decode_min_workgroups" (default 2048): a partition size (256 .. 16384 keys, a power of two) is chosen as
 *   the largest for which partitions x KV heads reaches this many workgroups; a decode row with more keys than
 *   that is cut into equal shares of whole 32-key blocks, and the longest shares are launched first.
 *   "overlap_attention" (default 1): prefill attention of a layer runs on an internal side stream next to
 *   decode attention (forked from and joined back into the caller's stream with events); 0 keeps every
 *   kernel on the caller's stream.  Per-kernel profiling always uses the single-stream order.  (The runtime maps
 *   streams onto a few hardware queues; when the side stream happens to share the caller's queue the two kernels
 *   simply run one after the other.  Callers that run several stages on several streams of their own may do better
 *   with 0: every further stream competes for those queues.)
 *   "gemm_row_mixed" (default 1; a property of this stage only): the stage's GEMM planner may cover a last band of at
 *   most 128 token rows with 64- or 128-row tiles instead of a whole band of 256 (tile 8 of gllm_op_gemm_bf16).
 *   "layer_begin" (default 0), "layer_end" (default num_layers): forward() runs only layers layer_begin .. layer_end-1
 *   of the stage, each with its own weights and its own slice of the KV pool: hidden_in is taken as the residual
 *   stream in front of layer_begin, hidden_out is the stream behind layer_end-1.  For testing one layer at its real
 *   shape with the activations the layers before it produce, and for timing a part of a stage.  layer_begin must lie
 *   in [0, num_layers), layer_end in [1, num_layers] (else GLLM_E_INVALID, nothing changes); the range never becomes
 *   empty: setting one end at or past the other moves the other so that exactly one layer is left.
 * Unknown names give GLLM_E_INVALID. */
gllm_status gllm_stage_set_option(gllm_stage* stage, const char* name /*HOST*/, int64_t value);

/* Runs all layers of the stage on the batch.
 *   hidden_in       DEVICE bf16 [T][hidden]   (T = sum of new_tokens)
 *   hidden_out      DEVICE bf16 [T][hidden]   residual stream after the last layer, RNE to bf16
 *   hidden_out_f32  DEVICE float [T][hidden] or NULL: the fp32 residual stream before that rounding
 * The residual stream is kept in fp32 across the layers; GEMM and attention operands are bf16
 * with fp32 accumulation.  Enqueues on `stream` and returns. */
gllm_status gllm_stage_forward(gllm_stage* stage, const gllm_batch* batch /*HOST*/, const void* hidden_in,
                               void* hidden_out, float* hidden_out_f32, void* stream);

/* Per-kernel timing.  With profiling on, forward() brackets every kernel with HIP events on
 * the caller's stream; gllm_stage_read_profile() synchronises those events and adds their
 * durations to per-class totals.  Classes are listed by gllm_profile_class_name(i) for
 * i in [0, gllm_profile_num_classes()).  ms and launches are HOST arrays of that length. */
gllm_status gllm_stage_set_profiling(gllm_stage* stage, int32_t on);
gllm_status gllm_stage_read_profile(gllm_stage* stage, double* ms /*HOST*/, int64_t* launches /*HOST*/, int32_t reset);
int32_t gllm_profile_num_classes(void);
const char* gllm_profile_class_name(int32_t i);

/* ---- single operations on DEVICE buffers (the kernels the stage is built from), exported so
 * that each can be tested and timed on its own.  All enqueue on `stream` and return. ---- */

/* The weight operand of the GEMMs below is "tiled": blocks of 64 output rows x 64 k values, each block contiguous
 * (64 rows of 128 bytes), blocks ordered [row block][k block]; element (r, c) of an [n][k] matrix sits at element index
 *   ((r/64)*(k/64) + c/64)*4096 + (r%64)*64 + c%64.
 * (A k-step of a workgroup tile then reads whole 8 KiB pieces, not one 128-byte piece per output row: with few token
 * rows the weights stream from HBM once per call, and HBM serves long pieces better.)  gllm_op_pack_weight writes this
 * layout from a row-major bf16 matrix w [n][ldw] (DEVICE, 16-byte aligned, ldw >= k and a multiple of 8) into
 * out (DEVICE, n*k elements, must not overlap w); n and k multiples of 64, else GLLM_E_UNSUPPORTED.  The stage and the
 * head repack the row-major weights they are given in the same way when these are loaded. */
gllm_status gllm_op_pack_weight(const void* w, int64_t ldw, int32_t n, int32_t k, void* out, void* stream);

/* out[m][n] (op)= sum_k a[m][k] * w[n][k];  a: bf16 [m_rows][lda] with lda >= k, w: bf16, n rows, tiled as above with
 * k extent ldw (a multiple of 64, >= k: the product may use a leading part of the k range).
 * Requirements: k a multiple of 64 and n a multiple of 128 (the stage pads its operands);
 * a must be readable for round_up(m,256) rows.  mode: 0 store fp32 to out[m][ldc];
 * 1 add into fp32 out[m][ldc]; 2 SwiGLU: columns come in groups of 64 = 32 gate + 32 up
 * outputs, out is bf16 [m][ldc] with n/2 columns, out = silu(gate) * up.
 * tile: -1 lets the library choose the workgroup tile; 0 = 128x128, 1 = 256x128, 2 = 256x256
 * (4 wavefronts), 3 = 256x256 (8 wavefronts), 4 = 256x256 tiles for whole rounds of the compute units plus
 * 256x128 tiles for the remainder (only for shapes with such a remainder), 5 = 256x192 (n a multiple of 192,
 * not for SwiGLU), 6 = 128x128 with four LDS stages instead of two (for few rows, where the weights stream
 * from HBM), 7 = 64x128 with three LDS stages (picked up to 64 rows: two workgroups per compute unit keep more
 * of the weight stream in flight), 8 = 256x256 tiles for the whole bands of 256 rows plus 64x256 or 128x256 tiles
 * for a last band of at most 128 rows (only for m > 256 with 0 < m mod 256 <= 128 and n a multiple of 256), 9 = 288x192
 * (six wavefronts; only for 256 < m <= 288, n a multiple of 192, not for SwiGLU: all rows in one band, so the weights
 * are read once), 10 / 11 / 12 = tiles 3 / 4 / 8 with a third LDS stage for the weight tile (all 160 KiB of LDS: the
 * weight loads get two k-steps to land; picked for long k and for few rows); a forced tile that does not fit the
 * shape gives GLLM_E_UNSUPPORTED. */
gllm_status gllm_op_gemm_bf16(const void* a, int64_t lda, const void* w, int64_t ldw, void* out, int64_t ldc,
                              int32_t m, int32_t n, int32_t k, int32_t mode, int32_t tile, void* stream);

/* Split-K form of the store mode: split s (0 <= s < splits) multiplies the k range [s*k/splits, (s+1)*k/splits)
 * and stores its partial product to out + s*plane_stride floats; the caller sums the planes.  k/64 must be a
 * multiple of splits. */
gllm_status gllm_op_gemm_bf16_splitk(const void* a, int64_t lda, const void* w, int64_t ldw, float* out, int64_t ldc,
                                     int32_t m, int32_t n, int32_t k, int32_t tile, int32_t splits, int64_t plane_stride,
                                     void* stream);

/* Host only (no device call): the tile id and split-K factor the library's cost model picks for a problem
 * when gllm_op_gemm_bf16 is called with tile = -1 (splits stays 1 unless mode is 0; at most max_splits).
 * tile, splits: HOST out.  The stage plans its QKV, O and down projections with max_splits = 8. */
gllm_status gllm_op_gemm_plan(int32_t m, int32_t n, int32_t k, int32_t mode, int32_t max_splits, int32_t* tile,
                              int32_t* splits);

/* h[t][j] = bf16(x[t][j] * rsqrt(mean_j x^2 + eps) * gamma[j]); x fp32 [rows][hidden]. */
gllm_status gllm_op_rmsnorm(const float* x, const void* gamma_bf16, void* h_bf16, int32_t rows, int32_t hidden,
                            double eps, void* stream);

/* Ceiling probes, used by the benchmark to report what this GPU sustains next to the published peaks
 * (the paper gives no kernel-level figure; these are measurement aids, not part of the stage).
 * peak_mfma: `workgroups` workgroups of 4 wavefronts, each wavefront issuing iters*16 independent
 * 32x32x16 bf16 MFMAs (2*32*32*16 flop each) with no memory traffic.  peak_read: reads `bytes` of DEVICE
 * memory once with 16-byte loads.  sink: DEVICE, at least 4 KiB; peak_mfma takes its operand bits from
 * it (fill it with bf16 data of the kind the GEMMs see); it is never written in practice. */
gllm_status gllm_op_peak_mfma(void* sink, int32_t workgroups, int32_t iters, void* stream);
gllm_status gllm_op_peak_read(const void* src, int64_t bytes, void* sink, int32_t workgroups, void* stream);
/* The same read with the non-temporal hint on every load (what the decode attention kernel uses for its K/V stream). */
gllm_status gllm_op_peak_read_nt(const void* src, int64_t bytes, void* sink, int32_t workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GLLM_STAGE_H */
