/* Micro-batch scheduler of a pipeline-parallel serving runtime: Token Throttling (arxiv 2504.14775, section 3)
 * and the chunked-prefill baseline it is compared with (section 2.2).  Host code only: no call here touches a
 * GPU.  The scheduler produces exactly the batch descriptor that gllm_stage_forward() consumes (new-token count
 * and cached length per sequence, block tables), so it can drive the stage library directly.
 *
 * Every pointer is HOST memory.  Calls on one scheduler object are not thread-safe.  Functions return a
 * gllm_status (gllm_stage.h) unless they return a count; a failed call changes nothing.
 */
#ifndef GLLM_SCHED_H
#define GLLM_SCHED_H

#include <stdint.h>

#include "gllm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gllm_sched gllm_sched;

enum { GLLM_POLICY_CHUNKED_PREFILL = 0, GLLM_POLICY_TOKEN_THROTTLING = 1 };

/* Hyper-parameters (section 4.1 gives #T = 8, #MaxP = 2048, #MinP = 32, KV_thresh = 0.05; the baseline's
 * token budget is 2048).  Pages hold 16 tokens. */
typedef struct gllm_sched_params {
    int32_t policy;        /* GLLM_POLICY_* */
    int32_t iters_t;       /* #T: iterations over which the waiting prompt tokens are spread (>= 1) */
    int32_t max_p;         /* #MaxP */
    int32_t min_p;         /* #MinP (1 <= min_p <= max_p) */
    int32_t kv_thresh_bp;  /* KV_thresh in 1/10000, 0 .. 9999 */
    int32_t pp_depth;      /* #PP_depth: micro-batches in flight at most (>= 1) */
    int32_t token_budget;  /* chunked-prefill baseline: new tokens per micro-batch */
    int32_t use_wt;        /* 0 drops the waiting-tokens term of Eq. 3 (the paper's "w/o WT" ablation) */
    int32_t use_ut;        /* 0 drops the idle-rate term of Eq. 3 ("w/o UT"); the threshold still suspends prefill */
    int32_t prefix_caching; /* 1: requests added with their token ids share cached whole pages of equal prompt prefixes */
    int64_t total_pages;   /* size of the KV pool the scheduler hands out */
} gllm_sched_params;

/* Eq. 3 (section 3.1, with Eq. 1, Eq. 2 and the threshold as special cases): prefill tokens to batch now, given
 * the prompt tokens awaiting prefill (#WP) and the free pages (idle rate KV_free = free_pages / total_pages).
 * Integer arithmetic: #WP / #T rounds up, #MaxP x (KV_free - KV_thresh) / (1 - KV_thresh) rounds down; an idle
 * rate below the threshold gives 0; the result never exceeds wp or max_p.  Returns -1 for invalid arguments. */
int64_t gllm_sched_prefill_budget(const gllm_sched_params* p, int64_t wp, int64_t free_pages);

/* Eq. 4 (section 3.2): decode rows per micro-batch = ceil(#RD / #PP_depth).  Returns -1 for invalid arguments. */
int64_t gllm_sched_decode_budget(const gllm_sched_params* p, int64_t rd);

gllm_status gllm_sched_create(const gllm_sched_params* p, gllm_sched** out);
void gllm_sched_destroy(gllm_sched* s);

/* A new request enters the waiting queue (first come, first served).  prompt_len, output_len >= 1; the request
 * ends when it has produced output_len tokens (the last prefill chunk produces the first). */
gllm_status gllm_sched_add_request(gllm_sched* s, int64_t request_id, int32_t prompt_len, int32_t output_len);

/* The same with the prompt's token ids (prompt_tokens[0 .. prompt_len), copied).  With prefix_caching = 1 the
 * scheduler's page pool is the one of gllm_kv.h (section 3.4 lists prefix caching among the integrated techniques):
 * a request about to receive its first chunk -- or starting over after a preemption -- looks its prompt up and
 * skips the whole pages found (cached_len of its first chunk is then 16 x pages found; at least one token is always
 * left to compute); whole pages of this prompt are registered when the chunk that fills them has left the last
 * stage, until one registration fails; registered pages nobody holds count as free pages in Eq. 3.  Generated tokens
 * are registered only when reported (gllm_sched_complete_batch_tokens).  Shared pages are only read: a chunk's new tokens always start on a page of its own.  With
 * prefix_caching = 0, or a null prompt_tokens, this is gllm_sched_add_request(). */
gllm_status gllm_sched_add_request_tokens(gllm_sched* s, int64_t request_id, const int32_t* prompt_tokens, int32_t prompt_len,
                                          int32_t output_len);

/* Forms the next micro-batch (opening of section 3: decode and prefill tokens are budgeted separately, then merged).
 * Outputs (each with room for `capacity` rows): request ids, new-token counts, cached lengths; decode rows (one
 * new token) come first, then prefill chunks in queue order.  *num_rows = 0 and *batch_id = -1 when the pipeline
 * already holds pp_depth micro-batches or nothing can be scheduled.  Pages for the new tokens are assigned here,
 * before the micro-batch runs (caption of the prefill case study, section 3.1).  A request is in at most one
 * micro-batch in flight.  GLLM_E_CAPACITY (and no change) when capacity is below the number of requests that
 * are waiting or idle in their decode phase (each contributes at most one row). */
gllm_status gllm_sched_next_batch(gllm_sched* s, int64_t* batch_id, int64_t* request_ids, int32_t* new_tokens,
                                  int32_t* cached_len, int32_t capacity, int32_t* num_rows);

/* Block tables of the rows of a micro-batch in flight, row-major [num_rows][stride], unused entries -1: the
 * pages of each request in logical order, covering cached_len + new_tokens tokens. */
gllm_status gllm_sched_batch_block_tables(const gllm_sched* s, int64_t batch_id, int32_t* block_tables, int32_t stride);

/* The micro-batch has left the last stage: prefill progress and generated-token counts advance, requests that
 * reached output_len end and return their pages.  finished_ids (room for `capacity`) receives their ids. */
gllm_status gllm_sched_complete_batch(gllm_sched* s, int64_t batch_id, int64_t* finished_ids, int32_t capacity,
                                      int32_t* num_finished);

/* The same, reporting the tokens the micro-batch produced: row_tokens[i] is the token row i yielded (decode rows and
 * the chunk that completes a prompt yield one; the entry is ignored for other rows; negative = not reported), num_rows
 * must equal the micro-batch's row count.  With prefix caching a request's reported tokens extend its known tokens, so
 * pages filled during decoding are registered as well (a page is registered when the step that computes its last
 * position has completed): a follow-up request that repeats the conversation so far, and the request itself after a
 * preemption, find them.  A request whose tokens were not reported without gaps simply stops extending. */
gllm_status gllm_sched_complete_batch_tokens(gllm_sched* s, int64_t batch_id, const int32_t* row_tokens, int32_t num_rows,
                                             int64_t* finished_ids, int32_t capacity, int32_t* num_finished);

typedef struct gllm_sched_state {
    int64_t tokens_waiting;   /* #WP */
    int64_t decode_requests;  /* #RD */
    int64_t free_pages;       /* pages that can be handed out: never used, returned, or cached without a holder */
    int64_t batches_in_flight;
    int64_t waiting_requests;
    int64_t preemptions;      /* requests sent back for recomputation so far */
    int64_t idle_cached_pages; /* the part of free_pages that still holds a registered prefix */
    int64_t prefix_hit_tokens; /* prompt tokens skipped thanks to cached pages so far */
    int64_t evictions;        /* cached pages recycled so far */
} gllm_sched_state;
gllm_status gllm_sched_get_state(const gllm_sched* s, gllm_sched_state* out);

/* ---- a measuring device, not part of the paper: a pipeline of pp_depth equal stages fed by the scheduler ----
 * Stage time of a micro-batch, in ns: base + token_ns per new token + decode_ctx_ns per key read by a decode
 * row + prefill_pair_ns_per_1024 / 1024 per (query row, key) pair of prefill attention.  Stage s of micro-batch
 * j starts when stage s-1 of j and stage s of j-1 are done; the scheduler runs whenever stage 0 is free.
 * Requests are given by arrival time (ns, ascending), prompt and output length; ids are their indices. */
typedef struct gllm_stage_time_model {
    int64_t base_ns, token_ns, decode_ctx_ns, prefill_pair_ns_per_1024;
} gllm_stage_time_model;

typedef struct gllm_sim_result {
    int64_t end_ns, batches, tokens, busy_ns_last_stage, bubble_ppm_last_stage, mean_batch_tokens_x1000,
        var_batch_tokens_x1000, sum_ttft_ns, sum_e2e_ns, preemptions, prefix_hit_tokens;
} gllm_sim_result;

gllm_status gllm_sched_simulate(const gllm_sched_params* p, const gllm_stage_time_model* model,
                                const int64_t* arrival_ns, const int32_t* prompt_len, const int32_t* output_len,
                                int64_t num_requests, gllm_sim_result* out);

/* The same with token ids: prompt_tokens holds the prompts back to back in arrival order (sum of prompt_len
 * entries); null = no content.  Only matters with prefix_caching = 1. */
gllm_status gllm_sched_simulate_tokens(const gllm_sched_params* p, const gllm_stage_time_model* model,
                                       const int64_t* arrival_ns, const int32_t* prompt_len, const int32_t* output_len,
                                       const int32_t* prompt_tokens, int64_t num_requests, gllm_sim_result* out);

#ifdef __cplusplus
}
#endif
#endif
