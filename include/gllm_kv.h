/* KV page pool with prefix caching for a paged KV cache whose page tables all pipeline stages share.  Host code
 * only: no call here touches a GPU; page ids are the block ids that gllm_stage_forward() takes in its block tables.
 *
 * The paper (arxiv 2504.14775) assigns KV pages before a micro-batch runs (section 3.1, caption of the prefill case
 * study), has the driver worker manage the KV cache for every stage (section 3.3), feeds the idle rate of that
 * cache into Eq. 2 / Eq. 3, and names PagedAttention and prefix caching as integrated techniques (section 3.4; the
 * reuse of KV across requests is switched off in its measurements, section 4.1).  It gives no algorithm, so the
 * rules are this library's:
 *   - a page holds 16 tokens; a page completely filled with prompt tokens can be registered under the key
 *     (page holding the previous 16 tokens | none, its 16 token ids): a radix tree over whole pages, exact
 *     comparison, no hashing of content into identities;
 *   - every page counts its holders; a registered page without holders keeps its content, waits in an eviction
 *     queue and counts as available;
 *   - a new page comes from the free stack (last in first out; ids 0, 1, 2, ... at the start), and from the front
 *     of the eviction queue once the stack is empty;
 *   - releasing a block table puts unregistered pages that lost their last holder on the free stack in table
 *     order, registered ones at the back of the eviction queue, last entry first: a page leaves the tree before
 *     the page it extends.  A holder must release a page together with the pages that extend it (release whole
 *     block tables), which is what keeps that order valid.
 *
 * Every pointer is HOST memory.  Calls on one pool are not thread-safe.  A failed call changes nothing.
 */
#ifndef GLLM_KV_H
#define GLLM_KV_H

#include <stdint.h>

#include "gllm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gllm_kv gllm_kv;

enum { GLLM_KV_PAGE_TOKENS = 16, GLLM_KV_ROOT = -1 };

/* total_pages in [1, 2^31).  GLLM_E_INVALID otherwise. */
gllm_status gllm_kv_create(int64_t total_pages, gllm_kv** out);
void gllm_kv_destroy(gllm_kv* kv);

/* Pages gllm_kv_alloc() can still hand out (free + registered without holders); -1 for a null pool.  Divided by
 * the pool size this is the idle rate KV_free of Eq. 2. */
int64_t gllm_kv_available(const gllm_kv* kv);

/* n new pages, each with one holder (the caller), written to pages[0 .. n).  GLLM_E_CAPACITY when fewer than n
 * are available. */
gllm_status gllm_kv_alloc(gllm_kv* kv, int32_t n, int32_t* pages);

/* Looks up the whole pages of the prompt tokens[0 .. num_tokens) from its start, at most max_pages of them, stops
 * at the first page that is not registered; the pages found are written to pages[0 .. *num_found) (room for
 * max_pages) and each gets one more holder: they are the first *num_found entries of the caller's block table and
 * 16 * *num_found tokens need not be computed.  A caller that needs the last token's output bounds the walk with
 * max_pages = (num_tokens - 1) / 16. */
gllm_status gllm_kv_match(gllm_kv* kv, const int32_t* tokens, int64_t num_tokens, int32_t max_pages, int32_t* pages,
                          int32_t* num_found);

/* Registers `page` (held by the caller, not registered, its 16 slots written with the KV of tokens16) behind
 * parent_page (registered and held by the caller; GLLM_KV_ROOT for the first page of a prompt).  *registered = 0 and
 * no change when that key is present already (somebody else computed the same prefix): the page stays private.
 * GLLM_E_INVALID for a page or parent that does not meet the conditions above. */
gllm_status gllm_kv_register(gllm_kv* kv, int32_t parent_page, const int32_t* tokens16, int32_t page, int32_t* registered);

/* One holder less on each of pages[0 .. n) (a block table: no page twice, every page held).  GLLM_E_INVALID and no
 * change otherwise. */
gllm_status gllm_kv_release(gllm_kv* kv, const int32_t* pages, int32_t n);

typedef struct gllm_kv_state {
    int64_t total_pages, free_pages, idle_cached_pages, registered_pages, evictions;
} gllm_kv_state;
gllm_status gllm_kv_get_state(const gllm_kv* kv, gllm_kv_state* out);

/* Holders, registration flag and number of registered pages that extend `page` directly (diagnostics). */
gllm_status gllm_kv_page_info(const gllm_kv* kv, int32_t page, int32_t* holders, int32_t* is_registered, int32_t* children);

#ifdef __cplusplus
}
#endif
#endif
