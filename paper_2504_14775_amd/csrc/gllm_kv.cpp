// C ABI of the KV page pool (include/gllm_kv.h): argument checks around gllm::PagePool.
#include "../../include/gllm_kv.h"

#include <algorithm>
#include <new>
#include <vector>

#include "page_pool.h"

struct gllm_kv {
    gllm::PagePool pool;
    explicit gllm_kv(int64_t n) : pool(n) {}
};

namespace {
inline bool page_ok(const gllm_kv* kv, int64_t page) { return page >= 0 && page < kv->pool.total(); }
}  // namespace

extern "C" {

gllm_status gllm_kv_create(int64_t total_pages, gllm_kv** out) {
    if (!out) return GLLM_E_INVALID;
    *out = nullptr;
    if (total_pages < 1 || total_pages >= (int64_t)1 << 31) return GLLM_E_INVALID;
    gllm_kv* kv = new (std::nothrow) gllm_kv(total_pages);
    if (!kv) return GLLM_E_CAPACITY;
    *out = kv;
    return GLLM_OK;
}

void gllm_kv_destroy(gllm_kv* kv) { delete kv; }

int64_t gllm_kv_available(const gllm_kv* kv) { return kv ? kv->pool.available() : -1; }

gllm_status gllm_kv_alloc(gllm_kv* kv, int32_t n, int32_t* pages) {
    if (!kv || n < 0 || (n > 0 && !pages)) return GLLM_E_INVALID;
    if (n > kv->pool.available()) return GLLM_E_CAPACITY;
    for (int32_t i = 0; i < n; ++i) pages[i] = kv->pool.alloc();
    return GLLM_OK;
}

gllm_status gllm_kv_match(gllm_kv* kv, const int32_t* tokens, int64_t num_tokens, int32_t max_pages, int32_t* pages,
                          int32_t* num_found) {
    if (!kv || !num_found || num_tokens < 0 || max_pages < 0 || (num_tokens > 0 && !tokens) || (max_pages > 0 && !pages))
        return GLLM_E_INVALID;
    std::vector<int32_t> found;
    kv->pool.match(tokens, num_tokens, max_pages, found);
    std::copy(found.begin(), found.end(), pages);
    *num_found = (int32_t)found.size();
    return GLLM_OK;
}

gllm_status gllm_kv_register(gllm_kv* kv, int32_t parent_page, const int32_t* tokens16, int32_t page, int32_t* registered) {
    if (!kv || !tokens16 || !registered || !page_ok(kv, page)) return GLLM_E_INVALID;
    if (kv->pool.holders(page) < 1 || kv->pool.is_registered(page)) return GLLM_E_INVALID;
    if (parent_page != GLLM_KV_ROOT) {
        if (!page_ok(kv, parent_page) || parent_page == page) return GLLM_E_INVALID;
        if (kv->pool.holders(parent_page) < 1 || !kv->pool.is_registered(parent_page)) return GLLM_E_INVALID;
    }
    *registered = kv->pool.enter(parent_page, tokens16, page) ? 1 : 0;
    return GLLM_OK;
}

gllm_status gllm_kv_release(gllm_kv* kv, const int32_t* pages, int32_t n) {
    if (!kv || n < 0 || (n > 0 && !pages)) return GLLM_E_INVALID;
    std::vector<int32_t> sorted(pages, pages + n);
    std::sort(sorted.begin(), sorted.end());
    for (int32_t i = 0; i < n; ++i) {
        if (!page_ok(kv, sorted[(size_t)i]) || kv->pool.holders(sorted[(size_t)i]) < 1) return GLLM_E_INVALID;
        if (i > 0 && sorted[(size_t)i] == sorted[(size_t)i - 1]) return GLLM_E_INVALID;
    }
    kv->pool.release(pages, (size_t)n);
    return GLLM_OK;
}

gllm_status gllm_kv_get_state(const gllm_kv* kv, gllm_kv_state* out) {
    if (!kv || !out) return GLLM_E_INVALID;
    out->total_pages = kv->pool.total();
    out->free_pages = kv->pool.free_count();
    out->idle_cached_pages = kv->pool.idle_cached();
    out->registered_pages = kv->pool.registered();
    out->evictions = kv->pool.evictions();
    return GLLM_OK;
}

gllm_status gllm_kv_page_info(const gllm_kv* kv, int32_t page, int32_t* holders, int32_t* is_registered, int32_t* children) {
    if (!kv || !holders || !is_registered || !children || !page_ok(kv, page)) return GLLM_E_INVALID;
    *holders = kv->pool.holders(page);
    *is_registered = kv->pool.is_registered(page) ? 1 : 0;
    *children = kv->pool.children(page);
    return GLLM_OK;
}

}  // extern "C"
