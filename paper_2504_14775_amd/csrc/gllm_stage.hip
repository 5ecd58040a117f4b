// C ABI and host-side executor of the stage forward (see include/gllm_stage.h).
//
// A forward call validates the batch descriptor, builds the per-batch metadata once (it is
// shared by all layers because every layer uses the same page tables, paper section 3.3),
// uploads it with one asynchronous copy from pinned staging, and enqueues, per layer:
//   RMSNorm -> QKV GEMM -> RoPE + paged KV write -> prefill attention, decode attention (+merge)
//   -> O GEMM -> residual add + RMSNorm -> gate/up GEMM (SwiGLU) -> down GEMM -> (residual add fused into the
//   next layer's RMSNorm)
// and finally the last residual add with the cast of the fp32 residual stream to bf16.  The O and down
// projections may be split along k; their partial products are summed in fixed order by the consumer.  Nothing in the call waits for the
// device, so consecutive batches queue back to back (the host-side preparation of batch i+1
// overlaps the execution of batch i, the "metadata ahead of data" idea of section 3.3).
#include "../../include/gllm_stage.h"
#include "common.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

namespace {

enum ProfClass {
    PC_RMSNORM = 0, PC_GEMM_QKV, PC_ROPE_KV, PC_ATTN_PREFILL, PC_ATTN_DECODE, PC_ATTN_MERGE, PC_GEMM_O,
    PC_GEMM_GATEUP, PC_GEMM_DOWN, PC_CAST, PC_COUNT
};
const char* kProfNames[PC_COUNT] = {"rmsnorm", "gemm_qkv", "rope_kv_write", "attn_prefill", "attn_decode",
                                    "attn_decode_merge", "gemm_o", "gemm_gate_up_swiglu", "gemm_down", "cast_out"};

thread_local std::string g_create_error;

struct LayerBuffers {
    bf16_t *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wd = nullptr, *norm1 = nullptr, *norm2 = nullptr,
           *bias = nullptr;
    bool loaded = false;
};

constexpr int kStagingSlots = 4;
constexpr int kMaxSplits = kMaxPlanes;

struct MetaLayout {  // offsets in bytes inside the metadata block (host staging and device copy alike)
    size_t tok_pos, tok_page, tok_own_v, bt_flat, dec_items, dec_order, dec_rows, pre_items, v_tiles, total;
};

}  // namespace

struct gllm_stage {
    gllm_stage_config cfg{};
    int device = 0;
    std::string err;
    // derived sizes
    int q_dim = 0, kv_dim = 0, n_qkv = 0, n_qkv_pad = 0, inter_pad = 0, hidden_pad_n = 0;
    int64_t m_pad = 0;
    int max_items = 0, max_pre_items = 0, max_v_tiles = 0, pre_rows = 64;
    std::vector<LayerBuffers> layers;
    bool borrowed_weights = false;  // the layer buffers belong to another stage (gllm_stage_share_weights)
    float* rope_cs = nullptr;  // device [max_position][d/2][2]
    // workspace
    void* ws = nullptr;
    size_t ws_bytes = 0;
    float* x = nullptr;
    bf16_t* h = nullptr;
    float* qkv = nullptr;
    bf16_t* q = nullptr;
    bf16_t* attn = nullptr;
    bf16_t* act = nullptr;
    float* part_o = nullptr;
    float* part_ml = nullptr;
    float* y = nullptr;  // [kMaxSplits][max_tokens][hidden] partial outputs of the O / down projections
    // pool
    bf16_t *k_pool = nullptr, *v_pool = nullptr;
    int64_t num_blocks = 0;
    // metadata
    MetaLayout ml{};  // capacities
    unsigned char* meta_dev = nullptr;
    unsigned char* staging[kStagingSlots] = {};
    hipEvent_t staging_ev[kStagingSlots] = {};
    bool staging_used[kStagingSlots] = {};
    int next_slot = 0;
    // prefill attention runs on a side stream, concurrently with decode attention (one is bound by the matrix
    // cores and latency, the other by HBM); fork/join events order it inside the caller's stream
    hipStream_t side = nullptr;
    hipEvent_t fork_ev[8] = {}, join_ev[8] = {};
    bool overlap_attention = true;
    bool alias_check = true;
    bool gemm_row_mixed = true;  // the GEMM planner may cover a short last row band with 64- or 128-row tiles
    int layer_begin = 0, layer_end = 0;  // forward() runs layers [layer_begin, layer_end) (layer_end is set at creation)
    int64_t decode_min_workgroups = 2048;  // partition the keys of decode rows until at least this many workgroups exist
    // profiling
    bool profiling = false;
    struct Span { int cls; hipEvent_t a, b; };
    std::vector<Span> spans;
    std::vector<hipEvent_t> ev_pool;
    double prof_ms[PC_COUNT] = {};
    int64_t prof_n[PC_COUNT] = {};
    // scratch for validation
    std::vector<int32_t> written_pages;
};

namespace {

gllm_status fail(gllm_stage* s, gllm_status code, const std::string& msg) {
    if (s) s->err = msg; else g_create_error = msg;
    return code;
}

gllm_status hip_fail(gllm_stage* s, hipError_t e, const char* what) {
    return fail(s, GLLM_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

void free_layer(LayerBuffers& L) {
    bf16_t** ps[] = {&L.wqkv, &L.wo, &L.wgu, &L.wd, &L.norm1, &L.norm2, &L.bias};
    for (bf16_t** p : ps) {
        if (*p) (void)hipFree(*p);
        *p = nullptr;
    }
    L.loaded = false;
}

// The repacked weights of one layer, zero filled (on the stream that will fill them) so that the padding is zero.
hipError_t alloc_layer(const gllm_stage* s, LayerBuffers& L, hipStream_t st) {
    const gllm_stage_config& c = s->cfg;
    struct { bf16_t** p; size_t n; } bufs[] = {
        {&L.wqkv, (size_t)s->n_qkv_pad * c.hidden},
        {&L.wo, (size_t)s->hidden_pad_n * s->q_dim},
        {&L.wgu, (size_t)2 * s->inter_pad * c.hidden},
        {&L.wd, (size_t)s->hidden_pad_n * s->inter_pad},
        {&L.norm1, (size_t)c.hidden}, {&L.norm2, (size_t)c.hidden},
        {&L.bias, (size_t)s->n_qkv_pad}};
    for (auto& b : bufs) {
        hipError_t e = hipMalloc((void**)b.p, b.n * 2);
        if (e == hipSuccess) e = hipMemsetAsync(*b.p, 0, b.n * 2, st);
        if (e != hipSuccess) {
            free_layer(L);
            return e;
        }
    }
    return hipSuccess;
}

#define HIP_TRY(stage, call)                                   \
    do {                                                       \
        hipError_t _e = (call);                                \
        if (_e != hipSuccess) return hip_fail(stage, _e, #call); \
    } while (0)

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t workspace_layout(gllm_stage* s, unsigned char* base) {
    const gllm_stage_config& c = s->cfg;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return base ? base + o : nullptr; };
    s->x = (float*)take((size_t)c.max_tokens * c.hidden * 4);
    s->h = (bf16_t*)take((size_t)s->m_pad * c.hidden * 2);
    s->qkv = (float*)take((size_t)kMaxSplits * c.max_tokens * s->n_qkv_pad * 4);
    s->q = (bf16_t*)take((size_t)c.max_tokens * s->q_dim * 2);
    s->attn = (bf16_t*)take((size_t)s->m_pad * s->q_dim * 2);
    s->act = (bf16_t*)take((size_t)s->m_pad * s->inter_pad * 2);
    s->part_o = (float*)take((size_t)s->max_items * c.n_q_heads * c.head_dim * 4);
    s->part_ml = (float*)take((size_t)s->max_items * c.n_q_heads * 2 * 4);
    s->y = (float*)take((size_t)kMaxSplits * c.max_tokens * c.hidden * 4);
    return off;
}

hipEvent_t get_event(gllm_stage* s) {
    if (!s->ev_pool.empty()) {
        hipEvent_t e = s->ev_pool.back();
        s->ev_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct ProfScope {
    gllm_stage* s;
    hipStream_t st;
    int cls;
    hipEvent_t a = nullptr, b = nullptr;
    ProfScope(gllm_stage* s_, hipStream_t st_, int cls_) : s(s_), st(st_), cls(cls_) {
        if (s->profiling) {
            a = get_event(s);
            b = get_event(s);
            if (a && b) (void)hipEventRecord(a, st);
        }
    }
    ~ProfScope() {
        if (s->profiling && a && b) {
            (void)hipEventRecord(b, st);
            s->spans.push_back({cls, a, b});
        }
    }
};

}  // namespace

extern "C" {

const char* gllm_status_name(gllm_status st) {
    switch (st) {
        case GLLM_OK: return "GLLM_OK";
        case GLLM_E_INVALID: return "GLLM_E_INVALID";
        case GLLM_E_CAPACITY: return "GLLM_E_CAPACITY";
        case GLLM_E_BLOCK_RANGE: return "GLLM_E_BLOCK_RANGE";
        case GLLM_E_BLOCK_ALIAS: return "GLLM_E_BLOCK_ALIAS";
        case GLLM_E_STATE: return "GLLM_E_STATE";
        case GLLM_E_HIP: return "GLLM_E_HIP";
        case GLLM_E_UNSUPPORTED: return "GLLM_E_UNSUPPORTED";
        default: return "GLLM_E_UNKNOWN";
    }
}

const char* gllm_last_error(const gllm_stage* stage) { return stage ? stage->err.c_str() : g_create_error.c_str(); }

int32_t gllm_profile_num_classes(void) { return PC_COUNT; }
const char* gllm_profile_class_name(int32_t i) { return (i >= 0 && i < PC_COUNT) ? kProfNames[i] : ""; }

gllm_status gllm_stage_create(const gllm_stage_config* cfg, gllm_stage** out) {
    if (!cfg || !out) return fail(nullptr, GLLM_E_INVALID, "null argument");
    *out = nullptr;
    const gllm_stage_config& c = *cfg;
    if (c.num_layers < 1 || c.hidden < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.intermediate < 1 ||
        c.max_tokens < 1 || c.max_seqs < 1 || c.max_blocks_per_seq < 1 || c.max_position < 1)
        return fail(nullptr, GLLM_E_INVALID, "non-positive size in config");
    if (c.page_size != kPage) return fail(nullptr, GLLM_E_UNSUPPORTED, "page_size must be 16");
    if (c.head_dim != 64 && c.head_dim != 128) return fail(nullptr, GLLM_E_UNSUPPORTED, "head_dim must be 64 or 128");
    if (c.n_q_heads % c.n_kv_heads != 0 || c.n_q_heads / c.n_kv_heads > 16)
        return fail(nullptr, GLLM_E_UNSUPPORTED, "n_q_heads must be a multiple of n_kv_heads with group size <= 16");
    if (c.hidden % 128 != 0) return fail(nullptr, GLLM_E_UNSUPPORTED, "hidden must be a multiple of 128");
    if ((c.n_q_heads * c.head_dim) % 64 != 0) return fail(nullptr, GLLM_E_UNSUPPORTED, "n_q_heads*head_dim must be a multiple of 64");
    if (c.intermediate % 8 != 0) return fail(nullptr, GLLM_E_UNSUPPORTED, "intermediate must be a multiple of 8");
    if ((int64_t)c.max_blocks_per_seq * kPage < c.max_position)
        return fail(nullptr, GLLM_E_INVALID, "max_blocks_per_seq * 16 is smaller than max_position");
    if (!(c.rms_eps >= 0.0) || !(c.rope_theta > 0.0)) return fail(nullptr, GLLM_E_INVALID, "bad rms_eps or rope_theta");

    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev < 1) return fail(nullptr, GLLM_E_HIP, "no HIP device available (this library has no CPU path)");
    gllm_stage* s = new gllm_stage();
    s->cfg = c;
    if (hipGetDevice(&s->device) != hipSuccess) { delete s; return fail(nullptr, GLLM_E_HIP, "hipGetDevice failed"); }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, s->device) != hipSuccess || std::string(prop.gcnArchName).rfind("gfx950", 0) != 0) {
        delete s;
        return fail(nullptr, GLLM_E_UNSUPPORTED, "the current device is not gfx950");
    }
    s->q_dim = c.n_q_heads * c.head_dim;
    s->kv_dim = c.n_kv_heads * c.head_dim;
    s->n_qkv = s->q_dim + 2 * s->kv_dim;
    s->n_qkv_pad = (int)round_up(s->n_qkv, kGemmPadN);
    s->inter_pad = (int)round_up(c.intermediate, kGemmPadN / 2);
    s->hidden_pad_n = (int)round_up(c.hidden, kGemmPadN);
    s->m_pad = round_up(c.max_tokens, kGemmPadM);
    s->max_items = 4 * c.max_seqs + 1024;
    s->pre_rows = prefill_item_rows(c.n_q_heads, c.n_kv_heads);
    s->max_pre_items = c.max_tokens / s->pre_rows + c.max_seqs + 1;
    s->max_v_tiles = c.max_tokens / kPage + 2 * c.max_seqs + 1;
    s->layers.resize(c.num_layers);
    s->layer_end = c.num_layers;

    auto bail = [&](hipError_t err, const char* what) {
        gllm_status st = hip_fail(nullptr, err, what);
        gllm_stage_destroy(s);
        return st;
    };
    // (the weight buffers of a layer are allocated when the layer is first loaded)
    // RoPE table: angle = pos * theta^(-2j/d), formed in double
    {
        const int half = c.head_dim / 2;
        std::vector<float> tab((size_t)c.max_position * half * 2);
        for (int p = 0; p < c.max_position; ++p)
            for (int j = 0; j < half; ++j) {
                double ang = (double)p * std::pow(c.rope_theta, -2.0 * j / (double)c.head_dim);
                tab[((size_t)p * half + j) * 2] = (float)std::cos(ang);
                tab[((size_t)p * half + j) * 2 + 1] = (float)std::sin(ang);
            }
        if ((e = hipMalloc((void**)&s->rope_cs, tab.size() * 4)) != hipSuccess) return bail(e, "hipMalloc(rope)");
        if ((e = hipMemcpy(s->rope_cs, tab.data(), tab.size() * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return bail(e, "hipMemcpy(rope)");
    }
    // metadata block
    {
        MetaLayout& m = s->ml;
        size_t off = 0;
        auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
        m.tok_pos = take((size_t)c.max_tokens * 4);
        m.tok_page = take((size_t)c.max_tokens * 4);
        m.tok_own_v = take((size_t)c.max_tokens * 4);
        m.bt_flat = take((size_t)c.max_seqs * c.max_blocks_per_seq * 4);
        m.dec_items = take((size_t)s->max_items * sizeof(DecodeItem));
        m.dec_order = take((size_t)s->max_items * 4);
        m.dec_rows = take((size_t)c.max_seqs * sizeof(DecodeRow));
        m.pre_items = take((size_t)s->max_pre_items * sizeof(PrefillItem));
        m.v_tiles = take((size_t)s->max_v_tiles * sizeof(VTile));
        m.total = off;
        if ((e = hipMalloc((void**)&s->meta_dev, m.total)) != hipSuccess) return bail(e, "hipMalloc(metadata)");
        for (int i = 0; i < kStagingSlots; ++i) {
            if ((e = hipHostMalloc((void**)&s->staging[i], m.total, hipHostMallocDefault)) != hipSuccess)
                return bail(e, "hipHostMalloc(staging)");
            if ((e = hipEventCreateWithFlags(&s->staging_ev[i], hipEventDisableTiming)) != hipSuccess)
                return bail(e, "hipEventCreate");
        }
    }
    if ((e = hipStreamCreateWithFlags(&s->side, hipStreamNonBlocking)) != hipSuccess) return bail(e, "hipStreamCreate");
    for (int i = 0; i < 8; ++i) {
        if ((e = hipEventCreateWithFlags(&s->fork_ev[i], hipEventDisableTiming)) != hipSuccess) return bail(e, "hipEventCreate");
        if ((e = hipEventCreateWithFlags(&s->join_ev[i], hipEventDisableTiming)) != hipSuccess) return bail(e, "hipEventCreate");
    }
    s->ws_bytes = workspace_layout(s, nullptr);
    *out = s;
    return GLLM_OK;
}

void gllm_stage_destroy(gllm_stage* s) {
    if (!s) return;
    (void)hipDeviceSynchronize();
    if (!s->borrowed_weights)
        for (auto& L : s->layers) free_layer(L);
    if (s->rope_cs) (void)hipFree(s->rope_cs);
    if (s->meta_dev) (void)hipFree(s->meta_dev);
    for (int i = 0; i < kStagingSlots; ++i) {
        if (s->staging[i]) (void)hipHostFree(s->staging[i]);
        if (s->staging_ev[i]) (void)hipEventDestroy(s->staging_ev[i]);
    }
    for (int i = 0; i < 8; ++i) {
        if (s->fork_ev[i]) (void)hipEventDestroy(s->fork_ev[i]);
        if (s->join_ev[i]) (void)hipEventDestroy(s->join_ev[i]);
    }
    if (s->side) (void)hipStreamDestroy(s->side);
    for (auto& sp : s->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (auto ev : s->ev_pool) (void)hipEventDestroy(ev);
    delete s;
}

size_t gllm_stage_workspace_bytes(const gllm_stage* s) { return s ? s->ws_bytes : 0; }

gllm_status gllm_stage_bind_workspace(gllm_stage* s, void* workspace, size_t bytes) {
    if (!s) return GLLM_E_INVALID;
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(s, GLLM_E_INVALID, "workspace must be a 256-byte aligned device pointer");
    if (bytes < s->ws_bytes) return fail(s, GLLM_E_CAPACITY, "workspace smaller than gllm_stage_workspace_bytes()");
    s->ws = workspace;
    workspace_layout(s, (unsigned char*)workspace);
    return GLLM_OK;
}

gllm_status gllm_stage_load_layer(gllm_stage* s, int32_t layer, const gllm_layer_weights* w, void* stream_) {
    if (!s) return GLLM_E_INVALID;
    if (!w || layer < 0 || layer >= s->cfg.num_layers) return fail(s, GLLM_E_INVALID, "bad layer index or null weights");
    if (s->borrowed_weights) return fail(s, GLLM_E_STATE, "this stage borrows its weights: load them into the owner");
    const gllm_stage_config& c = s->cfg;
    if (!w->wq || !w->wk || !w->wv || !w->wo || !w->wgate || !w->wup || !w->wdown || !w->norm1 || !w->norm2)
        return fail(s, GLLM_E_INVALID, "null weight pointer");
    if (c.has_qkv_bias && (!w->bq || !w->bk || !w->bv)) return fail(s, GLLM_E_INVALID, "has_qkv_bias set but a bias pointer is null");
    hipStream_t st = (hipStream_t)stream_;
    LayerBuffers& L = s->layers[layer];
    const int H = c.hidden;
    if (!L.wqkv) HIP_TRY(s, alloc_layer(s, L, st));
    HIP_TRY(s, launch_pack_rows_tiled((const bf16_t*)w->wq, H, s->q_dim, H, L.wqkv, H, 0, st));
    HIP_TRY(s, launch_pack_rows_tiled((const bf16_t*)w->wk, H, s->kv_dim, H, L.wqkv, H, s->q_dim, st));
    HIP_TRY(s, launch_pack_rows_tiled((const bf16_t*)w->wv, H, s->kv_dim, H, L.wqkv, H, s->q_dim + s->kv_dim, st));
    HIP_TRY(s, launch_pack_rows_tiled((const bf16_t*)w->wo, s->q_dim, H, s->q_dim, L.wo, s->q_dim, 0, st));
    HIP_TRY(s, launch_pack_gate_up((const bf16_t*)w->wgate, (const bf16_t*)w->wup, c.intermediate, H, L.wgu, H, st));
    HIP_TRY(s, launch_pack_rows_tiled((const bf16_t*)w->wdown, c.intermediate, H, c.intermediate, L.wd, s->inter_pad, 0, st));
    HIP_TRY(s, hipMemcpyAsync(L.norm1, w->norm1, (size_t)H * 2, hipMemcpyDeviceToDevice, st));
    HIP_TRY(s, hipMemcpyAsync(L.norm2, w->norm2, (size_t)H * 2, hipMemcpyDeviceToDevice, st));
    if (c.has_qkv_bias) {
        HIP_TRY(s, hipMemcpyAsync(L.bias, w->bq, (size_t)s->q_dim * 2, hipMemcpyDeviceToDevice, st));
        HIP_TRY(s, hipMemcpyAsync(L.bias + s->q_dim, w->bk, (size_t)s->kv_dim * 2, hipMemcpyDeviceToDevice, st));
        HIP_TRY(s, hipMemcpyAsync(L.bias + s->q_dim + s->kv_dim, w->bv, (size_t)s->kv_dim * 2, hipMemcpyDeviceToDevice, st));
    }
    L.loaded = true;
    return GLLM_OK;
}

gllm_status gllm_stage_share_weights(gllm_stage* s, const gllm_stage* owner) {
    if (!s) return GLLM_E_INVALID;
    if (!owner || owner == s) return fail(s, GLLM_E_INVALID, "no owner stage");
    const gllm_stage_config &a = s->cfg, &b = owner->cfg;
    if (a.num_layers != b.num_layers || a.hidden != b.hidden || a.n_q_heads != b.n_q_heads || a.n_kv_heads != b.n_kv_heads ||
        a.head_dim != b.head_dim || a.intermediate != b.intermediate || (a.has_qkv_bias != 0) != (b.has_qkv_bias != 0))
        return fail(s, GLLM_E_INVALID, "the two stages differ in their layer shapes");
    if (owner->borrowed_weights) return fail(s, GLLM_E_INVALID, "the owner stage borrows its weights itself");
    for (const LayerBuffers& L : owner->layers)
        if (!L.loaded) return fail(s, GLLM_E_STATE, "the owner stage has layers without weights");
    HIP_TRY(s, hipDeviceSynchronize());  // nothing of this stage may still read the buffers that are freed now
    if (!s->borrowed_weights)
        for (auto& L : s->layers) free_layer(L);
    s->layers = owner->layers;
    s->borrowed_weights = true;
    return GLLM_OK;
}

gllm_status gllm_stage_bind_kv_pool(gllm_stage* s, void* k_pool, void* v_pool, int64_t num_blocks) {
    if (!s) return GLLM_E_INVALID;
    if (!k_pool || !v_pool || num_blocks < 1) return fail(s, GLLM_E_INVALID, "null pool or no blocks");
    if (((uintptr_t)k_pool & 15) || ((uintptr_t)v_pool & 15)) return fail(s, GLLM_E_INVALID, "pools must be 16-byte aligned");
    if (num_blocks > INT32_MAX) return fail(s, GLLM_E_CAPACITY, "too many blocks");
    s->k_pool = (bf16_t*)k_pool;
    s->v_pool = (bf16_t*)v_pool;
    s->num_blocks = num_blocks;
    return GLLM_OK;
}

gllm_status gllm_stage_set_alias_check(gllm_stage* s, int32_t on) {
    if (!s) return GLLM_E_INVALID;
    s->alias_check = on != 0;
    return GLLM_OK;
}

gllm_status gllm_stage_set_option(gllm_stage* s, const char* name, int64_t value) {
    if (!s || !name) return GLLM_E_INVALID;
    if (std::strcmp(name, "overlap_attention") == 0) {
        s->overlap_attention = value != 0;
        return GLLM_OK;
    }
    if (std::strcmp(name, "gemm_row_mixed") == 0) {
        s->gemm_row_mixed = value != 0;
        return GLLM_OK;
    }
    if (std::strcmp(name, "layer_begin") == 0) {
        if (value < 0 || value >= s->cfg.num_layers) return fail(s, GLLM_E_INVALID, "layer_begin outside [0, num_layers)");
        s->layer_begin = (int)value;
        if (s->layer_end <= s->layer_begin) s->layer_end = s->layer_begin + 1;
        return GLLM_OK;
    }
    if (std::strcmp(name, "layer_end") == 0) {
        if (value < 1 || value > s->cfg.num_layers) return fail(s, GLLM_E_INVALID, "layer_end outside [1, num_layers]");
        s->layer_end = (int)value;
        if (s->layer_begin >= s->layer_end) s->layer_begin = s->layer_end - 1;
        return GLLM_OK;
    }
    if (std::strcmp(name, "decode_min_workgroups") == 0) {
        if (value < 1) return fail(s, GLLM_E_INVALID, "decode_min_workgroups must be positive");
        s->decode_min_workgroups = value;
        return GLLM_OK;
    }
    return fail(s, GLLM_E_INVALID, std::string("unknown option: ") + name);
}

gllm_status gllm_stage_set_profiling(gllm_stage* s, int32_t on) {
    if (!s) return GLLM_E_INVALID;
    s->profiling = on != 0;
    return GLLM_OK;
}

gllm_status gllm_stage_read_profile(gllm_stage* s, double* ms, int64_t* launches, int32_t reset) {
    if (!s) return GLLM_E_INVALID;
    for (auto& sp : s->spans) {
        HIP_TRY(s, hipEventSynchronize(sp.b));
        float t = 0.f;
        HIP_TRY(s, hipEventElapsedTime(&t, sp.a, sp.b));
        s->prof_ms[sp.cls] += t;
        s->prof_n[sp.cls] += 1;
        s->ev_pool.push_back(sp.a);
        s->ev_pool.push_back(sp.b);
    }
    s->spans.clear();
    for (int i = 0; i < PC_COUNT; ++i) {
        if (ms) ms[i] = s->prof_ms[i];
        if (launches) launches[i] = s->prof_n[i];
        if (reset) { s->prof_ms[i] = 0; s->prof_n[i] = 0; }
    }
    return GLLM_OK;
}

gllm_status gllm_stage_forward(gllm_stage* s, const gllm_batch* b, const void* hidden_in, void* hidden_out,
                               float* hidden_out_f32, void* stream_) {
    if (!s) return GLLM_E_INVALID;
    const gllm_stage_config& c = s->cfg;
    if (!b || !hidden_in || !hidden_out) return fail(s, GLLM_E_INVALID, "null argument");
    if (!s->ws) return fail(s, GLLM_E_STATE, "workspace not bound");
    if (!s->k_pool) return fail(s, GLLM_E_STATE, "KV pool not bound");
    for (int l = s->layer_begin; l < s->layer_end; ++l)
        if (!s->layers[l].loaded) return fail(s, GLLM_E_STATE, "layer " + std::to_string(l) + " not loaded");
    const int S = b->num_seqs;
    if (S < 0 || (S > 0 && (!b->new_tokens || !b->cached_len || !b->block_tables)))
        return fail(s, GLLM_E_INVALID, "null batch arrays or negative num_seqs");
    if (S > c.max_seqs) return fail(s, GLLM_E_INVALID, "num_seqs exceeds max_seqs");

    // ---- validation (no side effects before it has passed) ----
    int64_t T = 0, total_pages = 0;
    for (int i = 0; i < S; ++i) {
        const int n = b->new_tokens[i], cl = b->cached_len[i];
        if (n < 1) return fail(s, GLLM_E_INVALID, "new_tokens < 1 for sequence " + std::to_string(i));
        if (cl < 0) return fail(s, GLLM_E_INVALID, "cached_len < 0 for sequence " + std::to_string(i));
        const int64_t end = (int64_t)n + cl;
        if (end > c.max_position) return fail(s, GLLM_E_CAPACITY, "sequence " + std::to_string(i) + " exceeds max_position");
        const int64_t pages = ceil_div(end, kPage);
        if (pages > c.max_blocks_per_seq || pages > b->block_table_stride)
            return fail(s, GLLM_E_CAPACITY, "sequence " + std::to_string(i) + " needs more pages than the table holds");
        T += n;
        total_pages += pages;
        if (T > c.max_tokens) return fail(s, GLLM_E_CAPACITY, "batch exceeds max_tokens");
        const int32_t* row = b->block_tables + (int64_t)i * b->block_table_stride;
        for (int64_t p = 0; p < pages; ++p)
            if (row[p] < 0 || row[p] >= s->num_blocks)
                return fail(s, GLLM_E_BLOCK_RANGE, "sequence " + std::to_string(i) + " logical page " + std::to_string(p) +
                                                       " names page " + std::to_string(row[p]) + " outside the pool");
    }
    if (s->alias_check) {
        s->written_pages.clear();
        for (int i = 0; i < S; ++i) {
            const int32_t* row = b->block_tables + (int64_t)i * b->block_table_stride;
            const int first = b->cached_len[i] / kPage, last = (b->cached_len[i] + b->new_tokens[i] - 1) / kPage;
            for (int p = first; p <= last; ++p) s->written_pages.push_back(row[p]);
        }
        std::sort(s->written_pages.begin(), s->written_pages.end());
        if (std::adjacent_find(s->written_pages.begin(), s->written_pages.end()) != s->written_pages.end())
            return fail(s, GLLM_E_BLOCK_ALIAS, "two (sequence, logical page) pairs receiving new tokens share a physical page");
    }
    if (T == 0) return GLLM_OK;

    // ---- decode partitioning ----
    int n_dec = 0;
    for (int i = 0; i < S; ++i) n_dec += b->new_tokens[i] == 1;
    int part = 256;
    if (n_dec > 0) {
        auto items_for = [&](int P) {
            int64_t n = 0;
            for (int i = 0; i < S; ++i)
                if (b->new_tokens[i] == 1) n += ceil_div((int64_t)b->cached_len[i] + 1, P);
            return n;
        };
        // largest partition that still yields a few workgroups per compute unit
        const int64_t want = s->decode_min_workgroups;
        part = 256;
        for (int P = 16384; P >= 256; P >>= 1)
            if (items_for(P) * c.n_kv_heads >= want) { part = P; break; }
        while (items_for(part) > s->max_items) part <<= 1;
    }

    // ---- metadata into a pinned staging slot ----
    const int slot = s->next_slot;
    s->next_slot = (slot + 1) % kStagingSlots;
    if (s->staging_used[slot]) HIP_TRY(s, hipEventSynchronize(s->staging_ev[slot]));
    unsigned char* st_base = s->staging[slot];
    // compact layout for this batch: only what is used travels to the device
    int64_t cnt_items = 0, cnt_pre = 0, cnt_vt = 0;
    for (int i = 0; i < S; ++i) {
        if (b->new_tokens[i] == 1) cnt_items += ceil_div((int64_t)b->cached_len[i] + 1, part);
        else {
            cnt_pre += ceil_div(b->new_tokens[i], s->pre_rows);
            cnt_vt += ((int64_t)b->cached_len[i] + b->new_tokens[i] - 1) / kPage - b->cached_len[i] / kPage + 1;
        }
    }
    if (cnt_items > s->max_items || cnt_pre > s->max_pre_items || cnt_vt > s->max_v_tiles)
        return fail(s, GLLM_E_CAPACITY, "internal work list overflow");
    MetaLayout ml{};
    {
        size_t off = 0;
        auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
        ml.tok_pos = take((size_t)T * 4);
        ml.tok_page = take((size_t)T * 4);
        ml.tok_own_v = take((size_t)T * 4);
        ml.bt_flat = take((size_t)total_pages * 4);
        ml.dec_items = take((size_t)cnt_items * sizeof(DecodeItem));
        ml.dec_order = take((size_t)cnt_items * 4);
        ml.dec_rows = take((size_t)n_dec * sizeof(DecodeRow));
        ml.pre_items = take((size_t)cnt_pre * sizeof(PrefillItem));
        ml.v_tiles = take((size_t)cnt_vt * sizeof(VTile));
        ml.total = off;
    }
    int32_t* tok_pos = (int32_t*)(st_base + ml.tok_pos);
    int32_t* tok_page = (int32_t*)(st_base + ml.tok_page);
    int32_t* tok_own_v = (int32_t*)(st_base + ml.tok_own_v);
    VTile* v_tiles = (VTile*)(st_base + ml.v_tiles);
    int32_t* bt_flat = (int32_t*)(st_base + ml.bt_flat);
    DecodeItem* dec_items = (DecodeItem*)(st_base + ml.dec_items);
    int32_t* dec_order = (int32_t*)(st_base + ml.dec_order);
    DecodeRow* dec_rows = (DecodeRow*)(st_base + ml.dec_rows);
    PrefillItem* pre_items = (PrefillItem*)(st_base + ml.pre_items);
    int n_items = 0, n_rows = 0, n_pre = 0, n_vt = 0;
    int64_t bt_off = 0, row = 0;
    for (int i = 0; i < S; ++i) {
        const int n = b->new_tokens[i], cl = b->cached_len[i];
        const int32_t* tab = b->block_tables + (int64_t)i * b->block_table_stride;
        const int pages = (int)ceil_div((int64_t)n + cl, kPage);
        std::memcpy(bt_flat + bt_off, tab, (size_t)pages * 4);
        for (int t = 0; t < n; ++t) {
            tok_pos[row + t] = cl + t;
            tok_page[row + t] = tab[(cl + t) / kPage];
            tok_own_v[row + t] = n == 1;
        }
        if (n > 1)  // the V of a chunk is written run by run: the tokens that share a page
            for (int p0 = cl; p0 < cl + n;) {
                const int p1 = std::min(cl + n, (p0 / kPage + 1) * kPage);
                v_tiles[n_vt++] = VTile{(int32_t)(row + p0 - cl), p1 - p0, tab[p0 / kPage], p0 % kPage};
                p0 = p1;
            }
        if (n == 1) {
            const int len = cl + 1;
            // equal shares (whole 32-key blocks) rather than full partitions plus a short remainder
            const int nparts = (int)ceil_div(len, part);
            const int share = (int)ceil_div(ceil_div(len, nparts), 32) * 32;
            const int first = n_items;
            for (int k0 = 0; k0 < len; k0 += share)
                dec_items[n_items++] = DecodeItem{(int32_t)row, (int32_t)bt_off, k0, std::min(k0 + share, len), 0};
            // a row with a single item is finished by the attention kernel; the others are merged afterwards
            if (n_items - first == 1) dec_items[first].single = 1;
            else dec_rows[n_rows++] = DecodeRow{(int32_t)row, first, n_items - first, 0};
        } else {
            for (int t0 = 0; t0 < n; t0 += s->pre_rows)
                pre_items[n_pre++] = PrefillItem{(int32_t)(row + t0), std::min(s->pre_rows, n - t0), cl + t0,
                                                 (int32_t)bt_off};
        }
        bt_off += pages;
        row += n;
    }
    // launch order, both kinds of attention: longest first, so that the last workgroups to start are the shortest
    // (a chunk deep in a long prompt attends to many times the keys of a chunk that starts one)
    std::stable_sort(pre_items, pre_items + n_pre, [](const PrefillItem& x, const PrefillItem& y) {
        return x.pos0 + x.n_rows > y.pos0 + y.n_rows;
    });
    for (int i = 0; i < n_items; ++i) dec_order[i] = i;
    std::stable_sort(dec_order, dec_order + n_items, [&](int32_t x, int32_t y) {
        return dec_items[x].kv_end - dec_items[x].kv_begin > dec_items[y].kv_end - dec_items[y].kv_begin;
    });
    hipStream_t st = (hipStream_t)stream_;
    HIP_TRY(s, hipMemcpyAsync(s->meta_dev, st_base, ml.total, hipMemcpyHostToDevice, st));
    HIP_TRY(s, hipEventRecord(s->staging_ev[slot], st));
    s->staging_used[slot] = true;

    const int32_t* d_tok_pos = (const int32_t*)(s->meta_dev + ml.tok_pos);
    const int32_t* d_tok_page = (const int32_t*)(s->meta_dev + ml.tok_page);
    const int32_t* d_tok_own_v = (const int32_t*)(s->meta_dev + ml.tok_own_v);
    const VTile* d_v_tiles = (const VTile*)(s->meta_dev + ml.v_tiles);
    const int32_t* d_bt = (const int32_t*)(s->meta_dev + ml.bt_flat);
    const DecodeItem* d_items = (const DecodeItem*)(s->meta_dev + ml.dec_items);
    const int32_t* d_order = (const int32_t*)(s->meta_dev + ml.dec_order);
    const DecodeRow* d_rows = (const DecodeRow*)(s->meta_dev + ml.dec_rows);
    const PrefillItem* d_pre = (const PrefillItem*)(s->meta_dev + ml.pre_items);

    const int Ti = (int)T, H = c.hidden, d = c.head_dim;
    const int64_t pool_layer = (int64_t)s->num_blocks * c.n_kv_heads * kPage * d;
    const float eps = (float)c.rms_eps;
    const int64_t y_plane = (int64_t)c.max_tokens * H;
    // tile shapes and split-K factors for this batch size (the consumers sum the partial planes in order)
    const bool rm = s->gemm_row_mixed;
    const GemmPlan plan_qkv = gemm_plan(Ti, s->n_qkv_pad, H, GEMM_STORE_F32, kMaxSplits, rm);
    const GemmPlan plan_o = gemm_plan(Ti, H, s->q_dim, GEMM_STORE_F32, kMaxSplits, rm);
    const GemmPlan plan_gu = gemm_plan(Ti, 2 * s->inter_pad, H, GEMM_SWIGLU_BF16, 1, rm);
    const GemmPlan plan_d = gemm_plan(Ti, H, s->inter_pad, GEMM_STORE_F32, kMaxSplits, rm);
    const int split_o = plan_o.splits, split_d = plan_d.splits;
    const int64_t qkv_plane = (int64_t)c.max_tokens * s->n_qkv_pad;
    int pending = 0;  // planes of y still to be added to the residual stream
    for (int l = s->layer_begin; l < s->layer_end; ++l) {
        const LayerBuffers& L = s->layers[l];
        {
            ProfScope ps(s, st, PC_RMSNORM);
            if (l == s->layer_begin) HIP_TRY(s, launch_rmsnorm_from_bf16((const bf16_t*)hidden_in, s->x, L.norm1, s->h, H, Ti, H, eps, st));
            else HIP_TRY(s, launch_add_rmsnorm(s->x, s->y, pending, y_plane, L.norm1, s->h, H, Ti, H, eps, st));
        }
        {
            ProfScope ps(s, st, PC_GEMM_QKV);
            HIP_TRY(s, launch_gemm_bf16(s->h, H, L.wqkv, H, s->qkv, s->n_qkv_pad, Ti, s->n_qkv_pad, H, GEMM_STORE_F32, plan_qkv.tile,
                                        plan_qkv.splits, qkv_plane, st));
        }
        {
            ProfScope ps(s, st, PC_ROPE_KV);
            RopeKvArgs a{};
            a.qkv = s->qkv; a.ld_qkv = s->n_qkv_pad; a.planes = plan_qkv.splits; a.plane_stride = qkv_plane;
            a.bias = c.has_qkv_bias ? L.bias : nullptr;
            a.rope_cs = s->rope_cs; a.tok_pos = d_tok_pos; a.tok_page = d_tok_page;
            a.q_out = s->q; a.ld_q = s->q_dim;
            a.k_pool = s->k_pool + (int64_t)l * pool_layer; a.v_pool = s->v_pool + (int64_t)l * pool_layer;
            a.T = Ti; a.n_q = c.n_q_heads; a.n_kv = c.n_kv_heads; a.d = d;
            a.v_tiles = d_v_tiles; a.n_vtiles = n_vt; a.tok_own_v = d_tok_own_v;
            HIP_TRY(s, launch_rope_kv_write(a, st));
        }
        AttnArgs aa{};
        aa.q = s->q; aa.ld_q = s->q_dim;
        aa.k_pool = s->k_pool + (int64_t)l * pool_layer; aa.v_pool = s->v_pool + (int64_t)l * pool_layer;
        aa.bt_flat = d_bt; aa.out = s->attn; aa.ld_o = s->q_dim;
        aa.n_q = c.n_q_heads; aa.n_kv = c.n_kv_heads; aa.d = d;
        aa.scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)d));
        // both attention kernels read q and the pool and write disjoint rows of attn
        const bool fork = n_pre > 0 && n_items > 0 && s->overlap_attention && !s->profiling;
        if (n_pre > 0) {
            hipStream_t ps_stream = st;
            if (fork) {
                HIP_TRY(s, hipEventRecord(s->fork_ev[l & 7], st));
                HIP_TRY(s, hipStreamWaitEvent(s->side, s->fork_ev[l & 7], 0));
                ps_stream = s->side;
            }
            ProfScope ps(s, ps_stream, PC_ATTN_PREFILL);
            HIP_TRY(s, launch_prefill_attention(aa, d_pre, n_pre, ps_stream));
            if (fork) HIP_TRY(s, hipEventRecord(s->join_ev[l & 7], s->side));
        }
        if (n_items > 0) {
            {
                ProfScope ps(s, st, PC_ATTN_DECODE);
                HIP_TRY(s, launch_decode_attention(aa, d_items, d_order, n_items, s->part_o, s->part_ml, st));
            }
            ProfScope ps(s, st, PC_ATTN_MERGE);
            HIP_TRY(s, launch_decode_combine(aa, d_rows, n_rows, s->part_o, s->part_ml, st));
        }
        if (fork) HIP_TRY(s, hipStreamWaitEvent(st, s->join_ev[l & 7], 0));
        {
            // the projection writes split_o partial products; the next RMSNorm adds them to the residual stream
            ProfScope ps(s, st, PC_GEMM_O);
            HIP_TRY(s, launch_gemm_bf16(s->attn, s->q_dim, L.wo, s->q_dim, s->y, H, Ti, H, s->q_dim, GEMM_STORE_F32, plan_o.tile, split_o, y_plane, st));
        }
        {
            ProfScope ps(s, st, PC_RMSNORM);
            HIP_TRY(s, launch_add_rmsnorm(s->x, s->y, split_o, y_plane, L.norm2, s->h, H, Ti, H, eps, st));
        }
        {
            ProfScope ps(s, st, PC_GEMM_GATEUP);
            HIP_TRY(s, launch_gemm_bf16(s->h, H, L.wgu, H, s->act, s->inter_pad, Ti, 2 * s->inter_pad, H, GEMM_SWIGLU_BF16, plan_gu.tile, 1, 0, st));
        }
        {
            ProfScope ps(s, st, PC_GEMM_DOWN);
            HIP_TRY(s, launch_gemm_bf16(s->act, s->inter_pad, L.wd, s->inter_pad, s->y, H, Ti, H, s->inter_pad, GEMM_STORE_F32, plan_d.tile, split_d, y_plane, st));
        }
        pending = split_d;
    }
    {
        ProfScope ps(s, st, PC_CAST);
        HIP_TRY(s, launch_add_cast_out(s->x, s->y, pending, y_plane, (bf16_t*)hidden_out, hidden_out_f32, (int64_t)Ti * H, st));
    }
    return GLLM_OK;
}

gllm_status gllm_op_gemm_bf16(const void* a, int64_t lda, const void* w, int64_t ldw, void* out, int64_t ldc,
                              int32_t m, int32_t n, int32_t k, int32_t mode, int32_t tile, void* stream) {
    if (!a || !w || !out) return GLLM_E_INVALID;
    hipError_t e = launch_gemm_bf16((const bf16_t*)a, lda, (const bf16_t*)w, ldw, out, ldc, m, n, k, mode, tile, 1, 0, (hipStream_t)stream);
    return e == hipSuccess ? GLLM_OK : (e == hipErrorInvalidValue ? GLLM_E_UNSUPPORTED : GLLM_E_HIP);
}

gllm_status gllm_op_gemm_bf16_splitk(const void* a, int64_t lda, const void* w, int64_t ldw, float* out, int64_t ldc,
                                     int32_t m, int32_t n, int32_t k, int32_t tile, int32_t splits, int64_t plane_stride,
                                     void* stream) {
    if (!a || !w || !out) return GLLM_E_INVALID;
    hipError_t e = launch_gemm_bf16((const bf16_t*)a, lda, (const bf16_t*)w, ldw, out, ldc, m, n, k, GEMM_STORE_F32, tile,
                                    splits, plane_stride, (hipStream_t)stream);
    return e == hipSuccess ? GLLM_OK : (e == hipErrorInvalidValue ? GLLM_E_UNSUPPORTED : GLLM_E_HIP);
}

gllm_status gllm_op_pack_weight(const void* w, int64_t ldw, int32_t n, int32_t k, void* out, void* stream) {
    if (!w || !out || n < 1 || k < 1) return GLLM_E_INVALID;
    if (n % kWBlock != 0 || k % kWBlock != 0 || ldw < k || ldw % 8 != 0 || ((uintptr_t)w & 15) || ((uintptr_t)out & 15))
        return GLLM_E_UNSUPPORTED;
    hipError_t e = launch_pack_rows_tiled((const bf16_t*)w, ldw, n, k, (bf16_t*)out, k, 0, (hipStream_t)stream);
    return e == hipSuccess ? GLLM_OK : GLLM_E_HIP;
}

gllm_status gllm_op_gemm_plan(int32_t m, int32_t n, int32_t k, int32_t mode, int32_t max_splits, int32_t* tile,
                              int32_t* splits) {
    if (!tile || !splits || m < 1 || n < 1 || k < 1 || n % 64 != 0 || k % 64 != 0 || max_splits < 1 || mode < 0 ||
        mode > GEMM_SWIGLU_BF16)
        return GLLM_E_INVALID;
    const GemmPlan p = gemm_plan(m, n, k, mode, max_splits);
    *tile = p.tile;
    *splits = p.splits;
    return GLLM_OK;
}

gllm_status gllm_op_rmsnorm(const float* x, const void* gamma, void* h, int32_t rows, int32_t hidden, double eps,
                            void* stream) {
    if (!x || !gamma || !h || hidden % 4 != 0) return GLLM_E_INVALID;
    hipError_t e = launch_add_rmsnorm(const_cast<float*>(x), nullptr, 0, 0, (const bf16_t*)gamma, (bf16_t*)h, hidden, rows, hidden, (float)eps, (hipStream_t)stream);
    return e == hipSuccess ? GLLM_OK : GLLM_E_HIP;
}

gllm_status gllm_op_peak_mfma(void* sink, int32_t workgroups, int32_t iters, void* stream) {
    if (!sink || workgroups < 1 || iters < 1) return GLLM_E_INVALID;
    return launch_peak_mfma((float*)sink, workgroups, iters, (hipStream_t)stream) == hipSuccess ? GLLM_OK : GLLM_E_HIP;
}

gllm_status gllm_op_peak_read(const void* src, int64_t bytes, void* sink, int32_t workgroups, void* stream) {
    if (!src || !sink || bytes < 16 || workgroups < 1) return GLLM_E_INVALID;
    return launch_peak_read(src, bytes, sink, workgroups, (hipStream_t)stream) == hipSuccess ? GLLM_OK : GLLM_E_HIP;
}

gllm_status gllm_op_peak_read_nt(const void* src, int64_t bytes, void* sink, int32_t workgroups, void* stream) {
    if (!src || !sink || bytes < 16 || workgroups < 1) return GLLM_E_INVALID;
    return launch_peak_read(src, bytes, sink, workgroups, (hipStream_t)stream, true) == hipSuccess ? GLLM_OK : GLLM_E_HIP;
}

}  // extern "C"
