// Token Throttling micro-batch scheduler (arxiv 2504.14775, section 3) and the chunked-prefill baseline
// (section 2.2); host code only.  See include/gllm_sched.h for the contract of every entry point.
#include "../../include/gllm_sched.h"

#include <algorithm>
#include <cstdint>
#include <deque>
#include <limits>
#include <new>
#include <unordered_map>
#include <vector>

#include "page_pool.h"

namespace {

constexpr int64_t kPageTokens = 16;
constexpr int64_t kNoLimit = std::numeric_limits<int64_t>::max() / 4;

inline int64_t div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }

bool params_ok(const gllm_sched_params* p) {
    return p && (p->policy == GLLM_POLICY_CHUNKED_PREFILL || p->policy == GLLM_POLICY_TOKEN_THROTTLING) &&
           p->iters_t >= 1 && p->min_p >= 1 && p->max_p >= p->min_p && p->kv_thresh_bp >= 0 && p->kv_thresh_bp <= 9999 &&
           p->pp_depth >= 1 && p->token_budget >= 1 && p->total_pages >= 1 && p->total_pages < (int64_t)1 << 31 &&
           (p->prefix_caching == 0 || p->prefix_caching == 1);
}

// Eq. 3.  The idle-rate comparison and the idle-rate term are kept in integers: KV_free = free / total and
// KV_thresh = bp / 10000 give (KV_free - KV_thresh) / (1 - KV_thresh) = (10000 free - bp total) / ((10000 - bp) total).
int64_t prefill_tokens(const gllm_sched_params& p, int64_t wp, int64_t free_pages) {
    if (wp <= 0) return 0;
    const int64_t idle = free_pages * 10000, bar = (int64_t)p.kv_thresh_bp * p.total_pages;
    if (idle < bar) return 0;  // the text of "Threshold": prefill is suspended
    int64_t n = p.max_p;
    if (p.use_wt) n = std::min(n, div_up(wp, p.iters_t));
    if (p.use_ut) n = std::min(n, (int64_t)p.max_p * (idle - bar) / ((int64_t)(10000 - p.kv_thresh_bp) * p.total_pages));
    n = std::max<int64_t>(n, p.min_p);
    return std::min(n, wp);
}

struct Seq {
    int64_t prompt = 0, output = 0;
    int64_t prefilled = 0;   // prompt tokens in the cache
    int64_t produced = 0;    // output tokens so far
    int64_t chunk = 0;       // prompt tokens in flight
    int64_t decode_rank = -1;  // order of entering the decode phase
    bool flying = false;
    std::vector<int32_t> pages;
    // prefix caching: the token ids known from position 0 on (the prompt as given on arrival, then the output
    // tokens the caller has reported), how many leading pages of `pages` are in the pool's tree, and whether this
    // request still registers the pages it fills
    std::vector<int32_t> tokens;
    int64_t entered = 0;
    bool entering = true;
};

struct Row {
    int64_t id;
    int32_t count, cached;
    bool decode;
};

}  // namespace

struct gllm_sched {
    gllm_sched_params p;
    std::unordered_map<int64_t, Seq> seqs;
    std::deque<int64_t> waiting;  // first come, first served
    std::deque<int64_t> idle_decode;  // decode requests not in flight, least recently run in front
    gllm::PagePool pool;
    std::unordered_map<int64_t, std::vector<Row>> flying;
    int64_t decode_total = 0, waiting_tokens = 0, next_batch_id = 0, next_rank = 0, preempted = 0, hit_tokens = 0;

    explicit gllm_sched(const gllm_sched_params& q) : p(q), pool(q.total_pages) {}
    void admit(int64_t id, int32_t prompt_len, int32_t output_len, const int32_t* tokens) {
        Seq q;
        q.prompt = prompt_len;
        q.output = output_len;
        if (tokens && p.prefix_caching) q.tokens.assign(tokens, tokens + prompt_len);
        seqs.emplace(id, std::move(q));
        waiting.push_back(id);
        waiting_tokens += prompt_len;
    }
    int64_t spare() const { return pool.available(); }
    void grab(Seq& s, int64_t n) {
        for (int64_t i = 0; i < n; ++i) s.pages.push_back(pool.alloc());
    }
    void give_back(Seq& s) {
        pool.release(s.pages.data(), s.pages.size());
        s.pages.clear();
        s.entered = 0;
        s.entering = true;
    }
    // A request about to receive its first chunk (again): the cached whole pages of its prompt open its block
    // table, but at least one token is left to compute.
    void look_up(Seq& s) {
        const int64_t found = pool.match(s.tokens.data(), (int64_t)s.tokens.size(), (s.prompt - 1) / kPageTokens, s.pages);
        s.entered = found;
        s.prefilled = found * kPageTokens;
        waiting_tokens -= s.prefilled;
        hit_tokens += s.prefilled;
    }
    // The whole pages of known tokens among the first in_cache positions (those whose KV has been computed) enter
    // the pool's tree, until a page turns out to be there already.
    void enter_filled_pages(Seq& s, int64_t in_cache) {
        const int64_t whole = std::min<int64_t>(in_cache, (int64_t)s.tokens.size()) / kPageTokens;
        while (s.entering && s.entered < whole) {
            const size_t i = (size_t)s.entered;
            const int32_t parent = i ? s.pages[i - 1] : gllm::PagePool::kRoot;
            if (pool.enter(parent, s.tokens.data() + i * kPageTokens, s.pages[i])) ++s.entered;
            else s.entering = false;
        }
    }
    // Recomputation: the request goes back to the head of the waiting queue, its output so far becomes prompt.
    void evict(int64_t id) {
        Seq& s = seqs[id];
        idle_decode.erase(std::find(idle_decode.begin(), idle_decode.end(), id));
        --decode_total;
        give_back(s);
        s.prompt += s.produced;
        s.output -= s.produced;
        s.produced = 0;
        s.prefilled = 0;
        s.decode_rank = -1;
        waiting.push_front(id);
        waiting_tokens += s.prompt;
        ++preempted;
    }
    // Takes back the pages of the last waiting request that holds some and is not in flight, looking only behind
    // queue position `from`; that request keeps its place and starts its prompt over.
    bool strip_last_waiting(size_t from) {
        for (size_t i = waiting.size(); i-- > from;) {
            Seq& s = seqs[waiting[i]];
            if (s.flying || s.pages.empty()) continue;
            give_back(s);
            waiting_tokens += s.prefilled;
            s.prefilled = 0;
            ++preempted;
            return true;
        }
        return false;
    }
    // The rows of the next micro-batch; empty when nothing can run (evictions made on the way stay in force).
    std::vector<Row> plan() {
        std::vector<Row> rows;
        if ((int64_t)flying.size() >= p.pp_depth) return rows;
        const int64_t free_before = spare();
        int64_t slots = p.policy == GLLM_POLICY_TOKEN_THROTTLING ? div_up(decode_total, p.pp_depth) : p.token_budget;
        for (; slots > 0 && !idle_decode.empty(); --slots) {
            const int64_t id = idle_decode.front();
            Seq& s = seqs[id];
            const int64_t cached = s.prompt + s.produced - 1;
            const int64_t extra = div_up(cached + 1, kPageTokens) - (int64_t)s.pages.size();
            while (extra > spare()) {
                int64_t victim = -1, best = -1;
                for (int64_t other : idle_decode)
                    if (other != id && seqs[other].decode_rank > best) {
                        best = seqs[other].decode_rank;
                        victim = other;
                    }
                if (victim >= 0) evict(victim);
                else if (!strip_last_waiting(0)) break;
            }
            if (extra > spare()) break;
            idle_decode.pop_front();
            grab(s, extra);
            s.flying = true;
            rows.push_back(Row{id, 1, (int32_t)cached, true});
        }
        const int64_t decode_rows = (int64_t)rows.size();
        int64_t left = p.policy == GLLM_POLICY_TOKEN_THROTTLING
                           ? prefill_tokens(p, waiting_tokens, free_before)
                           : std::min(std::max<int64_t>(p.token_budget - decode_rows, 0), waiting_tokens);
        for (size_t i = 0; i < waiting.size() && left > 0; ++i) {
            Seq& s = seqs[waiting[i]];
            if (s.flying) continue;
            if (!s.tokens.empty() && s.prefilled == 0 && s.pages.empty()) look_up(s);
            auto room_for = [&]() { return ((int64_t)s.pages.size() + spare()) * kPageTokens - s.prefilled; };
            int64_t room = room_for();
            while (room <= 0 && strip_last_waiting(i + 1)) room = room_for();
            if (room <= 0) break;  // the head of the queue blocks the rest
            const int64_t n = std::min({s.prompt - s.prefilled, left, room});
            grab(s, div_up(s.prefilled + n, kPageTokens) - (int64_t)s.pages.size());
            s.flying = true;
            s.chunk = n;
            waiting_tokens -= n;
            left -= n;
            rows.push_back(Row{waiting[i], (int32_t)n, (int32_t)s.prefilled, false});
        }
        return rows;
    }
    int64_t launch(std::vector<Row>&& rows) {
        const int64_t id = next_batch_id++;
        flying.emplace(id, std::move(rows));
        return id;
    }
    // Returns the ids of the requests that ended, in row order.  row_tokens: per row the token it produced (null or
    // negative: not reported).
    std::vector<int64_t> retire(int64_t batch, const int32_t* row_tokens = nullptr) {
        std::vector<int64_t> ended;
        auto it = flying.find(batch);
        std::vector<Row> rows = std::move(it->second);
        flying.erase(it);
        for (size_t i = 0; i < rows.size(); ++i) {
            const Row& r = rows[i];
            Seq& s = seqs[r.id];
            s.flying = false;
            if (r.decode) {
                ++s.produced;
            } else {
                s.chunk = 0;
                s.prefilled += r.count;
                if (s.prefilled < s.prompt) {
                    if (!s.tokens.empty()) enter_filled_pages(s, s.prefilled);
                    continue;
                }
                waiting.erase(std::find(waiting.begin(), waiting.end(), r.id));
                s.produced = 1;
                s.decode_rank = next_rank++;
                ++decode_total;
            }
            if (!s.tokens.empty()) {
                const int64_t in_cache = s.prompt + s.produced - 1;  // the newest token's KV is not computed yet
                if (row_tokens && row_tokens[i] >= 0 && (int64_t)s.tokens.size() == in_cache) s.tokens.push_back(row_tokens[i]);
                enter_filled_pages(s, in_cache);
            }
            if (s.produced >= s.output) {
                --decode_total;
                give_back(s);
                ended.push_back(r.id);
            } else {
                idle_decode.push_back(r.id);
            }
        }
        return ended;
    }
};

extern "C" {

int64_t gllm_sched_prefill_budget(const gllm_sched_params* p, int64_t wp, int64_t free_pages) {
    if (!params_ok(p) || wp < 0 || free_pages < 0 || free_pages > p->total_pages) return -1;
    return prefill_tokens(*p, wp, free_pages);
}

int64_t gllm_sched_decode_budget(const gllm_sched_params* p, int64_t rd) {
    if (!params_ok(p) || rd < 0) return -1;
    return div_up(rd, p->pp_depth);
}

gllm_status gllm_sched_create(const gllm_sched_params* p, gllm_sched** out) {
    if (!out) return GLLM_E_INVALID;
    *out = nullptr;
    if (!params_ok(p)) return GLLM_E_INVALID;
    gllm_sched* s = new (std::nothrow) gllm_sched(*p);
    if (!s) return GLLM_E_CAPACITY;
    *out = s;
    return GLLM_OK;
}

void gllm_sched_destroy(gllm_sched* s) { delete s; }

gllm_status gllm_sched_add_request_tokens(gllm_sched* s, int64_t request_id, const int32_t* prompt_tokens, int32_t prompt_len,
                                          int32_t output_len) {
    if (!s || prompt_len < 1 || output_len < 1 || s->seqs.count(request_id)) return GLLM_E_INVALID;
    // a request that could never fit in the pool, even alone, is refused instead of blocking the queue for ever
    if (div_up((int64_t)prompt_len + output_len, kPageTokens) > s->p.total_pages) return GLLM_E_CAPACITY;
    s->admit(request_id, prompt_len, output_len, prompt_tokens);
    return GLLM_OK;
}

gllm_status gllm_sched_add_request(gllm_sched* s, int64_t request_id, int32_t prompt_len, int32_t output_len) {
    return gllm_sched_add_request_tokens(s, request_id, nullptr, prompt_len, output_len);
}

gllm_status gllm_sched_next_batch(gllm_sched* s, int64_t* batch_id, int64_t* request_ids, int32_t* new_tokens,
                                  int32_t* cached_len, int32_t capacity, int32_t* num_rows) {
    if (!s || !batch_id || !request_ids || !new_tokens || !cached_len || !num_rows || capacity < 0) return GLLM_E_INVALID;
    // rows are bounded by the requests that exist; check before anything changes
    if ((int64_t)capacity < (int64_t)(s->idle_decode.size() + s->waiting.size())) return GLLM_E_CAPACITY;
    std::vector<Row> rows = s->plan();
    *num_rows = (int32_t)rows.size();
    *batch_id = -1;
    if (rows.empty()) return GLLM_OK;
    for (size_t i = 0; i < rows.size(); ++i) {
        request_ids[i] = rows[i].id;
        new_tokens[i] = rows[i].count;
        cached_len[i] = rows[i].cached;
    }
    *batch_id = s->launch(std::move(rows));
    return GLLM_OK;
}

gllm_status gllm_sched_batch_block_tables(const gllm_sched* s, int64_t batch_id, int32_t* block_tables, int32_t stride) {
    if (!s || !block_tables || stride < 1) return GLLM_E_INVALID;
    auto it = s->flying.find(batch_id);
    if (it == s->flying.end()) return GLLM_E_INVALID;
    for (const Row& r : it->second)
        if ((int64_t)s->seqs.at(r.id).pages.size() > stride) return GLLM_E_CAPACITY;
    size_t row = 0;
    for (const Row& r : it->second) {
        const std::vector<int32_t>& pg = s->seqs.at(r.id).pages;
        int32_t* dst = block_tables + row * (size_t)stride;
        std::copy(pg.begin(), pg.end(), dst);
        std::fill(dst + pg.size(), dst + stride, -1);
        ++row;
    }
    return GLLM_OK;
}

gllm_status gllm_sched_complete_batch(gllm_sched* s, int64_t batch_id, int64_t* finished_ids, int32_t capacity,
                                      int32_t* num_finished) {
    return gllm_sched_complete_batch_tokens(s, batch_id, nullptr, 0, finished_ids, capacity, num_finished);
}

gllm_status gllm_sched_complete_batch_tokens(gllm_sched* s, int64_t batch_id, const int32_t* row_tokens, int32_t num_rows,
                                             int64_t* finished_ids, int32_t capacity, int32_t* num_finished) {
    if (!s || !num_finished || capacity < 0 || (capacity > 0 && !finished_ids)) return GLLM_E_INVALID;
    auto it = s->flying.find(batch_id);
    if (it == s->flying.end()) return GLLM_E_INVALID;
    if (row_tokens && (size_t)num_rows != it->second.size()) return GLLM_E_INVALID;
    if ((size_t)capacity < it->second.size()) return GLLM_E_CAPACITY;
    const std::vector<int64_t> ended = s->retire(batch_id, row_tokens);
    std::copy(ended.begin(), ended.end(), finished_ids);
    *num_finished = (int32_t)ended.size();
    return GLLM_OK;
}

gllm_status gllm_sched_get_state(const gllm_sched* s, gllm_sched_state* out) {
    if (!s || !out) return GLLM_E_INVALID;
    out->tokens_waiting = s->waiting_tokens;
    out->decode_requests = s->decode_total;
    out->free_pages = s->spare();
    out->batches_in_flight = (int64_t)s->flying.size();
    out->waiting_requests = (int64_t)s->waiting.size();
    out->preemptions = s->preempted;
    out->idle_cached_pages = s->pool.idle_cached();
    out->prefix_hit_tokens = s->hit_tokens;
    out->evictions = s->pool.evictions();
    return GLLM_OK;
}

gllm_status gllm_sched_simulate(const gllm_sched_params* p, const gllm_stage_time_model* model,
                                const int64_t* arrival_ns, const int32_t* prompt_len, const int32_t* output_len,
                                int64_t num_requests, gllm_sim_result* out) {
    return gllm_sched_simulate_tokens(p, model, arrival_ns, prompt_len, output_len, nullptr, num_requests, out);
}

gllm_status gllm_sched_simulate_tokens(const gllm_sched_params* p, const gllm_stage_time_model* model,
                                       const int64_t* arrival_ns, const int32_t* prompt_len, const int32_t* output_len,
                                       const int32_t* prompt_tokens, int64_t num_requests, gllm_sim_result* out) {
    if (!params_ok(p) || !model || !arrival_ns || !prompt_len || !output_len || !out || num_requests < 1)
        return GLLM_E_INVALID;
    for (int64_t i = 0; i < num_requests; ++i) {
        if (prompt_len[i] < 1 || output_len[i] < 1 || arrival_ns[i] < 0 || (i > 0 && arrival_ns[i] < arrival_ns[i - 1]))
            return GLLM_E_INVALID;
        if (div_up((int64_t)prompt_len[i] + output_len[i], kPageTokens) > p->total_pages) return GLLM_E_CAPACITY;
    }
    gllm_sched sch(*p);
    const int depth = p->pp_depth;
    int64_t token_cursor = 0;  // start of the next arriving prompt in prompt_tokens
    std::vector<int64_t> stage_free((size_t)depth, 0), first_token((size_t)num_requests, -1), ended_at((size_t)num_requests, -1);
    std::vector<std::pair<int64_t, int64_t>> landing;  // (time the micro-batch leaves the last stage, batch id), ascending
    int64_t busy_last = 0, clock = 0, arrived = 0, ended = 0, batches = 0, token_sum = 0;
    std::vector<int64_t> batch_tokens;
    while (true) {
        for (; arrived < num_requests && arrival_ns[arrived] <= clock; ++arrived) {
            sch.admit(arrived, prompt_len[arrived], output_len[arrived], prompt_tokens ? prompt_tokens + token_cursor : nullptr);
            token_cursor += prompt_len[arrived];
        }
        while (!landing.empty() && landing.front().first <= clock) {
            const int64_t t = landing.front().first, b = landing.front().second;
            landing.erase(landing.begin());
            const std::vector<Row> rows = sch.flying.at(b);
            for (int64_t id : sch.retire(b)) {
                ended_at[(size_t)id] = t;
                ++ended;
            }
            for (const Row& r : rows) {  // the chunk that completes a prompt yields the first token
                const Seq& q = sch.seqs.at(r.id);
                if (!r.decode && first_token[(size_t)r.id] < 0 && q.prefilled >= q.prompt) first_token[(size_t)r.id] = t;
            }
        }
        if (ended >= num_requests) break;
        if (stage_free[0] <= clock) {
            std::vector<Row> rows = sch.plan();
            if (!rows.empty()) {
                int64_t dt = model->base_ns, pairs = 0, tokens = 0;
                for (const Row& r : rows) {
                    dt += (int64_t)r.count * model->token_ns;
                    tokens += r.count;
                    if (r.count == 1) dt += ((int64_t)r.cached + 1) * model->decode_ctx_ns;
                    else pairs += (int64_t)r.count * r.cached + (int64_t)r.count * (r.count + 1) / 2;
                }
                dt += pairs * model->prefill_pair_ns_per_1024 / 1024;
                int64_t t = clock;
                for (int s = 0; s < depth; ++s) {
                    t = std::max(t, stage_free[(size_t)s]) + dt;
                    stage_free[(size_t)s] = t;
                }
                busy_last += dt;
                const int64_t b = sch.launch(std::move(rows));
                landing.insert(std::upper_bound(landing.begin(), landing.end(), std::make_pair(t, b)), std::make_pair(t, b));
                batch_tokens.push_back(tokens);
                token_sum += tokens;
                ++batches;
                continue;
            }
        }
        int64_t next = kNoLimit;
        if (arrived < num_requests && arrival_ns[arrived] > clock) next = std::min(next, arrival_ns[arrived]);
        if (!landing.empty() && landing.front().first > clock) next = std::min(next, landing.front().first);
        if (stage_free[0] > clock) next = std::min(next, stage_free[0]);
        if (next == kNoLimit) return GLLM_E_STATE;  // nothing in flight, nothing schedulable, nothing arriving
        clock = next;
    }
    int64_t end = 0, ttft = 0, e2e = 0;
    for (int64_t i = 0; i < num_requests; ++i) {
        end = std::max(end, ended_at[(size_t)i]);
        ttft += first_token[(size_t)i] - arrival_ns[i];
        e2e += ended_at[(size_t)i] - arrival_ns[i];
    }
    const int64_t mean_k = token_sum * 1000 / batches;
    // the squared deviations are summed in 128 bits: a batch of 4000 tokens contributes (4e6)^2
    __int128 acc = 0;
    for (int64_t b : batch_tokens) {
        const __int128 d = (__int128)1000 * b - mean_k;
        acc += d * d;
    }
    out->end_ns = end;
    out->batches = batches;
    out->tokens = token_sum;
    out->busy_ns_last_stage = busy_last;
    out->bubble_ppm_last_stage = (int64_t)((__int128)(end - busy_last) * 1000000 / end);
    out->mean_batch_tokens_x1000 = mean_k;
    out->var_batch_tokens_x1000 = (int64_t)(acc / batches / 1000);
    out->sum_ttft_ns = ttft;
    out->sum_e2e_ns = e2e;
    out->preemptions = sch.preempted;
    out->prefix_hit_tokens = sch.hit_tokens;
    return GLLM_OK;
}

}  // extern "C"
