// KV page pool with prefix caching: host code shared by the C ABI of include/gllm_kv.h and by the scheduler.
// The paper (arxiv 2504.14775) hands the KV cache out in pages before a micro-batch runs (section 3.1, caption of
// the prefill case study), lets the driver worker manage it for all stages (section 3.3) and lists PagedAttention
// and prefix caching among the integrated techniques (section 3.4) without giving an algorithm; include/gllm_kv.h
// states the rules chosen here.  Callers check their arguments: the methods below assume them valid.
#pragma once

#include <cstddef>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>

namespace gllm {

class PagePool {
  public:
    static constexpr int kPageTokens = 16;
    static constexpr int32_t kRoot = -1;

    explicit PagePool(int64_t total)
        : total_(total), holders_((size_t)total, 0), kids_((size_t)total, 0), keyed_((size_t)total, 0),
          keys_((size_t)total), before_((size_t)total + 1), after_((size_t)total + 1) {
        free_.resize((size_t)total);
        for (int64_t i = 0; i < total; ++i) free_[(size_t)i] = (int32_t)(total - 1 - i);  // 0 is handed out first
        before_[(size_t)total] = after_[(size_t)total] = (int32_t)total;                   // empty ring around the sentinel
    }

    int64_t total() const { return total_; }
    int64_t free_count() const { return (int64_t)free_.size(); }
    int64_t idle_cached() const { return queued_; }
    int64_t available() const { return (int64_t)free_.size() + queued_; }
    int64_t registered() const { return (int64_t)index_.size(); }
    int64_t evictions() const { return evictions_; }
    int32_t holders(int32_t page) const { return holders_[(size_t)page]; }
    bool is_registered(int32_t page) const { return keyed_[(size_t)page] != 0; }
    int32_t children(int32_t page) const { return kids_[(size_t)page]; }

    // A page nobody holds: from the free stack, else the registered page that has waited longest.
    int32_t alloc() {
        int32_t page;
        if (!free_.empty()) {
            page = free_.back();
            free_.pop_back();
        } else {
            page = after_[(size_t)total_];
            unlink(page);
            const Key& k = keys_[(size_t)page];
            if (k.parent != kRoot) --kids_[(size_t)k.parent];
            index_.erase(k);
            keyed_[(size_t)page] = 0;
            ++evictions_;
        }
        holders_[(size_t)page] = 1;
        return page;
    }

    // Walks the tree along the whole pages of tokens[0 .. n), at most max_pages of them; every page found is
    // appended to `out` and gets one more holder.  Returns the number found.
    int64_t match(const int32_t* tokens, int64_t n, int64_t max_pages, std::vector<int32_t>& out) {
        const int64_t whole = n / kPageTokens, limit = whole < max_pages ? whole : max_pages;
        Key k;
        k.parent = kRoot;
        int64_t found = 0;
        for (; found < limit; ++found) {
            std::memcpy(k.tok, tokens + found * kPageTokens, sizeof k.tok);
            auto it = index_.find(k);
            if (it == index_.end()) break;
            const int32_t page = it->second;
            if (holders_[(size_t)page]++ == 0) unlink(page);
            out.push_back(page);
            k.parent = page;
        }
        return found;
    }

    // The page (held, not yet in the tree) becomes the node for these 16 tokens behind `parent`; false when that
    // node exists already.
    bool enter(int32_t parent, const int32_t* tokens16, int32_t page) {
        Key k;
        k.parent = parent;
        std::memcpy(k.tok, tokens16, sizeof k.tok);
        if (!index_.emplace(k, page).second) return false;
        keys_[(size_t)page] = k;
        keyed_[(size_t)page] = 1;
        if (parent != kRoot) ++kids_[(size_t)parent];
        return true;
    }

    // One holder less on each page of a block table.  Unregistered pages nobody holds any more go onto the free
    // stack in table order; registered ones to the back of the eviction queue, last table entry first, so that a
    // page always leaves the tree before the page it extends.
    void release(const int32_t* pages, size_t n) {
        for (size_t i = 0; i < n; ++i)
            if (--holders_[(size_t)pages[i]] == 0 && !keyed_[(size_t)pages[i]]) free_.push_back(pages[i]);
        for (size_t i = n; i-- > 0;)
            if (holders_[(size_t)pages[i]] == 0 && keyed_[(size_t)pages[i]]) link_back(pages[i]);
    }

  private:
    struct Key {
        int32_t parent;
        int32_t tok[kPageTokens];
        bool operator==(const Key& o) const { return parent == o.parent && std::memcmp(tok, o.tok, sizeof tok) == 0; }
    };
    struct KeyHash {
        size_t operator()(const Key& k) const {
            uint64_t h = 0x9E3779B97F4A7C15ull ^ (uint64_t)(uint32_t)k.parent;
            for (int i = 0; i < kPageTokens; ++i) {
                h ^= (uint64_t)(uint32_t)k.tok[i] + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
                h *= 0xD6E8FEB86659FD93ull;
            }
            return (size_t)(h ^ (h >> 32));
        }
    };

    void unlink(int32_t page) {
        const int32_t b = before_[(size_t)page], a = after_[(size_t)page];
        after_[(size_t)b] = a;
        before_[(size_t)a] = b;
        --queued_;
    }
    void link_back(int32_t page) {
        const int32_t s = (int32_t)total_, last = before_[(size_t)s];
        after_[(size_t)last] = page;
        before_[(size_t)page] = last;
        after_[(size_t)page] = s;
        before_[(size_t)s] = page;
        ++queued_;
    }

    int64_t total_, queued_ = 0, evictions_ = 0;
    std::vector<int32_t> free_;               // stack, the top is handed out next
    std::vector<int32_t> holders_, kids_;
    std::vector<uint8_t> keyed_;
    std::vector<Key> keys_;                   // of registered pages
    std::vector<int32_t> before_, after_;     // eviction queue as a ring through the sentinel index total_
    std::unordered_map<Key, int32_t, KeyHash> index_;
};

}  // namespace gllm
