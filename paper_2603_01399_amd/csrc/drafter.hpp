// Prompt-lookup n-gram drafter (host code, no GPU work): proposes the tokens that followed the
// most recent earlier occurrence of the last k context tokens, k from k_max down to k_min.
//
// The context only grows (prompt, then accepted tokens).  For every lookup length k the
// k-grams are indexed as they are completed: a bucket array keyed by a hash of the k tokens
// holds the most recent start, and a per-start link leads to the previous start of the same
// bucket.  A proposal hashes the last k tokens and walks that chain, newest first, comparing
// tokens (so hash collisions cost time, never correctness): O(k_max) per appended token and
// per proposal on typical text, instead of a scan of the whole context.
#pragma once

#include <cstdint>
#include <vector>

namespace quasar {

class NgramDrafter {
public:
    NgramDrafter(int k_min, int k_max, int64_t capacity_hint) : k_min_(k_min), k_max_(k_max) {
        size_t buckets = 1u << 12;
        while ((int64_t)buckets < 2 * capacity_hint && buckets < (size_t(1) << 28)) buckets <<= 1;
        heads_.assign(k_max_ - k_min_ + 1, std::vector<int64_t>(buckets, -1));
        links_.assign(k_max_ - k_min_ + 1, std::vector<int64_t>());
        if (capacity_hint > 0) tokens_.reserve((size_t)capacity_hint);
    }

    int64_t length() const { return (int64_t)tokens_.size(); }

    void append(const int32_t *t, int64_t n) {
        for (int64_t i = 0; i < n; ++i) {
            tokens_.push_back(t[i]);
            const int64_t len = (int64_t)tokens_.size();
            if ((size_t)len * 2 > heads_[0].size() && heads_[0].size() < (size_t(1) << 28)) grow();
            for (int k = k_min_; k <= k_max_; ++k)
                if (len >= k) insert(k, len - k);
        }
    }

    // Writes up to gamma tokens to out; returns their number, *k_used = lookup length (0: none).
    int64_t propose(int64_t gamma, int32_t *out, int *k_used) const {
        const int64_t n = (int64_t)tokens_.size();
        for (int k = k_max_; k >= k_min_; --k) {
            if (n < k + 1) continue;
            const int64_t p = n - k;                       // the pattern's own start (it is indexed too)
            const std::vector<int64_t> &head = heads_[k - k_min_];
            const std::vector<int64_t> &link = links_[k - k_min_];
            for (int64_t s = head[hash(p, k) & (head.size() - 1)]; s >= 0; s = link[s]) {
                if (s == p || !same(s, p, k)) continue;
                int64_t m = 0;
                for (int64_t j = s + k; j < n && m < gamma; ++j) out[m++] = tokens_[j];
                if (k_used) *k_used = k;
                return m;
            }
        }
        if (k_used) *k_used = 0;
        return 0;
    }

private:
    uint64_t hash(int64_t start, int k) const {
        uint64_t h = 0x9E3779B97F4A7C15ull;
        for (int j = 0; j < k; ++j) {
            h ^= (uint64_t)(uint32_t)tokens_[start + j];
            h *= 0xFF51AFD7ED558CCDull;
            h ^= h >> 29;
        }
        return h;
    }
    bool same(int64_t a, int64_t b, int k) const {
        for (int j = 0; j < k; ++j)
            if (tokens_[a + j] != tokens_[b + j]) return false;
        return true;
    }
    void insert(int k, int64_t start) {
        std::vector<int64_t> &head = heads_[k - k_min_];
        std::vector<int64_t> &link = links_[k - k_min_];
        const size_t b = hash(start, k) & (head.size() - 1);
        if ((int64_t)link.size() <= start) link.resize((size_t)start + 1, -1);
        link[start] = head[b];
        head[b] = start;
    }
    void grow() {
        const size_t buckets = heads_[0].size() * 4;
        const int64_t len = (int64_t)tokens_.size();
        for (int k = k_min_; k <= k_max_; ++k) {
            heads_[k - k_min_].assign(buckets, -1);
            links_[k - k_min_].clear();
            // every k-gram completed so far, oldest first, except the one the caller is about to add
            for (int64_t start = 0; start + k <= len - 1; ++start) insert(k, start);
        }
    }

    int k_min_, k_max_;
    std::vector<int32_t> tokens_;
    std::vector<std::vector<int64_t>> heads_, links_;
};

}  // namespace quasar
