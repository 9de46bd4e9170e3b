// Example-based drafter of the paper's Sec. 4.3: a per-query n-gram lookup table built from one
// token stream (few-shot examples followed by the user query) and the draft generation that
// indexes it with the n-1 most recent tokens.  Pure host code, O(stream length) to build.
#pragma once

#include <cstdint>
#include <unordered_map>
#include <vector>

namespace ax {

inline uint64_t splitmix64(uint64_t x) {          // output function of the splitmix64 generator
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct NgramLut {
    int n = 3;                                    // window length; keys are n-1 tokens
    int vocab = 0;
    // key -> id of the key; values[id] = most frequent next token
    struct KeyHash {
        size_t operator()(const std::vector<int32_t>& k) const {
            uint64_t h = 0x243F6A8885A308D3ull;
            for (int32_t t : k) h = splitmix64(h ^ (uint32_t)t);
            return (size_t)h;
        }
    };
    std::unordered_map<std::vector<int32_t>, int32_t, KeyHash> table;

    void build(const int32_t* stream, int64_t len, int n_, int vocab_) {
        n = n_;
        vocab = vocab_;
        table.clear();
        // per key: next tokens in first-recorded order with their counts
        struct Cand { int32_t tok; int64_t cnt; };
        std::unordered_map<std::vector<int32_t>, std::vector<Cand>, KeyHash> counts;
        std::vector<int32_t> key((size_t)(n - 1));
        for (int64_t i = 0; i + n <= len; ++i) {
            for (int j = 0; j < n - 1; ++j) key[(size_t)j] = stream[i + j];
            const int32_t nxt = stream[i + n - 1];
            auto& c = counts[key];
            bool found = false;
            for (auto& e : c)
                if (e.tok == nxt) { ++e.cnt; found = true; break; }
            if (!found) c.push_back({nxt, 1});
        }
        for (auto& kv : counts) {
            int32_t best = -1;
            int64_t best_n = 0;
            for (auto& e : kv.second)             // strict >: ties go to the earliest recorded
                if (e.cnt > best_n) { best = e.tok; best_n = e.cnt; }
            table.emplace(kv.first, best);
        }
    }

    // -1 on a miss (also when fewer than n-1 tokens of context exist)
    int32_t lookup(const int32_t* ctx_end, int64_t n_ctx) const {
        if (n_ctx < n - 1) return -1;
        std::vector<int32_t> key(ctx_end - (n - 1), ctx_end);
        auto it = table.find(key);
        return it == table.end() ? -1 : it->second;
    }

    // Up to k drafts after ctx (most recent token last; ctx is extended in place by the drafts
    // and restored).  Selective: nothing when the first lookup misses.  A later miss yields
    // splitmix64(seed + stream_pos + i) % vocab.  Returns the number of drafts, *hits the
    // number that came from the table.
    int draft(std::vector<int32_t>& ctx, int k, bool selective, uint64_t seed, int64_t stream_pos,
              int32_t* out, int* hits) const {
        const size_t base = ctx.size();
        int n_out = 0;
        *hits = 0;
        for (int i = 0; i < k; ++i) {
            int32_t tok = lookup(ctx.data() + ctx.size(), (int64_t)ctx.size());
            if (tok < 0) {
                if (i == 0 && selective) break;
                tok = (int32_t)(splitmix64(seed + (uint64_t)stream_pos + (uint64_t)i) % (uint64_t)vocab);
            } else {
                ++*hits;
            }
            out[n_out++] = tok;
            ctx.push_back(tok);
        }
        ctx.resize(base);
        return n_out;
    }
};

}  // namespace ax
