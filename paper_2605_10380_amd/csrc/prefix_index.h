// Index of cached token sequences for automatic prefix reuse (paper Sec. 2.3 and 4.2: a new
// prompt reuses the cached KV up to the first mismatching token, the rest of the cached entry is
// cut off).  Host only.  Every 16-token block boundary of an inserted sequence is entered under a
// chained hash of the tokens up to it, so a lookup walks the prompt block by block in O(length),
// then compares token by token inside the entries that share the last matching block.
#pragma once

#include <algorithm>
#include <cstdint>
#include <unordered_map>
#include <vector>

namespace ax {

struct PrefixIndex {
    static constexpr int B = 16;
    struct Entry { std::vector<int32_t> tokens; void* owner; bool live; };
    std::vector<Entry> entries;
    std::unordered_map<uint64_t, std::vector<int32_t>> by_hash;   // chain hash after b blocks -> entries

    static uint64_t mix(uint64_t h, const int32_t* t, int n) {
        for (int i = 0; i < n; ++i) {
            h ^= (uint32_t)t[i] + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
            h *= 0xBF58476D1CE4E5B9ull;
            h ^= h >> 31;
        }
        return h;
    }

    int insert(const int32_t* tokens, int64_t n, void* owner) {
        const int id = (int)entries.size();
        entries.push_back({std::vector<int32_t>(tokens, tokens + n), owner, true});
        uint64_t h = 0x243F6A8885A308D3ull;
        by_hash[h].push_back(id);                                  // zero blocks: every entry
        for (int64_t b = 0; (b + 1) * B <= n; ++b) {
            h = mix(h, tokens + b * B, B);
            by_hash[h].push_back(id);
        }
        return id;
    }

    // Entry sharing the longest common prefix with the prompt (lowest id among equals) and that
    // length; -1 / 0 if nothing matches.
    int match(const int32_t* prompt, int64_t n, int64_t* matched) const {
        uint64_t h = 0x243F6A8885A308D3ull;
        const std::vector<int32_t>* last = nullptr;
        int64_t blocks = 0;
        auto it = by_hash.find(h);
        if (it != by_hash.end()) last = &it->second;
        for (int64_t b = 0; (b + 1) * B <= n; ++b) {
            h = mix(h, prompt + b * B, B);
            it = by_hash.find(h);
            if (it == by_hash.end()) break;
            bool any = false;                                      // guard against hash collisions
            for (int32_t id : it->second) {
                const Entry& e = entries[(size_t)id];
                if (e.live && std::equal(prompt, prompt + (b + 1) * B, e.tokens.begin())) { any = true; break; }
            }
            if (!any) break;
            last = &it->second;
            blocks = b + 1;
        }
        int best = -1;
        int64_t best_n = 0;
        if (last)
            for (int32_t id : *last) {
                const Entry& e = entries[(size_t)id];
                if (!e.live) continue;
                int64_t m = 0;
                const int64_t lim = std::min<int64_t>(n, (int64_t)e.tokens.size());
                while (m < lim && e.tokens[(size_t)m] == prompt[m]) ++m;
                if (m < blocks * B) continue;                      // collision: not a real match
                if (m > best_n) { best_n = m; best = id; }
            }
        *matched = best_n;
        return best;
    }
};

}  // namespace ax
