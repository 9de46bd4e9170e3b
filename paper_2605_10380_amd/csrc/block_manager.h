// Host-side paged KV bookkeeping: reference-counted fixed-size blocks shared between
// sequences with a common prefix (prefix caching, paper Sec. 2.3), tail cut (Sec. 4.2) and
// rollback of rejected drafts (Sec. 2.3).  Pure host code: it never calls HIP, so it can be
// unit-tested without a GPU and can never stall the device.
#pragma once

#include <cstdint>
#include <vector>

namespace ax {

struct BlockPool {
    int block_tokens = 16;
    std::vector<int32_t> refcount;   // per block
    std::vector<int32_t> free_list;  // stack; top = next block handed out
    int64_t live_seqs = 0;

    void init(int64_t n_blocks, int block_tokens_) {
        block_tokens = block_tokens_;
        refcount.assign((size_t)n_blocks, 0);
        free_list.resize((size_t)n_blocks);
        // hand blocks out in ascending order: a sequence built in one go gets consecutive
        // blocks, which makes its K/V stream contiguous in memory
        for (int64_t i = 0; i < n_blocks; ++i) free_list[(size_t)i] = (int32_t)(n_blocks - 1 - i);
    }
    int64_t n_free() const { return (int64_t)free_list.size(); }
    int64_t n_total() const { return (int64_t)refcount.size(); }
    int32_t take() {
        int32_t b = free_list.back();
        free_list.pop_back();
        refcount[(size_t)b] = 1;
        return b;
    }
    void share(int32_t b) { ++refcount[(size_t)b]; }
    void release(int32_t b) {
        if (--refcount[(size_t)b] == 0) free_list.push_back(b);
    }
};

struct Sequence {
    std::vector<int32_t> blocks;
    int64_t len = 0;
};

inline int64_t blocks_for(int64_t tokens, int block_tokens) {
    return (tokens + block_tokens - 1) / block_tokens;
}

// What an append of n positions needs from the pool.
struct AppendPlan {
    int64_t new_blocks = 0;   // blocks to add at the end
    bool cow = false;         // last block is shared and partly filled: replace it by a copy
    int64_t need() const { return new_blocks + (cow ? 1 : 0); }
};

inline AppendPlan plan_append(const BlockPool& pool, const Sequence& s, int64_t n) {
    AppendPlan p;
    const int B = pool.block_tokens;
    p.new_blocks = blocks_for(s.len + n, B) - (int64_t)s.blocks.size();
    if (p.new_blocks < 0) p.new_blocks = 0;
    if (n > 0 && s.len % B != 0) {
        int32_t last = s.blocks[(size_t)(s.len / B)];
        p.cow = pool.refcount[(size_t)last] > 1;
    }
    return p;
}

// Applies a plan that is known to fit.  Reports the copy-on-write pair (or -1, -1).
inline void apply_append(BlockPool& pool, Sequence& s, int64_t n, const AppendPlan& p,
                         int32_t* cow_src, int32_t* cow_dst) {
    *cow_src = *cow_dst = -1;
    const int B = pool.block_tokens;
    // a truncate may have left whole blocks beyond ceil(len/B) allocated; never the case here
    // because truncate releases them, so blocks.size() == ceil(len/B) on entry
    if (p.cow) {
        size_t idx = (size_t)(s.len / B);
        int32_t old = s.blocks[idx];
        int32_t fresh = pool.take();
        s.blocks[idx] = fresh;
        pool.release(old);
        *cow_src = old;
        *cow_dst = fresh;
    }
    for (int64_t i = 0; i < p.new_blocks; ++i) s.blocks.push_back(pool.take());
    s.len += n;
}

inline void truncate(BlockPool& pool, Sequence& s, int64_t new_len) {
    size_t keep = (size_t)blocks_for(new_len, pool.block_tokens);
    while (s.blocks.size() > keep) {
        pool.release(s.blocks.back());
        s.blocks.pop_back();
    }
    s.len = new_len;
}

inline void fork(BlockPool& pool, const Sequence& src, int64_t n_tokens, Sequence& dst) {
    size_t nb = (size_t)blocks_for(n_tokens, pool.block_tokens);
    dst.blocks.assign(src.blocks.begin(), src.blocks.begin() + (long)nb);
    for (int32_t b : dst.blocks) pool.share(b);
    dst.len = n_tokens;
}

}  // namespace ax
