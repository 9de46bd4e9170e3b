// Host-only half of the C ABI: handle registry, paged-KV bookkeeping, prefix index, n-gram table
// and the offline combination selection.  No HIP call and no HIP header: this file also builds
// with a plain C++17 compiler (the CPU test-suite compiles it under AddressSanitizer).
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "cluster_select.h"
#include "handles.h"

namespace ax {

namespace {
thread_local char g_err[512] = "";
std::mutex g_reg_mu;
std::unordered_map<const void*, int>& registry() {
    static auto* r = new std::unordered_map<const void*, int>();   // never destroyed: handles may be freed at exit
    return *r;
}
}  // namespace

ax_status fail(ax_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

void handle_register(const void* h, HandleKind kind) {
    std::lock_guard<std::mutex> lk(g_reg_mu);
    registry()[h] = (int)kind;
}

void handle_unregister(const void* h) {
    std::lock_guard<std::mutex> lk(g_reg_mu);
    registry().erase(h);
}

bool handle_live(const void* h, HandleKind kind) {
    if (!h) return false;
    std::lock_guard<std::mutex> lk(g_reg_mu);
    auto it = registry().find(h);
    return it != registry().end() && it->second == (int)kind;
}

bool config_ok(const ax_model_config* c, ax_status* why) {
    *why = AX_ERR_INVALID;
    if (!c) return false;
    if (c->n_layers <= 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 ||
        c->head_dim <= 0 || c->d_ff <= 0 || c->vocab <= 0 || c->max_pos <= 0 ||
        c->max_tokens <= 0 || c->max_seqs <= 0)
        return false;
    if (c->n_q_heads % c->n_kv_heads != 0) return false;
    if (c->dtype != AX_F32 && c->dtype != AX_BF16) return false;
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return false;
    if (c->act_split < -1 || c->act_split > 1) return false;
    *why = AX_ERR_UNSUPPORTED;
    if (c->head_dim % 2 != 0 || c->head_dim > 256) return false;
    if (c->dtype == AX_BF16) {
        if (c->head_dim != 64 && c->head_dim != 128) return false;
        if (c->d_model % 64 || c->d_ff % 64 || c->vocab % 64) return false;
    }
    return true;
}

}  // namespace ax

using ax::fail;
using ax::ok;

extern "C" {

const char* ax_last_error(void) { return ax::g_err; }

// ---- paged KV pool ---------------------------------------------------------------------------

size_t ax_pool_block_bytes(const ax_model_config* cfg, int block_tokens) {
    ax_status why;
    if (!ax::config_ok(cfg, &why) || block_tokens <= 0) return 0;
    return (size_t)2 * cfg->n_layers * cfg->n_kv_heads * cfg->head_dim * block_tokens * ax::itemsize(cfg->dtype);
}

ax_status ax_pool_create(const ax_model_config* cfg, void* dev_mem, size_t bytes, int block_tokens,
                         ax_pool** out) {
    ax_status why;
    if (!out) return fail(AX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (!ax::config_ok(cfg, &why)) return fail(why, "model config rejected");
    if (block_tokens != 16) return fail(AX_ERR_UNSUPPORTED, "block_tokens must be 16");
    if (((uintptr_t)dev_mem & 255) != 0) return fail(AX_ERR_INVALID, "pool memory not 256-byte aligned");
    const size_t bb = ax_pool_block_bytes(cfg, block_tokens);
    const size_t nb = bytes / bb;
    if (nb < 1) return fail(AX_ERR_OOM, "pool of %zu bytes holds no %zu-byte block", bytes, bb);
    if (nb > 0x7fffffff) return fail(AX_ERR_INVALID, "too many blocks");
    ax_pool* p = new ax_pool();
    p->cfg = *cfg;
    p->geom.base = dev_mem;
    p->geom.n_blocks = (long long)nb;
    p->geom.n_kv_heads = cfg->n_kv_heads;
    p->geom.head_dim = cfg->head_dim;
    p->geom.block_tokens = block_tokens;
    p->blocks.init((int64_t)nb, block_tokens);
    static std::mutex uid_mu;
    static uint64_t next_uid = 1;
    {
        std::lock_guard<std::mutex> lk(uid_mu);
        p->uid = next_uid++;
    }
    ax::handle_register(p, ax::H_POOL);
    *out = p;
    return AX_OK;
}

ax_status ax_pool_destroy(ax_pool* p) {
    if (!ok(p)) return fail(AX_ERR_INVALID, "bad pool handle");
    if (p->blocks.live_seqs != 0) return fail(AX_ERR_STATE, "%lld sequences still alive", (long long)p->blocks.live_seqs);
    ax::handle_unregister(p);
    delete p;
    return AX_OK;
}

ax_status ax_pool_stats(const ax_pool* p, int64_t* free_blocks, int64_t* total_blocks, int64_t* live_seqs) {
    if (!ok(p)) return fail(AX_ERR_INVALID, "bad pool handle");
    if (free_blocks) *free_blocks = p->blocks.n_free();
    if (total_blocks) *total_blocks = p->blocks.n_total();
    if (live_seqs) *live_seqs = p->blocks.live_seqs;
    return AX_OK;
}

ax_status ax_kv_alloc(ax_pool* p, ax_kv** out) {
    if (!out) return fail(AX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (!ok(p)) return fail(AX_ERR_INVALID, "bad pool handle");
    ax_kv* k = new ax_kv();
    k->pool = p;
    ++p->blocks.live_seqs;
    ax::handle_register(k, ax::H_KV);
    *out = k;
    return AX_OK;
}

ax_status ax_kv_fork(const ax_kv* src, int64_t n_tokens, ax_kv** out) {
    if (!out) return fail(AX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (!ok(src)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (n_tokens < 0) n_tokens = src->seq.len;
    if (n_tokens > src->seq.len) return fail(AX_ERR_INVALID, "fork of %lld tokens from a sequence of %lld",
                                             (long long)n_tokens, (long long)src->seq.len);
    ax_kv* k = new ax_kv();
    k->pool = src->pool;
    ax::fork(src->pool->blocks, src->seq, n_tokens, k->seq);
    ++src->pool->blocks.live_seqs;
    ax::handle_register(k, ax::H_KV);
    *out = k;
    return AX_OK;
}

ax_status ax_kv_truncate(ax_kv* kv, int64_t new_len) {
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (new_len < 0 || new_len > kv->seq.len)
        return fail(AX_ERR_INVALID, "truncate to %lld, length is %lld", (long long)new_len, (long long)kv->seq.len);
    ax::truncate(kv->pool->blocks, kv->seq, new_len);
    return AX_OK;
}

int64_t ax_kv_len(const ax_kv* kv) { return ok(kv) ? kv->seq.len : -1; }

ax_status ax_kv_free(ax_kv* kv) {
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle (double free?)");
    ax::truncate(kv->pool->blocks, kv->seq, 0);
    --kv->pool->blocks.live_seqs;
    ax::handle_unregister(kv);
    delete kv;
    return AX_OK;
}

int64_t ax_kv_blocks(const ax_kv* kv, int32_t* ids, int64_t cap) {
    if (!ok(kv)) return -1;
    const int64_t n = (int64_t)kv->seq.blocks.size();
    if (ids) for (int64_t i = 0; i < n && i < cap; ++i) ids[i] = kv->seq.blocks[(size_t)i];
    return n;
}

int ax_pool_refcount(const ax_pool* p, int64_t block) {
    if (!ok(p) || block < 0 || block >= p->blocks.n_total()) return -1;
    return p->blocks.refcount[(size_t)block];
}

ax_status ax_kv_reserve_host(ax_kv* kv, int64_t n, int32_t* cow_src, int32_t* cow_dst) {
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (n <= 0 || !cow_src || !cow_dst) return fail(AX_ERR_INVALID, "bad argument");
    ax::BlockPool& bp = kv->pool->blocks;
    const ax::AppendPlan plan = ax::plan_append(bp, kv->seq, n);
    if (plan.need() > bp.n_free())
        return fail(AX_ERR_OOM, "need %lld KV blocks, %lld free", (long long)plan.need(), (long long)bp.n_free());
    ax::apply_append(bp, kv->seq, n, plan, cow_src, cow_dst);
    return AX_OK;
}

// ---- automatic prefix reuse and offline combination selection ----------------------------------

ax_status ax_index_create(ax_pool* pool, ax_index** out) {
    if (!out) return fail(AX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (!ok(pool)) return fail(AX_ERR_INVALID, "bad pool handle");
    ax_index* x = new ax_index();
    x->pool = pool;
    ax::handle_register(x, ax::H_INDEX);
    *out = x;
    return AX_OK;
}

void ax_index_destroy(ax_index* x) {
    if (!ax::handle_live(x, ax::H_INDEX)) return;
    for (auto& e : x->idx.entries)
        if (e.live) ax_kv_free((ax_kv*)e.owner);          // a no-op for handles that are gone already
    ax::handle_unregister(x);
    delete x;
}

int64_t ax_index_entries(const ax_index* x) {
    if (!ok(x)) return -1;
    int64_t n = 0;
    for (auto& e : x->idx.entries) n += e.live ? 1 : 0;
    return n;
}

ax_status ax_index_insert(ax_index* x, const ax_kv* kv, const int32_t* tokens, int64_t n) {
    if (!ok(x)) return fail(AX_ERR_INVALID, "bad index handle");
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (kv->pool != x->pool) return fail(AX_ERR_INVALID, "sequence lives in another pool");
    if (n <= 0 || !tokens) return fail(AX_ERR_INVALID, "bad argument");
    if (n > kv->seq.len) return fail(AX_ERR_INVALID, "%lld tokens given, the sequence holds %lld", (long long)n, (long long)kv->seq.len);
    ax_kv* held = nullptr;
    ax_status st = ax_kv_fork(kv, n, &held);
    if (st != AX_OK) return st;
    x->idx.insert(tokens, n, held);
    return AX_OK;
}

ax_status ax_index_match(ax_index* x, const int32_t* prompt, int64_t n, int64_t max_reuse, ax_kv** out, int64_t* matched) {
    if (!out || !matched) return fail(AX_ERR_INVALID, "NULL argument");
    *out = nullptr;
    *matched = 0;
    if (!ok(x)) return fail(AX_ERR_INVALID, "bad index handle");
    if (n < 0 || (n > 0 && !prompt)) return fail(AX_ERR_INVALID, "bad argument");
    int64_t m = 0;
    const int id = x->idx.match(prompt, n, &m);
    if (max_reuse >= 0 && m > max_reuse) m = max_reuse;
    if (id < 0 || m == 0) return ax_kv_alloc(x->pool, out);
    ax_status st = ax_kv_fork((const ax_kv*)x->idx.entries[(size_t)id].owner, m, out);
    if (st == AX_OK) *matched = m;
    return st;
}

}  // extern "C"

namespace {
bool unpack_seqs(const int32_t* concat, const int32_t* len, int64_t n, std::vector<ax::ClusterSeq>& out) {
    if (n < 0 || (n > 0 && (!concat || !len))) return false;
    const int32_t* at = concat;
    for (int64_t i = 0; i < n; ++i) {
        if (len[i] < 0) return false;
        out.emplace_back(at, at + len[i]);
        at += len[i];
    }
    return true;
}
}  // namespace

extern "C" {

ax_status ax_select_combinations(const int32_t* samples_concat, const int32_t* sample_len, int64_t n_samples, int budget,
                                 int32_t* chosen_concat, int64_t chosen_cap, int32_t* chosen_len,
                                 int64_t* coverage_after, int* n_chosen) {
    if (!n_chosen || budget < 0) return fail(AX_ERR_INVALID, "bad argument");
    *n_chosen = 0;
    std::vector<ax::ClusterSeq> samples;
    if (!unpack_seqs(samples_concat, sample_len, n_samples, samples)) return fail(AX_ERR_INVALID, "bad sample list");
    const ax::SelectionResult r = ax::select_combinations(samples, budget);
    int64_t total = 0;
    for (auto& c : r.chosen) total += (int64_t)c.size();
    if (!r.chosen.empty() && (!chosen_concat || !chosen_len || total > chosen_cap))
        return fail(AX_ERR_INVALID, "output holds %lld cluster ids, %lld needed", (long long)chosen_cap, (long long)total);
    int32_t* at = chosen_concat;
    for (size_t i = 0; i < r.chosen.size(); ++i) {
        chosen_len[i] = (int32_t)r.chosen[i].size();
        for (int32_t c : r.chosen[i]) *at++ = c;
        if (coverage_after) coverage_after[i] = r.coverage[i];
    }
    *n_chosen = (int)r.chosen.size();
    return AX_OK;
}

int64_t ax_coverage(const int32_t* samples_concat, const int32_t* sample_len, int64_t n_samples,
                    const int32_t* cached_concat, const int32_t* cached_len, int64_t n_cached) {
    std::vector<ax::ClusterSeq> samples, cached;
    if (!unpack_seqs(samples_concat, sample_len, n_samples, samples) || !unpack_seqs(cached_concat, cached_len, n_cached, cached))
        return -1;
    return ax::coverage(samples, cached);
}

// ---- example-based drafter ---------------------------------------------------------------------

ax_status ax_lut_build(const int32_t* stream, int64_t n_tokens, int n, int vocab, ax_lut** out) {
    if (!out) return fail(AX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (n < 1 || vocab <= 0 || n_tokens < 0 || (n_tokens > 0 && !stream)) return fail(AX_ERR_INVALID, "bad argument");
    for (int64_t i = 0; i < n_tokens; ++i)
        if (stream[i] < 0 || stream[i] >= vocab) return fail(AX_ERR_INVALID, "token %d outside the vocabulary", stream[i]);
    ax_lut* l = new ax_lut();
    l->lut.build(stream, n_tokens, n, vocab);
    ax::handle_register(l, ax::H_LUT);
    *out = l;
    return AX_OK;
}

void ax_lut_free(ax_lut* lut) {
    if (!ok(lut)) return;
    ax::handle_unregister(lut);
    delete lut;
}

int64_t ax_lut_size(const ax_lut* lut) { return ok(lut) ? (int64_t)lut->lut.table.size() : -1; }

int ax_lut_draft(const ax_lut* lut, const int32_t* context, int64_t n_context, int k, int selective, uint64_t seed,
                 int64_t stream_pos, int32_t* drafts, int* hits) {
    if (!ok(lut) || k < 0 || n_context < 0 || (n_context > 0 && !context) || (k > 0 && !drafts)) return -1;
    std::vector<int32_t> ctx(context, context + n_context);
    int h = 0;
    const int n = lut->lut.draft(ctx, k, selective != 0, seed, stream_pos, drafts, &h);
    if (hits) *hits = h;
    return n;
}

}  // extern "C"
