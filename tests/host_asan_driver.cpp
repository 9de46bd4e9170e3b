// Driver for the host-only half of the C ABI (handle registry, paged-KV bookkeeping, prefix index,
// n-gram table, combination selection), built by tests/test_host_sanitizers.py together with
// csrc/ax_host.cpp under AddressSanitizer + UndefinedBehaviorSanitizer.  It goes through every
// misuse the header promises to reject (double free, use after free, foreign pointers) and through
// random alloc / append / fork / truncate / free traces checked against a copy-everything model;
// any invalid memory access aborts the process, any wrong answer returns non-zero.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <random>
#include <vector>

#include "../include/agentx.h"

static int g_fail = 0;
#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) { std::fprintf(stderr, "%s:%d: CHECK(%s) failed\n", __FILE__, __LINE__, #cond); ++g_fail; } \
    } while (0)

static ax_model_config tiny_config() {
    ax_model_config c{};
    c.n_layers = 2; c.d_model = 256; c.n_q_heads = 4; c.n_kv_heads = 2; c.head_dim = 64; c.d_ff = 688; c.vocab = 4096;
    c.rms_eps = 1e-5f; c.rope_base = 10000.f; c.dtype = AX_F32; c.max_pos = 1 << 20; c.max_tokens = 64; c.max_seqs = 1;
    return c;
}

static ax_pool* make_pool(int n_blocks) {
    ax_model_config c = tiny_config();
    ax_pool* p = nullptr;
    CHECK(ax_pool_create(&c, nullptr, ax_pool_block_bytes(&c, 16) * (size_t)n_blocks, 16, &p) == AX_OK);
    return p;
}

static void bad_handles() {
    ax_pool* pool = make_pool(64);
    ax_kv* kv = nullptr;
    CHECK(ax_kv_alloc(pool, &kv) == AX_OK);
    CHECK(ax_kv_free(kv) == AX_OK);
    CHECK(ax_kv_free(kv) == AX_ERR_INVALID);                     // double free: the freed object is never read
    CHECK(ax_kv_len(kv) == -1);
    CHECK(ax_kv_truncate(kv, 0) == AX_ERR_INVALID);
    CHECK(ax_kv_blocks(kv, nullptr, 0) == -1);
    ax_kv* out = (ax_kv*)0x1;
    CHECK(ax_kv_fork(kv, -1, &out) == AX_ERR_INVALID && out == nullptr);
    CHECK(ax_kv_alloc(nullptr, &out) == AX_ERR_INVALID);
    int on_stack = 7;                                            // a pointer that never was a handle
    CHECK(ax_kv_len((const ax_kv*)&on_stack) == -1);
    CHECK(ax_kv_free((ax_kv*)&on_stack) == AX_ERR_INVALID);
    CHECK(ax_pool_stats((const ax_pool*)&on_stack, nullptr, nullptr, nullptr) == AX_ERR_INVALID);
    CHECK(ax_kv_alloc((ax_pool*)kv, &out) == AX_ERR_INVALID);     // a handle of the wrong kind (and stale)

    ax_kv* live = nullptr;
    CHECK(ax_kv_alloc(pool, &live) == AX_OK);
    CHECK(ax_kv_alloc((ax_pool*)live, &out) == AX_ERR_INVALID);   // live handle of the wrong kind
    CHECK(ax_pool_destroy(pool) == AX_ERR_STATE);                 // sequences alive: nothing destroyed
    int64_t fr = 0, tot = 0, ls = 0;
    CHECK(ax_pool_stats(pool, &fr, &tot, &ls) == AX_OK && fr == 64 && tot == 64 && ls == 1);
    CHECK(ax_kv_free(live) == AX_OK);
    CHECK(ax_pool_destroy(pool) == AX_OK);
    CHECK(ax_pool_destroy(pool) == AX_ERR_INVALID);               // destroyed twice
    CHECK(ax_pool_refcount(pool, 0) == -1);
    CHECK(ax_kv_alloc(pool, &out) == AX_ERR_INVALID);             // use after destroy

    // an index over a pool: destroying the index releases its references; stale index handles are ignored
    pool = make_pool(64);
    ax_index* idx = nullptr;
    CHECK(ax_index_create(pool, &idx) == AX_OK);
    CHECK(ax_kv_alloc(pool, &kv) == AX_OK);
    int32_t cs, cd;
    CHECK(ax_kv_reserve_host(kv, 40, &cs, &cd) == AX_OK);
    std::vector<int32_t> toks(40);
    for (int i = 0; i < 40; ++i) toks[(size_t)i] = i * 3 % 17;
    CHECK(ax_index_insert(idx, kv, toks.data(), 40) == AX_OK);
    CHECK(ax_index_insert(idx, kv, toks.data(), 41) == AX_ERR_INVALID);
    CHECK(ax_kv_free(kv) == AX_OK);                               // the index keeps its own fork
    CHECK(ax_index_insert(idx, kv, toks.data(), 10) == AX_ERR_INVALID);
    CHECK(ax_index_entries(idx) == 1);
    CHECK(ax_pool_destroy(pool) == AX_ERR_STATE);
    ax_index_destroy(idx);
    ax_index_destroy(idx);                                        // twice: ignored
    CHECK(ax_index_entries(idx) == -1);
    int64_t matched = -1;
    CHECK(ax_index_match(idx, toks.data(), 40, -1, &out, &matched) == AX_ERR_INVALID);
    CHECK(ax_pool_destroy(pool) == AX_OK);

    ax_lut* lut = nullptr;
    const int32_t stream[] = {1, 2, 3, 1, 2, 4, 1, 2, 3};
    CHECK(ax_lut_build(stream, 9, 3, 16, &lut) == AX_OK);
    CHECK(ax_lut_size(lut) > 0);
    ax_lut_free(lut);
    ax_lut_free(lut);                                             // twice: ignored
    CHECK(ax_lut_size(lut) == -1);
    int32_t d[4];
    CHECK(ax_lut_draft(lut, stream, 9, 4, 1, 0, 0, d, nullptr) == -1);
    CHECK(std::strlen(ax_last_error()) > 0);
}

// Random traces: refcount of a block == number of sequences holding it, the free count is
// conserved, a block is written only while it has one owner, and every cell a sequence can read
// holds what the copy-everything model says.
static void random_traces(unsigned seed) {
    const int NB = 96, B = 16;
    std::mt19937 rng(seed);
    ax_pool* pool = make_pool(NB);
    struct Seq { ax_kv* h; std::vector<int> cells; };
    std::vector<Seq> seqs;
    std::map<std::pair<int, int>, int> content;
    int tag = 0;
    auto blocks_of = [&](ax_kv* h) {
        const int64_t n = ax_kv_blocks(h, nullptr, 0);
        std::vector<int32_t> ids((size_t)std::max<int64_t>(n, 1));
        ax_kv_blocks(h, ids.data(), n);
        ids.resize((size_t)n);
        return ids;
    };
    for (int step = 0; step < 600; ++step) {
        const int op = (int)(rng() % 10);
        if (op == 0 || seqs.empty()) {
            ax_kv* h = nullptr;
            CHECK(ax_kv_alloc(pool, &h) == AX_OK);
            seqs.push_back({h, {}});
        } else if (op <= 4) {
            Seq& s = seqs[rng() % seqs.size()];
            const int n = 1 + (int)(rng() % 39);
            int64_t free_before = 0;
            ax_pool_stats(pool, &free_before, nullptr, nullptr);
            const int64_t len_before = ax_kv_len(s.h);
            int32_t src, dst;
            const ax_status st = ax_kv_reserve_host(s.h, n, &src, &dst);
            if (st != AX_OK) {
                int64_t free_after = 0;
                ax_pool_stats(pool, &free_after, nullptr, nullptr);
                CHECK(st == AX_ERR_OOM && free_after == free_before && ax_kv_len(s.h) == len_before);
                continue;
            }
            if (src >= 0)
                for (int sl = 0; sl < B; ++sl) {
                    auto it = content.find({src, sl});
                    if (it != content.end()) content[{dst, sl}] = it->second;
                }
            const std::vector<int32_t> ids = blocks_of(s.h);
            for (int i = 0; i < n; ++i) {
                const int pos = (int)s.cells.size();
                s.cells.push_back(++tag);
                const int blk = ids[(size_t)(pos / B)];
                CHECK(ax_pool_refcount(pool, blk) == 1);
                content[{blk, pos % B}] = tag;
            }
        } else if (op <= 6) {
            const Seq& s = seqs[rng() % seqs.size()];
            const int n = (int)(rng() % (s.cells.size() + 1));
            ax_kv* h = nullptr;
            CHECK(ax_kv_fork(s.h, n, &h) == AX_OK);
            seqs.push_back({h, std::vector<int>(s.cells.begin(), s.cells.begin() + n)});
        } else if (op <= 8) {
            Seq& s = seqs[rng() % seqs.size()];
            const int n = (int)(rng() % (s.cells.size() + 1));
            CHECK(ax_kv_truncate(s.h, n) == AX_OK);
            s.cells.resize((size_t)n);
        } else {
            const size_t i = rng() % seqs.size();
            CHECK(ax_kv_free(seqs[i].h) == AX_OK);
            CHECK(ax_kv_free(seqs[i].h) == AX_ERR_INVALID);
            seqs.erase(seqs.begin() + (long)i);
        }
        std::vector<int> held((size_t)NB, 0);
        for (const Seq& s : seqs) {
            const std::vector<int32_t> ids = blocks_of(s.h);
            CHECK(ax_kv_len(s.h) == (int64_t)s.cells.size());
            CHECK(ids.size() == (s.cells.size() + B - 1) / B);
            for (int32_t b : ids) ++held[(size_t)b];
            for (size_t pos = 0; pos < s.cells.size(); ++pos)
                CHECK((content[{ids[pos / B], (int)(pos % B)}] == s.cells[pos]));
        }
        int used = 0;
        for (int b = 0; b < NB; ++b) {
            CHECK(ax_pool_refcount(pool, b) == held[(size_t)b]);
            used += held[(size_t)b] > 0;
        }
        int64_t fr = 0, tot = 0, ls = 0;
        CHECK(ax_pool_stats(pool, &fr, &tot, &ls) == AX_OK);
        CHECK(fr == NB - used && tot == NB && ls == (int64_t)seqs.size());
    }
    for (Seq& s : seqs) CHECK(ax_kv_free(s.h) == AX_OK);
    int64_t fr = 0;
    ax_pool_stats(pool, &fr, nullptr, nullptr);
    CHECK(fr == NB);
    CHECK(ax_pool_destroy(pool) == AX_OK);
}

// Prefix index, hand-worked: three cached sequences; the answers follow from comparing tokens by eye.
static void prefix_index() {
    ax_pool* pool = make_pool(64);
    ax_index* idx = nullptr;
    CHECK(ax_index_create(pool, &idx) == AX_OK);
    auto cached = [&](const std::vector<int32_t>& t) {
        ax_kv* kv = nullptr;
        int32_t cs, cd;
        CHECK(ax_kv_alloc(pool, &kv) == AX_OK);
        CHECK(ax_kv_reserve_host(kv, (int64_t)t.size(), &cs, &cd) == AX_OK);
        CHECK(ax_index_insert(idx, kv, t.data(), (int64_t)t.size()) == AX_OK);
        CHECK(ax_kv_free(kv) == AX_OK);
    };
    std::vector<int32_t> a(50), b(50), c(20);
    for (int i = 0; i < 50; ++i) { a[(size_t)i] = 100 + i; b[(size_t)i] = 100 + i; }
    b[37] = 7;                                     // a and b agree on tokens 0..36
    for (int i = 0; i < 20; ++i) c[(size_t)i] = 500 + i;
    cached(a); cached(b); cached(c);
    auto match = [&](const std::vector<int32_t>& p, int64_t max_reuse) {
        ax_kv* out = nullptr;
        int64_t m = -1;
        CHECK(ax_index_match(idx, p.data(), (int64_t)p.size(), max_reuse, &out, &m) == AX_OK);
        CHECK(out != nullptr && ax_kv_len(out) == m);
        CHECK(ax_kv_free(out) == AX_OK);
        return m;
    };
    CHECK(match(a, -1) == 50);                     // full match
    CHECK(match(a, 49) == 49);                     // keep one token to run
    std::vector<int32_t> p = a;
    p[40] = 9;
    CHECK(match(p, -1) == 40);                     // first mismatch at 40 (entry a)
    p = b;
    p.resize(45);
    CHECK(match(p, -1) == 45);                     // shorter than the entry: the tail is cut
    p = a;
    p[0] = 1;
    CHECK(match(p, -1) == 0);                      // mismatch at position 0: nothing reused
    CHECK(match(std::vector<int32_t>{500, 501, 502, 9}, -1) == 3);
    CHECK(match(std::vector<int32_t>{}, -1) == 0);
    ax_index_destroy(idx);
    int64_t fr = 0;
    ax_pool_stats(pool, &fr, nullptr, nullptr);
    CHECK(fr == 64);
    CHECK(ax_pool_destroy(pool) == AX_OK);
}

static void lut_and_selection() {
    // window of 3 over 1 2 3 1 2 4 1 2 3: key (1,2) -> 3 twice, 4 once; (2,3) -> 1; (3,1) -> 2; (2,4) -> 1; (4,1) -> 2
    const int32_t stream[] = {1, 2, 3, 1, 2, 4, 1, 2, 3};
    ax_lut* lut = nullptr;
    CHECK(ax_lut_build(stream, 9, 3, 16, &lut) == AX_OK);
    CHECK(ax_lut_size(lut) == 5);
    const int32_t ctx[] = {9, 1, 2};
    int32_t d[6];
    int hits = -1;
    CHECK(ax_lut_draft(lut, ctx, 3, 6, 1, 0, 0, d, &hits) == 6 && hits == 6);
    const int32_t want[] = {3, 1, 2, 3, 1, 2};
    CHECK(std::memcmp(d, want, sizeof want) == 0);
    const int32_t miss[] = {9, 9};
    CHECK(ax_lut_draft(lut, miss, 2, 4, 1, 0, 0, d, &hits) == 0 && hits == 0);       // selective: first lookup misses
    CHECK(ax_lut_draft(lut, miss, 2, 4, 0, 5, 0, d, &hits) == 4);                    // non-selective: guesses
    for (int i = 0; i < 4; ++i) CHECK(d[i] >= 0 && d[i] < 16);
    CHECK(ax_lut_draft(lut, miss, 1, 4, 1, 0, 0, d, &hits) == 0);                    // shorter context than a key
    const int32_t bad[] = {1, 99};
    ax_lut* none = (ax_lut*)0x1;
    CHECK(ax_lut_build(bad, 2, 3, 16, &none) == AX_ERR_INVALID && none == nullptr);
    ax_lut_free(lut);

    // samples over clusters; prefix (1) covers 3 samples, (1,3) two of them, (2) one
    const int32_t samples[] = {1, 3, 2, /**/ 1, 3, /**/ 1, /**/ 2};
    const int32_t lens[] = {3, 2, 1, 1};
    int32_t chosen[16], chosen_len[4];
    int64_t cov[4];
    int n = -1;
    CHECK(ax_select_combinations(samples, lens, 4, 3, chosen, 16, chosen_len, cov, &n) == AX_OK);
    CHECK(n == 3 && chosen_len[0] == 1 && chosen[0] == 1 && cov[0] == 3);
    CHECK(chosen_len[1] == 2 && chosen[1] == 1 && chosen[2] == 3 && cov[1] == 5);
    CHECK(cov[2] == 6);                                                              // (1,3,2) and (2) both add 1: (1,3,2) is smaller
    CHECK(chosen_len[2] == 3);
    CHECK(ax_select_combinations(samples, lens, 4, 3, chosen, 2, chosen_len, cov, &n) == AX_ERR_INVALID);
    const int32_t cached[] = {1, 1, 3};
    const int32_t cached_len[] = {1, 2};
    CHECK(ax_coverage(samples, lens, 4, cached, cached_len, 2) == 5);
    CHECK(ax_coverage(samples, lens, 4, nullptr, nullptr, 0) == 0);
    const int32_t neg[] = {-1};
    CHECK(ax_coverage(samples, neg, 1, nullptr, nullptr, 0) == -1);
}

int main() {
    bad_handles();
    for (unsigned seed = 0; seed < 4; ++seed) random_traces(seed);
    prefix_index();
    lut_and_selection();
    if (g_fail) { std::fprintf(stderr, "%d checks failed\n", g_fail); return 1; }
    std::puts("host driver: all checks passed");
    return 0;
}
