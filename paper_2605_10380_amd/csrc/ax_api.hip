// GPU half of the C ABI: models, per-call descriptors and the kernel sequence of one extend
// forward, verification, KV images, the draft / verify loop and the test-only entries.  (Pool,
// sequence, index and table handles live in ax_host.cpp.)  No device memory is allocated here:
// weights, KV pool and workspace are borrowed from the caller.
#include "../../include/agentx.h"
#include "../../include/agentx_debug.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "handles.h"
#include "kernels.h"

namespace {

using ax::fail;
using ax::ok;

#define HIP_TRY(expr)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) return fail(AX_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// The two events of a timed region (test / benchmark entry points): destroyed on every way out.
struct TimerEvents {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t create() {
        hipError_t e = hipEventCreate(&a);
        return e == hipSuccess ? hipEventCreate(&b) : e;
    }
    ~TimerEvents() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

constexpr int N_SLOTS = 4;            // staging ring for per-call descriptors
constexpr int LOGIT_ROWS = 256;       // rows per LM-head pass when only the argmax is wanted
constexpr long long kSharedMinKeys = 2048;   // (sequences - 1) x shared keys that justify a shared-prefix pass
constexpr int SPLIT_ITEMS = 2048;     // partial records the split attention may use (workspace size)

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
int isz(int dtype) { return ax::itemsize(dtype); }

using ax::config_ok;

constexpr int GUARD_BYTES = 256;      // after every workspace region: a pattern no kernel may touch (ax_dbg_check_guards)
constexpr unsigned char GUARD_FILL = 0xA5;
constexpr int MAX_REGIONS = 24;

struct Layout {                       // byte offsets into the workspace
    size_t guard_at[MAX_REGIONS];     // where the guard behind region i starts (regions in the order they are taken below)
    int n_regions;
    size_t splitk_bytes;
    size_t rope_cos, rope_sin, desc, x, h, ssq, qkv, q, attn, ffn, partials, splitk, logits, amax_scratch,
        amax_out, result, packed, total;
    size_t desc_ints;                 // capacity of one descriptor slot
    size_t max_records;               // split-attention partial records one pass may write (there is room for two passes)
    int max_tiles, max_bt;
    // split activations: element offsets from the hi part of each 16-bit activation buffer to its lo part (0 = off)
    long long h_lo, q_lo, attn_lo, ffn_lo;
    size_t h_bytes, q_bytes, attn_bytes, ffn_bytes;    // sizes of the hi parts (what ax_dbg_read hands out)
};

size_t packed_weight_bytes(const ax_model_config& c) {
    const size_t qkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, qd = (size_t)c.n_q_heads * c.head_dim;
    const size_t per_layer = qkv * c.d_model + (size_t)c.d_model * qd + 3 * (size_t)c.d_ff * c.d_model;
    return align_up(((size_t)c.n_layers * per_layer + (size_t)c.vocab * c.d_model) * 2 + 256 * (5 * (size_t)c.n_layers + 1));
}

Layout make_layout(const ax_model_config& c) {
    Layout L{};
    const size_t T = (size_t)c.max_tokens, S = (size_t)c.max_seqs, a = (size_t)isz(c.dtype);
    const int G = c.n_q_heads / c.n_kv_heads;
    L.max_tiles = (int)((T * G + 31) / 32 + S + (T * G) / 128 + 2);     // per-sequence tiles + groups of a shared-prefix pass
    L.max_bt = (c.max_pos + 15) / 16;
    L.desc_ints = 5 * T + 4 * S + S * (size_t)L.max_bt + 8 * (size_t)L.max_tiles + 32;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes);
        L.guard_at[L.n_regions++] = o;
        o += GUARD_BYTES;
        return at;
    };
    L.rope_cos = take((size_t)c.max_pos * (c.head_dim / 2) * 4);
    L.rope_sin = take((size_t)c.max_pos * (c.head_dim / 2) * 4);
    L.desc = take((N_SLOTS + 1) * align_up(L.desc_ints * 4));   // ring + the slot of captured graphs
    const size_t parts = ax::act_split_on(c) ? 2 : 1;         // hi part, then (split activations) the lo part
    const size_t qdim = (size_t)c.n_q_heads * c.head_dim;
    L.x = take(T * c.d_model * 4);
    L.h_bytes = T * c.d_model * a;
    L.h = take(parts * L.h_bytes);
    L.ssq = take(T * (size_t)(c.d_model / 8 + 1) * 4);        // sum-of-squares partials per row
    L.qkv = take(c.dtype == AX_F32 ? T * (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * 4 : 0);   // fp32 models only
    L.q_bytes = L.attn_bytes = T * qdim * a;
    L.q = take(parts * L.q_bytes);
    L.attn = take(parts * L.attn_bytes);
    L.ffn_bytes = T * (size_t)c.d_ff * a;
    L.ffn = take(parts * L.ffn_bytes);
    if (parts == 2) {
        L.h_lo = (long long)(T * c.d_model);
        L.q_lo = L.attn_lo = (long long)(T * qdim);
        L.ffn_lo = (long long)(T * c.d_ff);
    }
    // Partial records of the split attention: one per (q tile of 32 stacked rows, KV head, key slice).  A call
    // whose longest sequence runs on blocks of 4 or 8 tiles pads EVERY sequence to whole blocks, so the most a
    // call can need with one slice is (T G / 32 + 8 per sequence) tiles per KV head; the slice count is then
    // chosen to stay inside this capacity.  Room for two passes: the per-sequence one and the shared-prefix one.
    L.max_records = std::max<size_t>(SPLIT_ITEMS, ((T * G + 31) / 32 + 8 * S + 2) * (size_t)c.n_kv_heads);
    L.partials = take(c.dtype == AX_BF16 ? 2 * L.max_records * ((size_t)c.head_dim * 32 + 64) * 4 : 0);
    // fp32 slabs of GEMMs that finish in a second kernel: K-slice partials of the residual GEMMs (SPLITK_MAX slabs of
    // [T, d_model]; the SwiGLU GEMM's slices take what fits) and the raw products of the QKV GEMM above 64 rows, which
    // needs ONE whole [T, (Hq + 2 Hkv) hd] slab whatever the ratio of that width to d_model
    L.splitk_bytes = c.dtype == AX_BF16 ? std::max(T * c.d_model * 4 * ax::SPLITK_MAX,
                                                   T * (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * 4) : 0;
    L.splitk = take(L.splitk_bytes);
    L.logits = take(std::min<size_t>(T, LOGIT_ROWS) * (size_t)c.vocab * 4);
    L.amax_scratch = take(2 * std::min<size_t>(T, LOGIT_ROWS) * ax::ARGMAX_PARTS * 4);
    L.amax_out = take(T * 4);
    L.result = take(align_up(8 * S));
    // bf16 models: the library's own copy of every weight matrix in the kernels' packed layout
    L.packed = take(c.dtype == AX_BF16 ? packed_weight_bytes(c) : 0);
    L.total = o;
    return L;
}

}  // namespace

struct ax_model {
    ax_model_config cfg;
    Layout lay;
    char* ws;
    const void *tok_emb, *lm_head, *final_norm;
    std::vector<const void*> wqkv, wo, w_gate, w_up, w_down, norm_attn, norm_mlp;
    int* stage;                       // pinned: N_SLOTS + 1 descriptor slots + result words
    hipEvent_t slot_done[N_SLOTS];
    int next_slot;
    size_t slot_ints;
    // captured verify steps, keyed by (rows, key slices, pool)
    struct Graph { uint64_t key; uint64_t pool_uid; hipGraphExec_t exec; };
    std::vector<Graph> graphs;
    hipStream_t capture_stream = nullptr;
    bool use_graphs = true;
    // optional per-kernel timing (test / benchmark instrumentation, off by default)
    bool prof_on = false;
    struct ProfSpan { int cls; hipEvent_t a, b; };
    std::vector<ProfSpan> prof_spans;      // recorded spans since the last read
    std::vector<hipEvent_t> prof_free;     // events ready for reuse
};

namespace {

bool ok(const ax_model* m) { return ax::handle_live(m, ax::H_MODEL); }

struct ProfScope {                     // records a pair of events around one launch when profiling
    ax_model* m; hipStream_t st; hipEvent_t b = nullptr;
    ProfScope(ax_model* m_, int cls, hipStream_t st_) : m(m_), st(st_) {
        if (!m->prof_on) return;
        hipEvent_t ev[2] = {nullptr, nullptr};
        for (auto& e : ev) {
            if (!m->prof_free.empty()) { e = m->prof_free.back(); m->prof_free.pop_back(); }
            else if (hipEventCreate(&e) != hipSuccess) { e = nullptr; }
        }
        if (!ev[0] || !ev[1]) return;
        (void)hipEventRecord(ev[0], st);
        b = ev[1];
        m->prof_spans.push_back({cls, ev[0], ev[1]});
    }
    ~ProfScope() { if (b) (void)hipEventRecord(b, st); }
};

// Key slices of the split attention, from measurements on the ~1B and ~8B shapes: blocks of 4 q
// tiles (long extends) run best at about two blocks per CU (2048 wavefronts); single-tile
// wavefronts (verify steps, short extends) at about 512 wavefronts - beyond that the merge of the
// slices costs more than the shorter key loops save.  At least two 32-key steps per slice,
// rounded down to a power of two so that the choice (a launch dimension, hence part of a captured
// graph) changes only when the cache length doubles.
int choose_splits(const ax_model* m, int items, int nq, int max_steps) {
    const int target = nq == 1 ? 512 : 2048;
    int want = std::max(1, target / std::max(1, items * nq));
    // many sequences in one call: 512 wavefronts would leave each with a long serial key loop;
    // go up to 2048 wavefronts while a slice still has ~8 key steps
    if (nq == 1 && max_steps / want > 8) want = std::max(want, std::min(2048 / std::max(1, items), (max_steps + 7) / 8));
    want = std::min(want, std::max(1, max_steps / 2));
    const size_t cap = m->lay.max_records / ((size_t)items * nq);      // >= 1 for every call prepare_call lets through
    want = std::min(want, std::max(1, (int)cap));
    int p2 = 1;
    while (p2 * 2 <= want) p2 *= 2;
    return p2;
}

// Host half of a call: validation, KV reservation (all or nothing) and the descriptor, written
// into a pinned staging slot.  Nothing is launched here.
struct CallPlan {
    int n = 0, n_rows = 0, n_out = 0, n_tiles = 0, tile_nq = 1, bt_total = 0, max_steps = 1, out_mode = 0, slot = 0;
    int n_tiles_shared = 0, shared_nq = 4, shared_len = 0, shared_splits = 1;   // shared-prefix attention pass (0 groups = none)
    size_t o_tok = 0, o_pos = 0, o_seq = 0, o_slot = 0, o_out = 0, o_P = 0, o_T = 0, o_row0 = 0, o_bt = 0, o_tinfo = 0,
           o_tab = 0, ints = 0;
    ax_pool* pool = nullptr;
    std::vector<std::pair<int32_t, int32_t>> cows;
};

ax_status prepare_call(ax_model* m, int n, ax_kv* const* kvs, const int32_t* tokens, const int* T_each,
                       int out_mode, const void* out, bool graph_slot, CallPlan& cp) {
    const ax_model_config& c = m->cfg;
    if (n <= 0 || n > c.max_seqs) return fail(AX_ERR_INVALID, "n_seq %d outside 1..%d", n, c.max_seqs);
    if (!kvs || !tokens || !T_each) return fail(AX_ERR_INVALID, "NULL argument");
    if (out_mode < AX_OUT_NONE || out_mode > AX_OUT_ALL_ARGMAX) return fail(AX_ERR_INVALID, "bad out_mode");
    if (out_mode != AX_OUT_NONE && !out) return fail(AX_ERR_INVALID, "out is NULL");

    ax_pool* pool = nullptr;
    long long n_rows = 0;
    for (int s = 0; s < n; ++s) {
        if (!ok(kvs[s])) return fail(AX_ERR_INVALID, "bad KV handle (sequence %d)", s);
        if (s == 0) pool = kvs[s]->pool;
        if (kvs[s]->pool != pool) return fail(AX_ERR_INVALID, "sequences live in different pools");
        for (int u = 0; u < s; ++u)
            if (kvs[u] == kvs[s]) return fail(AX_ERR_INVALID, "sequence %d given twice", s);
        if (T_each[s] <= 0) return fail(AX_ERR_INVALID, "T <= 0 (sequence %d)", s);
        if (kvs[s]->seq.len + T_each[s] > c.max_pos)
            return fail(AX_ERR_INVALID, "P + T = %lld exceeds max_pos %d",
                        (long long)(kvs[s]->seq.len + T_each[s]), c.max_pos);
        n_rows += T_each[s];
    }
    if (n_rows > c.max_tokens) return fail(AX_ERR_INVALID, "%lld rows exceed max_tokens %d", n_rows, c.max_tokens);
    const ax_model_config& pc = pool->cfg;
    if (pc.n_layers != c.n_layers || pc.n_kv_heads != c.n_kv_heads || pc.head_dim != c.head_dim ||
        pc.dtype != c.dtype)
        return fail(AX_ERR_INVALID, "pool geometry does not match the model");
    if (!pool->geom.base) return fail(AX_ERR_INVALID, "pool has no device memory");
    for (long long i = 0; i < n_rows; ++i)
        if (tokens[i] < 0 || tokens[i] >= c.vocab)
            return fail(AX_ERR_INVALID, "token %d at row %lld outside the vocabulary", tokens[i], i);

    // ---- reserve KV room for every sequence, or fail with nothing changed
    std::vector<ax::AppendPlan> plans((size_t)n);
    long long need = 0;
    for (int s = 0; s < n; ++s) {
        plans[(size_t)s] = ax::plan_append(pool->blocks, kvs[s]->seq, T_each[s]);
        need += plans[(size_t)s].need();
    }
    if (need > pool->blocks.n_free())
        return fail(AX_ERR_OOM, "need %lld KV blocks, %lld free", need, (long long)pool->blocks.n_free());

    const int G = c.n_q_heads / c.n_kv_heads;
    cp.n = n;
    cp.n_rows = (int)n_rows;
    cp.out_mode = out_mode;
    cp.pool = pool;
    // attention q tiles (32 stacked rows).  Verify steps and short extends (<= 128 stacked rows
    // per sequence, <= 256 at head_dim 64): one tile per wavefront - measured, a wavefront that
    // carries two tiles (sharing the K/V loads) is no faster, its serial softmax chain per key step
    // is twice as long.  Longer extends: blocks of 4 or 8 tiles that share LDS-staged K/V.  (With
    // 65-128 stacked rows the blocks were tried first and lost by far: a verify round at k = 16
    // of the ~1B model 1.58 -> 1.29 ms, of the ~8B model 5.0 -> 4.4 ms.)
    const int split_rows_max = c.head_dim == 64 ? 256 : 128;
    cp.tile_nq = 1;
    for (int s = 0; s < n; ++s) {
        if (T_each[s] * G > split_rows_max && cp.tile_nq < 4) cp.tile_nq = 4;
        if (T_each[s] * G >= 2048) cp.tile_nq = 8;    // 8 tiles per block: ~10 % on the ~8B shape at T = 512, none below
    }
    cp.n_tiles = cp.bt_total = 0;
    for (int s = 0; s < n; ++s) {
        cp.n_tiles += (T_each[s] * G + 32 * cp.tile_nq - 1) / (32 * cp.tile_nq);
        cp.bt_total += (int)ax::blocks_for(kvs[s]->seq.len + T_each[s], 16);
    }
    // Several short sequences (verify rounds of many sessions) whose block tables begin with the
    // same blocks - forks of one cached prefix: the keys of those blocks are applied to the rows
    // of all sequences in one pass.  Only whole blocks below every sequence's length count (they
    // cannot be copied on write by this call); worth a pass of its own from ~2k saved key reads.
    cp.n_tiles_shared = 0;
    if (c.dtype == AX_BF16 && cp.tile_nq == 1 && n >= 2) {
        size_t common = (size_t)(kvs[0]->seq.len / 16);
        for (int s = 1; s < n && common > 0; ++s) {
            common = std::min(common, (size_t)(kvs[s]->seq.len / 16));
            size_t i = 0;
            while (i < common && kvs[s]->seq.blocks[i] == kvs[0]->seq.blocks[i]) ++i;
            common = i;
        }
        const int shared = (int)(common * 16) & ~31;
        if ((long long)(n - 1) * shared >= kSharedMinKeys) {
            cp.shared_len = shared;
            cp.shared_nq = n_rows * G > 128 ? 8 : 4;
            cp.n_tiles_shared = (int)((n_rows * G + 32 * cp.shared_nq - 1) / (32 * cp.shared_nq));
            int want = std::max(1, 2048 / (cp.n_tiles_shared * c.n_kv_heads * cp.shared_nq));
            want = std::min(want, std::max(1, shared / 64));
            const size_t cap = m->lay.max_records / ((size_t)cp.n_tiles_shared * c.n_kv_heads * cp.shared_nq);
            want = std::min(want, std::max(1, (int)cap));
            cp.shared_splits = 1;
            while (cp.shared_splits * 2 <= want) cp.shared_splits *= 2;
        }
    }
    cp.n_out = out_mode == AX_OUT_NONE ? 0
               : (out_mode == AX_OUT_LAST_LOGITS || out_mode == AX_OUT_LAST_ARGMAX) ? n : (int)n_rows;
    size_t at = 0;
    auto region = [&](size_t ints) { size_t o = at; at += ints; return o; };
    cp.o_tok = region((size_t)n_rows); cp.o_pos = region((size_t)n_rows); cp.o_seq = region((size_t)n_rows);
    cp.o_slot = region((size_t)n_rows);
    cp.o_out = region((size_t)std::max(cp.n_out, 1)); cp.o_P = region((size_t)n); cp.o_T = region((size_t)n);
    cp.o_row0 = region((size_t)n); cp.o_bt = region((size_t)n);
    at = (at + 7) / 8 * 8;                                                   // 32-byte aligned tile records
    cp.o_tinfo = region((size_t)(cp.n_tiles + cp.n_tiles_shared) * 8);
    cp.o_tab = region((size_t)(graph_slot ? m->lay.max_bt : cp.bt_total));   // fixed extent inside a graph
    cp.ints = at;
    if (cp.ints > m->slot_ints || cp.bt_total > n * m->lay.max_bt)
        return fail(AX_ERR_INVALID, "call descriptor does not fit its slot");
    // the split attention writes one partial record per (q tile, KV head, key slice): even with a single slice
    // each pass must fit the workspace region sized for it (it does for every call within max_tokens / max_seqs;
    // checked all the same, before anything is committed, because a kernel would write past the region otherwise)
    if (c.dtype == AX_BF16 &&
        ((size_t)cp.n_tiles * cp.tile_nq * c.n_kv_heads > m->lay.max_records ||
         (size_t)cp.n_tiles_shared * cp.shared_nq * c.n_kv_heads * cp.shared_splits > m->lay.max_records))
        return fail(AX_ERR_UNSUPPORTED, "%d attention tile groups of %d tiles exceed the workspace's %zu partial records",
                    cp.n_tiles, cp.tile_nq, m->lay.max_records);

    // ---- staging slot: the ring behind events, or the slot reserved for captured graphs
    if (graph_slot) {
        cp.slot = N_SLOTS;
    } else {
        cp.slot = m->next_slot;
        m->next_slot = (cp.slot + 1) % N_SLOTS;
        HIP_TRY(hipEventSynchronize(m->slot_done[cp.slot]));
    }
    int* d = m->stage + (size_t)cp.slot * m->slot_ints;

    // ---- from here on the call cannot fail on the host side: commit the KV reservation
    std::vector<int> P((size_t)n);
    for (int s = 0; s < n; ++s) {
        P[(size_t)s] = (int)kvs[s]->seq.len;
        int32_t cs, cd;
        ax::apply_append(pool->blocks, kvs[s]->seq, T_each[s], plans[(size_t)s], &cs, &cd);
        if (cs >= 0) cp.cows.push_back({cs, cd});
    }
    int row = 0, tile = 0, tab = 0, oi = 0;
    cp.max_steps = 1;
    for (int s = 0; s < n; ++s) {
        const int T = T_each[s];
        d[cp.o_P + s] = P[(size_t)s];
        d[cp.o_T + s] = T;
        d[cp.o_row0 + s] = row;
        d[cp.o_bt + s] = tab;
        for (int32_t b : kvs[s]->seq.blocks) d[cp.o_tab + tab++] = b;
        for (int r0 = 0; r0 < T * G; r0 += 32 * cp.tile_nq) {
            int* ti = d + cp.o_tinfo + (size_t)tile * 8;
            ti[0] = s; ti[1] = r0; ti[2] = P[(size_t)s]; ti[3] = T; ti[4] = row; ti[5] = d[cp.o_bt + s];
            ti[6] = 0;
            ti[7] = cp.n_tiles_shared > 0 ? cp.shared_len : 0;      // keys before it are the shared pass's
            ++tile;
        }
        for (int t = 0; t < T; ++t, ++row) {
            d[cp.o_tok + row] = tokens[row];
            d[cp.o_pos + row] = P[(size_t)s] + t;
            d[cp.o_seq + row] = s;
            d[cp.o_slot + row] = kvs[s]->seq.blocks[(size_t)((P[(size_t)s] + t) >> 4)] * 16 + ((P[(size_t)s] + t) & 15);
            if (out_mode == AX_OUT_ALL_LOGITS || out_mode == AX_OUT_ALL_ARGMAX) d[cp.o_out + oi++] = row;
        }
        if (out_mode == AX_OUT_LAST_LOGITS || out_mode == AX_OUT_LAST_ARGMAX) d[cp.o_out + oi++] = row - 1;
        cp.max_steps = std::max(cp.max_steps, (P[(size_t)s] + T - (cp.n_tiles_shared > 0 ? cp.shared_len : 0) + 31) / 32);
    }
    for (int g = 0; g < cp.n_tiles_shared; ++g) {                   // the shared pass: one virtual sequence of all rows
        int* ti = d + cp.o_tinfo + (size_t)(cp.n_tiles + g) * 8;
        ti[0] = 0; ti[1] = g * 32 * cp.shared_nq; ti[2] = cp.shared_len; ti[3] = (int)n_rows; ti[4] = 0; ti[5] = d[cp.o_bt + 0];
        ti[6] = cp.shared_len; ti[7] = 0;
    }
    return AX_OK;
}

// Device half: descriptor upload and the kernel sequence of one forward.  `verify_k` >= 0
// appends the greedy acceptance and the copy of (accepted, next token) to host_result.  With
// `capturing` the launches go into a stream capture: no event is recorded and the kernel
// arguments must not depend on anything but (n_rows, n_splits).
ax_status enqueue_call(ax_model* m, const CallPlan& cp, void* out, hipStream_t stream, int n_splits,
                       int verify_k, int* host_result, bool capturing) {
    const ax_model_config& c = m->cfg;
    const Layout& L = m->lay;
    int* d = m->stage + (size_t)cp.slot * m->slot_ints;
    int* dev_d = (int*)(m->ws + L.desc) + (size_t)cp.slot * m->slot_ints;
    HIP_TRY(hipMemcpyAsync(dev_d, d, cp.ints * sizeof(int), hipMemcpyHostToDevice, stream));

    ax::StepView sv{};
    sv.row_tok = dev_d + cp.o_tok;  sv.row_pos = dev_d + cp.o_pos;  sv.row_seq = dev_d + cp.o_seq; sv.row_slot = dev_d + cp.o_slot;
    sv.out_rows = dev_d + cp.o_out; sv.seq_P = dev_d + cp.o_P;      sv.seq_T = dev_d + cp.o_T;
    sv.seq_row0 = dev_d + cp.o_row0; sv.seq_bt = dev_d + cp.o_bt;   sv.tile_info = dev_d + cp.o_tinfo;
    sv.bt = dev_d + cp.o_tab;
    sv.n_rows = cp.n_rows; sv.n_seq = cp.n; sv.n_out = cp.n_out; sv.n_tiles = cp.n_tiles; sv.tile_nq = cp.tile_nq;
    sv.n_tiles_shared = cp.n_tiles_shared; sv.shared_nq = cp.shared_nq; sv.shared_len = cp.shared_len; sv.shared_splits = cp.shared_splits;

    const ax::DType dt = c.dtype == AX_F32 ? ax::F32 : ax::BF16;
    const ax::KVGeom& kg = cp.pool->geom;
    const int out_mode = cp.out_mode, n_out = cp.n_out;
    // verify calls whose rows fit one LM-head pass: second argmax stage, acceptance and the result's way to the
    // host in one launch (two launches and a copy node fewer per step)
    const bool fused_accept = verify_k >= 0 && n_out > 0 && n_out <= std::min(c.max_tokens, LOGIT_ROWS) &&
                              n_out <= ax::ACCEPT_MAX_ROWS;

    char* ws = m->ws;
    float* x = (float*)(ws + L.x);
    void* h = ws + L.h;
    float* qkv = (float*)(ws + L.qkv);
    void* qb = ws + L.q;
    void* attn = ws + L.attn;
    void* ffn = ws + L.ffn;
    const int d_model = c.d_model, qdim = c.n_q_heads * c.head_dim,
              qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, R = cp.n_rows;

    if (dt == ax::F32) {
        // fp32 models: one kernel per operation (the exactness configuration)
        ax::launch_embed(dt, m->tok_emb, sv.row_tok, x, R, d_model, stream);
        for (int l = 0; l < c.n_layers; ++l) {
            ax::launch_rmsnorm(dt, x, m->norm_attn[(size_t)l], h, nullptr, R, d_model, c.rms_eps, stream);
            { ProfScope ps(m, 0, stream);
              ax::launch_gemm(dt, ax::EPI_STORE_F32, h, m->wqkv[(size_t)l], nullptr, qkv, R, qkv_rows, d_model, stream); }
            ax::launch_rope_kv(dt, qkv, qb, kg, l, sv, (const float*)(ws + L.rope_cos),
                               (const float*)(ws + L.rope_sin), c.n_q_heads, stream);
            { ProfScope ps(m, 1, stream);
              ax::launch_attention(dt, qb, attn, kg, l, sv, c.n_q_heads, nullptr, 1, stream); }
            { ProfScope ps(m, 2, stream);
              ax::launch_gemm(dt, ax::EPI_RESIDUAL, attn, m->wo[(size_t)l], nullptr, x, R, d_model, qdim, stream); }
            ax::launch_rmsnorm(dt, x, m->norm_mlp[(size_t)l], h, nullptr, R, d_model, c.rms_eps, stream);
            { ProfScope ps(m, 3, stream);
              ax::launch_gemm(dt, ax::EPI_SWIGLU, h, m->w_gate[(size_t)l], m->w_up[(size_t)l], ffn, R, c.d_ff, d_model, stream); }
            { ProfScope ps(m, 4, stream);
              ax::launch_gemm(dt, ax::EPI_RESIDUAL, ffn, m->w_down[(size_t)l], nullptr, x, R, d_model, c.d_ff, stream); }
        }
        if (n_out > 0) {
            ax::launch_rmsnorm(dt, x, m->final_norm, h, sv.out_rows, n_out, d_model, c.rms_eps, stream);
            if (out_mode == AX_OUT_LAST_LOGITS || out_mode == AX_OUT_ALL_LOGITS) {
                ProfScope ps(m, 5, stream);
                ax::launch_gemm(dt, ax::EPI_STORE_F32, h, m->lm_head, nullptr, out, n_out, c.vocab, d_model, stream);
            } else {
                float* logits = (float*)(ws + L.logits);
                const int chunk = std::min(c.max_tokens, LOGIT_ROWS);
                for (int r0 = 0; r0 < n_out; r0 += chunk) {
                    const int rows = std::min(chunk, n_out - r0);
                    { ProfScope ps(m, 5, stream);
                      ax::launch_gemm(dt, ax::EPI_STORE_F32, (const char*)h + (size_t)r0 * d_model * 4, m->lm_head,
                                      nullptr, logits, rows, c.vocab, d_model, stream); }
                    if (fused_accept) ax::launch_argmax_partials(logits, rows, c.vocab, (int*)(ws + L.amax_scratch), stream);
                    else ax::launch_argmax(logits, rows, c.vocab, (int*)out + r0, (int*)(ws + L.amax_scratch), stream);
                }
            }
        }
    } else {
        // bf16-weight models: six launches per layer.  RMSNorm is split between the GEMM that
        // writes x (gain-scaled fp16 copy + per-row partial sums of x^2) and the GEMM that reads
        // it (1/rms in the epilogue); rotary embedding and the KV append live in the QKV epilogue.
        float* ssq = (float*)(ws + L.ssq);
        // partial sums of x^2 per row behind the pending norm: as many as the launch that wrote x left (the
        // embedding leaves one; the O and down projections report theirs)
        int nparts = 1;
        ax::GemmArgs base{};
        base.M = R;
        base.split_ws = (float*)(ws + L.splitk);
        base.split_ws_bytes = L.splitk_bytes;
        auto normed = [&](ax::GemmArgs& g) { g.A = h; g.a_lo_off = L.h_lo; g.ssq = ssq; g.nparts = nparts; g.d_norm = d_model; g.eps = c.rms_eps; g.K = d_model; };
        ax::launch_embed_norm(m->tok_emb, sv.row_tok, m->norm_attn[0], x, h, L.h_lo, ssq, nparts, R, d_model, stream);
        for (int l = 0; l < c.n_layers; ++l) {
            {
                ax::GemmArgs g = base;
                normed(g);
                g.W = m->wqkv[(size_t)l]; g.N = qkv_rows;
                g.rope.kv = kg; g.rope.layer = l; g.rope.n_q_heads = c.n_q_heads; g.rope.q_out = qb; g.c_lo_off = L.q_lo;
                g.rope.row_pos = sv.row_pos; g.rope.row_slot = sv.row_slot;
                g.rope.cos = (const float*)(ws + L.rope_cos); g.rope.sin = (const float*)(ws + L.rope_sin);
                ProfScope ps(m, 0, stream);
                (void)ax::launch_gemm_bf16(ax::EPI_QKV, g, stream);   // (its slab always fits: make_layout reserves max_tokens rows of it)
            }
            { ProfScope ps(m, 1, stream);
              ax::launch_attention(dt, qb, attn, kg, l, sv, c.n_q_heads, (float*)(ws + L.partials), n_splits, stream, L.q_lo, L.attn_lo); }
            { ProfScope empty(m, 6, stream); }         // bracket around nothing: the cost of the two events
            {
                ax::GemmArgs g = base;
                g.A = attn; g.a_lo_off = L.attn_lo; g.K = qdim; g.W = m->wo[(size_t)l]; g.N = d_model;
                g.Cf = x; g.C16 = h; g.c_lo_off = L.h_lo; g.gain_next = m->norm_mlp[(size_t)l]; g.ssq_out = ssq;
                ProfScope ps(m, 2, stream);
                nparts = ax::launch_gemm_bf16(ax::EPI_RESIDUAL, g, stream);
            }
            {
                ax::GemmArgs g = base;
                normed(g);
                g.W = m->w_gate[(size_t)l]; g.W2 = m->w_up[(size_t)l]; g.N = c.d_ff; g.C16 = ffn; g.c_lo_off = L.ffn_lo;
                ProfScope ps(m, 3, stream);
                ax::launch_gemm_bf16(ax::EPI_SWIGLU, g, stream);
            }
            {
                ax::GemmArgs g = base;
                g.A = ffn; g.a_lo_off = L.ffn_lo; g.K = c.d_ff; g.W = m->w_down[(size_t)l]; g.N = d_model;
                g.Cf = x; g.C16 = h; g.c_lo_off = L.h_lo; g.ssq_out = ssq;
                g.gain_next = l + 1 < c.n_layers ? m->norm_attn[(size_t)l + 1] : m->final_norm;
                ProfScope ps(m, 4, stream);
                nparts = ax::launch_gemm_bf16(ax::EPI_RESIDUAL, g, stream);
            }
        }
        if (n_out > 0) {
            ax::GemmArgs g = base;
            normed(g);
            g.W = m->lm_head; g.N = c.vocab;
            g.a_rows = n_out == R ? nullptr : sv.out_rows;
            if (out_mode == AX_OUT_LAST_LOGITS || out_mode == AX_OUT_ALL_LOGITS) {
                g.M = n_out; g.Cf = (float*)out;
                ProfScope ps(m, 5, stream);
                ax::launch_gemm_bf16(ax::EPI_STORE_F32, g, stream);
            } else {
                float* logits = (float*)(ws + L.logits);
                const int chunk = std::min(c.max_tokens, LOGIT_ROWS);
                for (int r0 = 0; r0 < n_out; r0 += chunk) {
                    const int rows = std::min(chunk, n_out - r0);
                    ax::GemmArgs gc = g;
                    gc.M = rows; gc.Cf = logits;
                    gc.a_rows = sv.out_rows + r0;            // out_rows lists every row in ALL modes
                    { ProfScope ps(m, 5, stream);
                      ax::launch_gemm_bf16(ax::EPI_STORE_F32, gc, stream); }
                    if (fused_accept) ax::launch_argmax_partials(logits, rows, c.vocab, (int*)(ws + L.amax_scratch), stream);
                    else ax::launch_argmax(logits, rows, c.vocab, (int*)out + r0, (int*)(ws + L.amax_scratch), stream);
                }
            }
        }
    }
    if (verify_k >= 0) {
        int* res = (int*)(ws + L.result);
        if (fused_accept) {
            // host_result is pinned memory the device addresses directly: the kernel writes it, no copy node
            ax::launch_argmax_accept((const int*)(ws + L.amax_scratch), n_out, (int*)out, sv, res, host_result, stream);
        } else {
            ax::launch_accept((const int*)out, sv, res, stream);
            HIP_TRY(hipMemcpyAsync(host_result, res, 2 * sizeof(int) * (size_t)cp.n, hipMemcpyDeviceToHost, stream));
        }
    }
    if (!capturing) {
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventRecord(m->slot_done[cp.slot], stream));
    }
    return AX_OK;
}

// Eager call: prepare, copy-on-write copies, launches.
ax_status run_extend(ax_model* m, int n, ax_kv* const* kvs, const int32_t* tokens, const int* T_each,
                     int out_mode, void* out, hipStream_t stream, int verify_k, int* host_result) {
    CallPlan cp;
    ax_status st = prepare_call(m, n, kvs, tokens, T_each, out_mode, out, false, cp);
    if (st != AX_OK) return st;
    const ax::DType dt = m->cfg.dtype == AX_F32 ? ax::F32 : ax::BF16;
    for (auto& cw : cp.cows) ax::launch_block_copy(dt, cp.pool->geom, m->cfg.n_layers, cw.first, cw.second, stream);
    const int n_splits = choose_splits(m, cp.n_tiles * m->cfg.n_kv_heads, cp.tile_nq, cp.max_steps);
    return enqueue_call(m, cp, out, stream, n_splits, verify_k, host_result, false);
}

// Verify round through a captured graph: the ~9 launches per layer of a (1 + k)-row step cost
// more host time than GPU time when enqueued one by one.  The graph for (k, n_splits) is
// captured once on the model's own stream (the caller's may be the default stream, which
// cannot be captured) and replayed on the caller's stream; everything that changes from round
// to round (tokens, positions, cache length, block table) lives in the descriptor that the
// graph's first node uploads from the reserved pinned slot.
ax_status run_verify_graph(ax_model* m, ax_kv* kv, const int32_t* toks, int T, void* out, hipStream_t stream,
                           int k, int* host_result) {
    CallPlan cp;
    ax_kv* one[1] = {kv};
    ax_status st = prepare_call(m, 1, one, toks, &T, AX_OUT_ALL_ARGMAX, out, true, cp);
    if (st != AX_OK) return st;
    const ax::DType dt = m->cfg.dtype == AX_F32 ? ax::F32 : ax::BF16;
    for (auto& cw : cp.cows) ax::launch_block_copy(dt, cp.pool->geom, m->cfg.n_layers, cw.first, cw.second, stream);
    const int n_splits = choose_splits(m, cp.n_tiles * m->cfg.n_kv_heads, cp.tile_nq, cp.max_steps);
    const uint64_t key = ((uint64_t)(uint32_t)T << 32) | (uint32_t)n_splits;
    hipGraphExec_t exec = nullptr;
    for (auto& g : m->graphs)
        if (g.key == key && g.pool_uid == cp.pool->uid) exec = g.exec;
    if (!exec) {
        hipGraph_t graph = nullptr;
        HIP_TRY(hipStreamBeginCapture(m->capture_stream, hipStreamCaptureModeThreadLocal));
        st = enqueue_call(m, cp, out, m->capture_stream, n_splits, k, host_result, true);
        hipError_t e = hipStreamEndCapture(m->capture_stream, &graph);
        if (st != AX_OK) { if (graph) (void)hipGraphDestroy(graph); return st; }
        if (e != hipSuccess) return fail(AX_ERR_DEVICE, "hipStreamEndCapture: %s", hipGetErrorString(e));
        e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e != hipSuccess) return fail(AX_ERR_DEVICE, "hipGraphInstantiate: %s", hipGetErrorString(e));
        m->graphs.push_back({key, cp.pool->uid, exec});
    }
    HIP_TRY(hipGraphLaunch(exec, stream));
    return AX_OK;
}

}  // namespace

extern "C" {

size_t ax_workspace_bytes(const ax_model_config* cfg) {
    ax_status why;
    if (!config_ok(cfg, &why)) return 0;
    return make_layout(*cfg).total;
}

ax_status ax_model_create(const ax_model_config* cfg, const ax_weights* w, void* workspace,
                          size_t workspace_bytes, ax_model** out) {
    ax_status why;
    if (!out) return fail(AX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (!config_ok(cfg, &why)) return fail(why, "model config rejected");
    if (!w || !workspace) return fail(AX_ERR_INVALID, "NULL weights or workspace");
    if (((uintptr_t)workspace & 255) != 0) return fail(AX_ERR_INVALID, "workspace not 256-byte aligned");
    const Layout L = make_layout(*cfg);
    if (workspace_bytes < L.total)
        return fail(AX_ERR_OOM, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
    if (!w->tok_emb || !w->lm_head || !w->final_norm || !w->wqkv || !w->wo || !w->w_gate ||
        !w->w_up || !w->w_down || !w->norm_attn || !w->norm_mlp)
        return fail(AX_ERR_INVALID, "NULL weight pointer");
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->wqkv[l] || !w->wo[l] || !w->w_gate[l] || !w->w_up[l] || !w->w_down[l] ||
            !w->norm_attn[l] || !w->norm_mlp[l])
            return fail(AX_ERR_INVALID, "NULL weight pointer in layer %d", l);

    ax_model* m = new ax_model();
    m->cfg = *cfg;
    m->lay = L;
    m->ws = (char*)workspace;
    m->tok_emb = w->tok_emb;
    m->lm_head = w->lm_head;
    m->final_norm = w->final_norm;
    const size_t nl = (size_t)cfg->n_layers;
    m->wqkv.assign(w->wqkv, w->wqkv + nl);
    m->wo.assign(w->wo, w->wo + nl);
    m->w_gate.assign(w->w_gate, w->w_gate + nl);
    m->w_up.assign(w->w_up, w->w_up + nl);
    m->w_down.assign(w->w_down, w->w_down + nl);
    m->norm_attn.assign(w->norm_attn, w->norm_attn + nl);
    m->norm_mlp.assign(w->norm_mlp, w->norm_mlp + nl);
    m->slot_ints = align_up(L.desc_ints * 4) / 4;
    m->next_slot = 0;
    m->stage = nullptr;
    for (auto& e : m->slot_done) e = nullptr;

    auto cleanup = [&]() {
        if (m->capture_stream) (void)hipStreamDestroy(m->capture_stream);
        for (auto& e : m->slot_done) if (e) (void)hipEventDestroy(e);
        if (m->stage) (void)hipHostFree(m->stage);
        delete m;
    };
    hipError_t e = hipHostMalloc((void**)&m->stage, ((N_SLOTS + 1) * m->slot_ints + 2 * (size_t)cfg->max_seqs + 16) * sizeof(int), hipHostMallocDefault);
    if (e != hipSuccess) { m->stage = nullptr; cleanup(); return fail(AX_ERR_DEVICE, "hipHostMalloc: %s", hipGetErrorString(e)); }
    for (auto& ev : m->slot_done) {
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) { ev = nullptr; cleanup(); return fail(AX_ERR_DEVICE, "hipEventCreate: %s", hipGetErrorString(e)); }
    }
    e = hipStreamCreateWithFlags(&m->capture_stream, hipStreamNonBlocking);
    if (e != hipSuccess) { m->capture_stream = nullptr; cleanup(); return fail(AX_ERR_DEVICE, "hipStreamCreate: %s", hipGetErrorString(e)); }
    // the guard behind every workspace region (never written again; ax_dbg_check_guards looks at them)
    for (int i = 0; i < L.n_regions; ++i) {
        e = hipMemset(m->ws + L.guard_at[i], GUARD_FILL, GUARD_BYTES);
        if (e != hipSuccess) { cleanup(); return fail(AX_ERR_DEVICE, "hipMemset: %s", hipGetErrorString(e)); }
    }
    // rotary table: angle = pos * base^(-2j/hd), evaluated in double on the host
    const int half = cfg->head_dim / 2;
    std::vector<float> cs((size_t)cfg->max_pos * half), sn((size_t)cfg->max_pos * half);
    for (int j = 0; j < half; ++j) {
        const double theta = std::pow((double)cfg->rope_base, -2.0 * j / cfg->head_dim);
        for (int p = 0; p < cfg->max_pos; ++p) {
            cs[(size_t)p * half + j] = (float)std::cos(p * theta);
            sn[(size_t)p * half + j] = (float)std::sin(p * theta);
        }
    }
    e = hipMemcpy(m->ws + L.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->ws + L.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) { cleanup(); return fail(AX_ERR_DEVICE, "rotary table upload: %s", hipGetErrorString(e)); }
    if (cfg->dtype == AX_BF16) {
        // the kernels read their own packed copies of the matrices (token embedding and gains stay as given)
        char* at = m->ws + L.packed;
        int* bad = (int*)(m->ws + L.result);       // set by the repack where a weight is not finite in fp16
        e = hipMemset(bad, 0, sizeof(int));
        if (e != hipSuccess) { cleanup(); return fail(AX_ERR_DEVICE, "hipMemset: %s", hipGetErrorString(e)); }
        const int d = cfg->d_model, qkv = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim, qd = cfg->n_q_heads * cfg->head_dim;
        auto pack = [&](const void*& w_ptr, int N, int K) {
            ax::launch_pack_weights(w_ptr, at, N, K, nullptr, bad);
            w_ptr = at;
            at += align_up((size_t)N * K * 2);
        };
        for (size_t l = 0; l < nl; ++l) {
            pack(m->wqkv[l], qkv, d);
            pack(m->wo[l], d, qd);
            pack(m->w_gate[l], cfg->d_ff, d);
            pack(m->w_up[l], cfg->d_ff, d);
            pack(m->w_down[l], d, cfg->d_ff);
        }
        pack(m->lm_head, cfg->vocab, d);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipDeviceSynchronize();
        int lost = 0;
        if (e == hipSuccess) e = hipMemcpy(&lost, bad, sizeof(int), hipMemcpyDeviceToHost);
        if (e != hipSuccess) { cleanup(); return fail(AX_ERR_DEVICE, "weight repack: %s", hipGetErrorString(e)); }
        if (lost) {
            cleanup();
            return fail(AX_ERR_UNSUPPORTED, "a weight is not finite in fp16 (|w| > 65504, infinity or NaN): the matrices are multiplied as fp16");
        }
    }
    ax::handle_register(m, ax::H_MODEL);
    *out = m;
    return AX_OK;
}

void ax_model_destroy(ax_model* m) {
    if (!ok(m)) return;
    (void)hipDeviceSynchronize();
    for (auto& e : m->slot_done) (void)hipEventDestroy(e);
    for (auto& g : m->graphs) (void)hipGraphExecDestroy(g.exec);
    (void)hipStreamDestroy(m->capture_stream);
    for (auto& sp : m->prof_spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (auto& e : m->prof_free) (void)hipEventDestroy(e);
    (void)hipHostFree(m->stage);
    ax::handle_unregister(m);
    delete m;
}

ax_status ax_extend(ax_model* model, ax_kv* kv, const int32_t* tokens, int T, int out_mode, void* out,
                    void* hip_stream) {
    if (!ok(model)) return fail(AX_ERR_INVALID, "bad model handle");
    ax_kv* one[1] = {kv};
    return run_extend(model, 1, one, tokens, &T, out_mode, out, (hipStream_t)hip_stream, -1, nullptr);
}

ax_status ax_extend_batch(ax_model* model, int n, ax_kv* const* kvs, const int32_t* tokens_concat,
                          const int* T_each, int out_mode, void* out, void* hip_stream) {
    if (!ok(model)) return fail(AX_ERR_INVALID, "bad model handle");
    return run_extend(model, n, kvs, tokens_concat, T_each, out_mode, out, (hipStream_t)hip_stream, -1, nullptr);
}

ax_status ax_verify(ax_model* model, ax_kv* kv, int32_t pending, const int32_t* drafts, int k,
                    int* accepted, int32_t* next_token, void* hip_stream) {
    if (!ok(model)) return fail(AX_ERR_INVALID, "bad model handle");
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (k < 0 || (k > 0 && !drafts) || !accepted || !next_token) return fail(AX_ERR_INVALID, "bad argument");
    if (1 + k > model->cfg.max_tokens) return fail(AX_ERR_INVALID, "1 + k exceeds max_tokens");
    std::vector<int32_t> toks((size_t)k + 1);
    toks[0] = pending;
    for (int i = 0; i < k; ++i) toks[(size_t)i + 1] = drafts[i];
    const int T = 1 + k;
    const int64_t P = kv->seq.len;
    int* host_res = model->stage + (N_SLOTS + 1) * model->slot_ints;      // pinned result words
    ax_kv* one[1] = {kv};
    hipStream_t stream = (hipStream_t)hip_stream;
    ax_status st = (model->use_graphs && !model->prof_on)
                       ? run_verify_graph(model, kv, toks.data(), T, model->ws + model->lay.amax_out, stream, k, host_res)
                       : run_extend(model, 1, one, toks.data(), &T, AX_OUT_ALL_ARGMAX,
                                    model->ws + model->lay.amax_out, stream, k, host_res);
    if (st != AX_OK) {
        if (kv->seq.len != P) ax::truncate(kv->pool->blocks, kv->seq, P);   // device error after the append
        return st;
    }
    hipError_t e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        ax::truncate(kv->pool->blocks, kv->seq, P);
        return fail(AX_ERR_DEVICE, "hipStreamSynchronize: %s", hipGetErrorString(e));
    }
    const int a = host_res[0];
    *accepted = a;
    *next_token = host_res[1];
    ax::truncate(kv->pool->blocks, kv->seq, P + 1 + a);                    // rollback of rejected drafts
    return AX_OK;
}

// ---- KV images -------------------------------------------------------------------------------

namespace {

struct ImageHeader {                  // 64 bytes, little endian
    uint32_t magic, version;
    int32_t n_layers, n_kv_heads, head_dim, dtype, block_tokens, reserved;
    int64_t n_tokens, payload_bytes;
    int64_t pad[2];
};
static_assert(sizeof(ImageHeader) == 64, "image header is 64 bytes");
constexpr uint32_t IMAGE_MAGIC = 0x564b5841;   // "AXKV"

// The image is read or written by a kernel: only memory the GPU can address will do.
ax_status device_view(const void* p, size_t bytes, char** dev) {
    hipPointerAttribute_t at{};
    hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(AX_ERR_INVALID, "image buffer is neither pinned host memory nor device memory");
    }
    if (at.type != hipMemoryTypeHost && at.type != hipMemoryTypeDevice)
        return fail(AX_ERR_INVALID, "image buffer is neither pinned host memory nor device memory");
    char* d = (char*)(at.type == hipMemoryTypeHost ? at.devicePointer : p);
    if (!d) return fail(AX_ERR_INVALID, "image buffer has no device address");
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)d) == hipSuccess) {
        if (d + bytes > (char*)base + size) return fail(AX_ERR_INVALID, "image buffer is smaller than the image");
    } else {
        (void)hipGetLastError();
    }
    *dev = d;
    return AX_OK;
}

// Uploads a sequence's block ids through the descriptor ring; returns their device address.
ax_status upload_ids(ax_model* m, const std::vector<int32_t>& ids, hipStream_t stream, int* slot_out, const int** dev_ids) {
    if (ids.size() > m->slot_ints) return fail(AX_ERR_INVALID, "sequence has more blocks than a descriptor slot holds");
    const int slot = m->next_slot;
    m->next_slot = (slot + 1) % N_SLOTS;
    HIP_TRY(hipEventSynchronize(m->slot_done[slot]));
    int* d = m->stage + (size_t)slot * m->slot_ints;
    std::memcpy(d, ids.data(), ids.size() * sizeof(int));
    int* dev_d = (int*)(m->ws + m->lay.desc) + (size_t)slot * m->slot_ints;
    HIP_TRY(hipMemcpyAsync(dev_d, d, ids.size() * sizeof(int), hipMemcpyHostToDevice, stream));
    *slot_out = slot;
    *dev_ids = dev_d;
    return AX_OK;
}

}  // namespace

int64_t ax_kv_image_bytes(const ax_pool* p, int64_t n_tokens) {
    if (!ok(p) || n_tokens < 0) return -1;
    return (int64_t)sizeof(ImageHeader) +
           ax::blocks_for(n_tokens, 16) * (int64_t)ax_pool_block_bytes(&p->cfg, 16);
}

ax_status ax_kv_export(ax_model* model, const ax_kv* kv, int64_t n_tokens, void* image, int64_t image_bytes,
                       void* hip_stream) {
    if (!ok(model)) return fail(AX_ERR_INVALID, "bad model handle");
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (n_tokens < 0) n_tokens = kv->seq.len;
    if (n_tokens > kv->seq.len)
        return fail(AX_ERR_INVALID, "export of %lld tokens from a sequence of %lld", (long long)n_tokens, (long long)kv->seq.len);
    const ax_pool* pool = kv->pool;
    if (!pool->geom.base) return fail(AX_ERR_INVALID, "pool has no device memory");
    const int64_t need = ax_kv_image_bytes(pool, n_tokens);
    if (!image || image_bytes < need) return fail(AX_ERR_INVALID, "image buffer of %lld bytes, %lld needed", (long long)image_bytes, (long long)need);
    char* dev = nullptr;
    ax_status st = device_view(image, (size_t)need, &dev);
    if (st != AX_OK) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    ImageHeader h{};
    h.magic = IMAGE_MAGIC; h.version = 1;
    h.n_layers = pool->cfg.n_layers; h.n_kv_heads = pool->cfg.n_kv_heads; h.head_dim = pool->cfg.head_dim;
    h.dtype = pool->cfg.dtype; h.block_tokens = 16;
    h.n_tokens = n_tokens; h.payload_bytes = need - (int64_t)sizeof(ImageHeader);
    HIP_TRY(hipMemcpyAsync(image, &h, sizeof h, hipMemcpyDefault, stream));
    const int64_t nb = ax::blocks_for(n_tokens, 16);
    if (nb > 0) {
        std::vector<int32_t> ids(kv->seq.blocks.begin(), kv->seq.blocks.begin() + nb);
        int slot = 0;
        const int* dev_ids = nullptr;
        st = upload_ids(model, ids, stream, &slot, &dev_ids);
        if (st != AX_OK) return st;
        ax::launch_kv_image(true, pool->cfg.dtype == AX_F32 ? ax::F32 : ax::BF16, pool->geom, pool->cfg.n_layers, dev_ids,
                            (int)nb, dev + sizeof(ImageHeader), (int)(n_tokens - (nb - 1) * 16), stream);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventRecord(model->slot_done[slot], stream));
    }
    HIP_TRY(hipStreamSynchronize(stream));
    return AX_OK;
}

// ---- export that allocates nothing --------------------------------------------------------------
// ax_kv_export borrows a descriptor slot of a model's workspace for the device copy of the sequence's
// block ids (the list the gather kernel walks).  This variant keeps that list in a fixed array of the
// library's own instead, so it needs no model, no workspace and no allocation of any kind.

constexpr int EXPORT_STATIC_MAX_BLOCKS = 16384;          // 64 KiB of block ids: sequences of up to 262 144 tokens
static __device__ __align__(256) int scratch[EXPORT_STATIC_MAX_BLOCKS];

namespace {

constexpr int MAX_DEVICES = 64;
int* g_scratch_ptr[MAX_DEVICES];                         // per device: where that GPU's copy of `scratch` lives
std::mutex g_scratch_mu;

// The array's name is only a stand-in on the host; its address on the current device is looked up
// once per device and kept.
ax_status scratch_of_current_device(int** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(AX_ERR_UNSUPPORTED, "device %d outside the %d this library keeps scratch for", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        int* p = nullptr;
        HIP_TRY(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(AX_ERR_DEVICE, "hipGetSymbolAddress returned no address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return AX_OK;
}

// Block ids travel as kernel arguments, 512 at a time: no host staging buffer, no copy node.
constexpr int ID_CHUNK = 512;
struct IdChunk { int first, count; int ids[ID_CHUNK]; };
__global__ __launch_bounds__(ID_CHUNK) void stage_ids_kernel(IdChunk c, int* __restrict__ dst) {
    const int i = threadIdx.x;
    if (i < c.count) dst[c.first + i] = c.ids[i];
}
struct HeaderWords { int w[16]; };
__global__ __launch_bounds__(64) void image_header_kernel(HeaderWords h, int* __restrict__ dst) {
    if (threadIdx.x < 16) dst[threadIdx.x] = h.w[threadIdx.x];
}

}  // namespace

ax_status ax_kv_export_static(const ax_kv* kv, int64_t n_tokens, void* image, int64_t image_bytes, void* hip_stream) {
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (n_tokens < 0) n_tokens = kv->seq.len;
    if (n_tokens > kv->seq.len)
        return fail(AX_ERR_INVALID, "export of %lld tokens from a sequence of %lld", (long long)n_tokens, (long long)kv->seq.len);
    const ax_pool* pool = kv->pool;
    if (!pool->geom.base) return fail(AX_ERR_INVALID, "pool has no device memory");
    const int64_t nb = ax::blocks_for(n_tokens, 16);
    if (nb > EXPORT_STATIC_MAX_BLOCKS)
        return fail(AX_ERR_UNSUPPORTED, "%lld blocks (%lld tokens) exceed the %d blocks (%d tokens) of the library's static scratch; use ax_kv_export",
                    (long long)nb, (long long)n_tokens, EXPORT_STATIC_MAX_BLOCKS, EXPORT_STATIC_MAX_BLOCKS * 16);
    const int64_t need = ax_kv_image_bytes(pool, n_tokens);
    if (!image || image_bytes < need || ((uintptr_t)image & 3) != 0)
        return fail(AX_ERR_INVALID, "image buffer of %lld bytes, %lld needed (4-byte aligned)", (long long)image_bytes, (long long)need);
    char* dev = nullptr;
    ax_status st = device_view(image, (size_t)need, &dev);
    if (st != AX_OK) return st;
    // the scratch used is the current device's: the pool must live there too
    hipPointerAttribute_t at{};
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur));
    if (hipPointerGetAttributes(&at, pool->geom.base) != hipSuccess || at.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(AX_ERR_INVALID, "pool memory is not device memory");
    }
    if (at.device != cur) return fail(AX_ERR_INVALID, "pool memory lives on device %d, the current device is %d", at.device, cur);
    int* ids = nullptr;
    st = scratch_of_current_device(&ids);
    if (st != AX_OK) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    ImageHeader h{};
    h.magic = IMAGE_MAGIC; h.version = 1;
    h.n_layers = pool->cfg.n_layers; h.n_kv_heads = pool->cfg.n_kv_heads; h.head_dim = pool->cfg.head_dim;
    h.dtype = pool->cfg.dtype; h.block_tokens = 16;
    h.n_tokens = n_tokens; h.payload_bytes = need - (int64_t)sizeof(ImageHeader);
    HeaderWords hw;
    static_assert(sizeof(HeaderWords) == sizeof(ImageHeader), "header travels as 16 words");
    std::memcpy(&hw, &h, sizeof hw);
    image_header_kernel<<<1, 64, 0, stream>>>(hw, (int*)dev);
    for (int64_t b0 = 0; b0 < nb; b0 += ID_CHUNK) {
        IdChunk c;
        c.first = (int)b0;
        c.count = (int)std::min<int64_t>(ID_CHUNK, nb - b0);
        for (int i = 0; i < c.count; ++i) c.ids[i] = kv->seq.blocks[(size_t)(b0 + i)];
        for (int i = c.count; i < ID_CHUNK; ++i) c.ids[i] = 0;
        stage_ids_kernel<<<1, ID_CHUNK, 0, stream>>>(c, ids);
    }
    if (nb > 0)
        ax::launch_kv_image(true, pool->cfg.dtype == AX_F32 ? ax::F32 : ax::BF16, pool->geom, pool->cfg.n_layers, ids,
                            (int)nb, dev + sizeof(ImageHeader), (int)(n_tokens - (nb - 1) * 16), stream);
    HIP_TRY(hipGetLastError());
    return AX_OK;
}

ax_status ax_kv_import(ax_model* model, ax_pool* pool, const void* image, int64_t image_bytes, ax_kv** out,
                       void* hip_stream) {
    if (!out) return fail(AX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (!ok(model)) return fail(AX_ERR_INVALID, "bad model handle");
    if (!ok(pool)) return fail(AX_ERR_INVALID, "bad pool handle");
    if (!pool->geom.base) return fail(AX_ERR_INVALID, "pool has no device memory");
    if (!image || image_bytes < (int64_t)sizeof(ImageHeader)) return fail(AX_ERR_INVALID, "image shorter than its header");
    char* dev = nullptr;
    ax_status st = device_view(image, (size_t)image_bytes, &dev);
    if (st != AX_OK) return st;
    ImageHeader h{};
    HIP_TRY(hipMemcpy(&h, image, sizeof h, hipMemcpyDefault));
    const ax_model_config& pc = pool->cfg;
    if (h.magic != IMAGE_MAGIC || h.version != 1) return fail(AX_ERR_INVALID, "not a KV image");
    if (h.n_layers != pc.n_layers || h.n_kv_heads != pc.n_kv_heads || h.head_dim != pc.head_dim || h.dtype != pc.dtype ||
        h.block_tokens != 16)
        return fail(AX_ERR_INVALID, "image geometry does not match the pool");
    if (h.n_tokens < 0 || h.n_tokens > model->cfg.max_pos) return fail(AX_ERR_INVALID, "image of %lld tokens exceeds max_pos", (long long)h.n_tokens);
    const int64_t need = ax_kv_image_bytes(pool, h.n_tokens);
    if (h.payload_bytes != need - (int64_t)sizeof(ImageHeader) || image_bytes < need) return fail(AX_ERR_INVALID, "image is truncated");
    const int64_t nb = ax::blocks_for(h.n_tokens, 16);
    if (nb > pool->blocks.n_free()) return fail(AX_ERR_OOM, "need %lld KV blocks, %lld free", (long long)nb, (long long)pool->blocks.n_free());
    ax_kv* k = nullptr;
    st = ax_kv_alloc(pool, &k);
    if (st != AX_OK) return st;
    if (nb > 0) {
        const ax::AppendPlan plan = ax::plan_append(pool->blocks, k->seq, h.n_tokens);
        int32_t cs, cd;
        ax::apply_append(pool->blocks, k->seq, h.n_tokens, plan, &cs, &cd);
        hipStream_t stream = (hipStream_t)hip_stream;
        int slot = 0;
        const int* dev_ids = nullptr;
        st = upload_ids(model, k->seq.blocks, stream, &slot, &dev_ids);
        if (st == AX_OK) {
            ax::launch_kv_image(false, pc.dtype == AX_F32 ? ax::F32 : ax::BF16, pool->geom, pc.n_layers, dev_ids, (int)nb,
                                dev + sizeof(ImageHeader), 16, stream);
            hipError_t e = hipGetLastError();
            if (e == hipSuccess) e = hipEventRecord(model->slot_done[slot], stream);
            if (e != hipSuccess) st = fail(AX_ERR_DEVICE, "KV import: %s", hipGetErrorString(e));
        }
        if (st != AX_OK) { ax_kv_free(k); return st; }
    }
    *out = k;
    return AX_OK;
}

ax_status ax_verify_batch(ax_model* model, int n, ax_kv* const* kvs, const int32_t* pending, const int32_t* drafts_concat,
                          const int* k_each, int* accepted, int32_t* next_token, void* hip_stream) {
    if (!ok(model)) return fail(AX_ERR_INVALID, "bad model handle");
    if (n <= 0 || n > model->cfg.max_seqs) return fail(AX_ERR_INVALID, "n_seq %d outside 1..%d", n, model->cfg.max_seqs);
    if (!kvs || !pending || !k_each || !accepted || !next_token) return fail(AX_ERR_INVALID, "NULL argument");
    std::vector<int32_t> toks;
    std::vector<int> T((size_t)n);
    std::vector<int64_t> P((size_t)n);
    long long nd = 0;
    for (int s = 0; s < n; ++s) {
        if (!ok(kvs[s])) return fail(AX_ERR_INVALID, "bad KV handle (sequence %d)", s);
        if (k_each[s] < 0) return fail(AX_ERR_INVALID, "k < 0 (sequence %d)", s);
        nd += k_each[s];
    }
    if (nd > 0 && !drafts_concat) return fail(AX_ERR_INVALID, "drafts is NULL");
    if (nd + n > model->cfg.max_tokens) return fail(AX_ERR_INVALID, "sum of 1 + k exceeds max_tokens");
    const int32_t* dr = drafts_concat;
    for (int s = 0; s < n; ++s) {
        toks.push_back(pending[s]);
        toks.insert(toks.end(), dr, dr + k_each[s]);
        dr += k_each[s];
        T[(size_t)s] = 1 + k_each[s];
        P[(size_t)s] = kvs[s]->seq.len;
    }
    auto undo = [&]() {
        for (int s = 0; s < n; ++s)
            if (kvs[s]->seq.len != P[(size_t)s]) ax::truncate(kvs[s]->pool->blocks, kvs[s]->seq, P[(size_t)s]);
    };
    int* host_res = model->stage + (N_SLOTS + 1) * model->slot_ints;
    hipStream_t stream = (hipStream_t)hip_stream;
    ax_status st = run_extend(model, n, kvs, toks.data(), T.data(), AX_OUT_ALL_ARGMAX, model->ws + model->lay.amax_out,
                              stream, 0, host_res);
    if (st != AX_OK) { undo(); return st; }
    hipError_t e = hipStreamSynchronize(stream);
    if (e != hipSuccess) { undo(); return fail(AX_ERR_DEVICE, "hipStreamSynchronize: %s", hipGetErrorString(e)); }
    for (int s = 0; s < n; ++s) {
        accepted[s] = host_res[2 * s];
        next_token[s] = host_res[2 * s + 1];
        ax::truncate(kvs[s]->pool->blocks, kvs[s]->seq, P[(size_t)s] + 1 + accepted[s]);
    }
    return AX_OK;
}

ax_status ax_exspec_generate(ax_model* model, ax_kv* kv, const ax_lut* lut, const int32_t* history, int64_t n_history,
                             int32_t pending, int max_new, int k, int selective, uint64_t seed, int32_t* out_tokens,
                             ax_exspec_stats* stats, void* hip_stream) {
    if (!ok(model)) return fail(AX_ERR_INVALID, "bad model handle");
    if (!ok(kv)) return fail(AX_ERR_INVALID, "bad KV handle");
    if (!ok(lut)) return fail(AX_ERR_INVALID, "bad table handle");
    if (max_new < 0 || k < 0 || n_history < 0 || (n_history > 0 && !history) || (max_new > 0 && !out_tokens))
        return fail(AX_ERR_INVALID, "bad argument");
    if (lut->lut.vocab != model->cfg.vocab) return fail(AX_ERR_INVALID, "table and model vocabularies differ");
    ax_exspec_stats st{0, 0, 0, 0};
    std::vector<int32_t> ctx(history, history + n_history);
    ctx.push_back(pending);
    std::vector<int32_t> drafts((size_t)std::max(k, 1));
    int emitted = 0;
    while (emitted < max_new) {
        const int kk = std::min(k, max_new - emitted - 1);           // never draft past the requested length
        int hits = 0;
        const int nd = kk > 0 ? lut->lut.draft(ctx, kk, selective != 0, seed, emitted, drafts.data(), &hits) : 0;
        if (nd == 0) ++st.fallbacks;
        int a = 0;
        int32_t nxt = 0;
        const ax_status rc = ax_verify(model, kv, pending, drafts.data(), nd, &a, &nxt, hip_stream);
        if (rc != AX_OK) {
            if (stats) *stats = st;
            return rc;
        }
        ++st.rounds;
        st.drafted += nd;
        st.accepted += a;
        for (int i = 0; i < a; ++i) { out_tokens[emitted++] = drafts[(size_t)i]; ctx.push_back(drafts[(size_t)i]); }
        out_tokens[emitted++] = nxt;
        ctx.push_back(nxt);
        pending = nxt;
    }
    if (stats) *stats = st;
    return AX_OK;
}

ax_status ax_dbg_gemm(int dtype, int epilogue, const void* A, const void* W, const void* W2, void* C, int M,
                      int N, int K, void* hip_stream) {
    if (!A || !W || !C || M <= 0 || N <= 0 || K <= 0 || epilogue < 0 || epilogue > 2 ||
        (epilogue == 2 && !W2) || (dtype != AX_F32 && dtype != AX_BF16))
        return fail(AX_ERR_INVALID, "bad argument");
    if (dtype == AX_BF16 && (K % 64 != 0 || N % 16 != 0)) return fail(AX_ERR_UNSUPPORTED, "bf16 needs K %% 64 == 0, N %% 16 == 0");
    hipStream_t s = (hipStream_t)hip_stream;
    // test-only entry: the kernels read packed weights, the caller passes row-major ones - repack
    // into temporary device memory (the only place the library allocates device memory)
    void *pw = nullptr, *pw2 = nullptr;
    if (dtype == AX_BF16) {
        const size_t bytes = (size_t)N * K * 2;
        HIP_TRY(hipMalloc(&pw, bytes));
        ax::launch_pack_weights(W, pw, N, K, s);
        if (W2) {
            hipError_t e2 = hipMalloc(&pw2, bytes);
            if (e2 != hipSuccess) { (void)hipFree(pw); return fail(AX_ERR_DEVICE, "hipMalloc: %s", hipGetErrorString(e2)); }
            ax::launch_pack_weights(W2, pw2, N, K, s);
        }
    }
    void* scratch = nullptr;
    if (dtype == AX_BF16 && epilogue == 2 && M > 16 && M <= 192) {
        // the row counts at which the SwiGLU GEMM may cut K into slices: give it the slab scratch a model's workspace has
        const size_t bytes = (size_t)ax::SPLITK_MAX * 2 * M * N * sizeof(float);
        if (hipMalloc(&scratch, bytes) != hipSuccess) scratch = nullptr;
        ax::GemmArgs g{};
        g.A = A; g.W = pw; g.W2 = pw2; g.M = M; g.N = N; g.K = K;
        g.Cf = (float*)C; g.C16 = C;
        g.split_ws = (float*)scratch;
        g.split_ws_bytes = scratch ? bytes : 0;
        ax::launch_gemm_bf16(ax::EPI_SWIGLU, g, s);
    } else {
        ax::launch_gemm(dtype == AX_F32 ? ax::F32 : ax::BF16, (ax::Epilogue)epilogue, A, pw ? pw : W, pw2 ? pw2 : W2, C, M, N, K, s);
    }
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (pw) (void)hipFree(pw);
    if (pw2) (void)hipFree(pw2);
    if (scratch) (void)hipFree(scratch);
    if (e != hipSuccess) return fail(AX_ERR_DEVICE, "debug GEMM: %s", hipGetErrorString(e));
    return AX_OK;
}

ax_status ax_dbg_gemm_residual(const void* A, const void* W, const void* gain, float* x, void* a16, float* ssq,
                               int* n_parts, int M, int N, int K, void* split_ws, size_t split_ws_bytes,
                               void* hip_stream) {
    if (!A || !W || !gain || !x || !a16 || !ssq || !n_parts || M <= 0 || N <= 0 || K <= 0 || (split_ws_bytes && !split_ws))
        return fail(AX_ERR_INVALID, "bad argument");
    if (K % 64 != 0 || N % 16 != 0) return fail(AX_ERR_UNSUPPORTED, "bf16 needs K %% 64 == 0, N %% 16 == 0");
    if (M > 16 && N % 32 != 0) return fail(AX_ERR_UNSUPPORTED, "more than 16 rows need N %% 32 == 0 (N is a model width)");
    hipStream_t s = (hipStream_t)hip_stream;
    void* pw = nullptr;
    HIP_TRY(hipMalloc(&pw, (size_t)N * K * 2));
    ax::launch_pack_weights(W, pw, N, K, s);
    ax::GemmArgs g{};
    g.A = A; g.W = pw; g.M = M; g.N = N; g.K = K;
    g.Cf = x; g.C16 = a16; g.gain_next = gain; g.ssq_out = ssq;
    g.split_ws = split_ws_bytes ? (float*)split_ws : nullptr;
    g.split_ws_bytes = split_ws_bytes;
    *n_parts = ax::launch_gemm_bf16(ax::EPI_RESIDUAL, g, s);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(pw);
    if (e != hipSuccess) return fail(AX_ERR_DEVICE, "debug GEMM: %s", hipGetErrorString(e));
    return AX_OK;
}

ax_status ax_dbg_gemm_time(int dtype, int epilogue, const void* A, const void* W, const void* W2, void* C, int M,
                           int N, int K, int iters, size_t w_stride_bytes, int w_count, float* avg_us,
                           void* hip_stream) {
    if (!A || !W || !C || !avg_us || M <= 0 || N <= 0 || K <= 0 || iters <= 0 || w_count <= 0 || epilogue < 0 ||
        epilogue > 2 || (epilogue == 2 && !W2) || (dtype != AX_F32 && dtype != AX_BF16))
        return fail(AX_ERR_INVALID, "bad argument");
    if (dtype == AX_BF16 && (K % 64 != 0 || N % 16 != 0)) return fail(AX_ERR_UNSUPPORTED, "bf16 needs K %% 64 == 0, N %% 16 == 0");
    hipStream_t s = (hipStream_t)hip_stream;
    TimerEvents ev;
    HIP_TRY(ev.create());
    const hipEvent_t e0 = ev.a, e1 = ev.b;
    const ax::DType dt = dtype == AX_F32 ? ax::F32 : ax::BF16;
    void *pw = nullptr, *pw2 = nullptr;                     // packed copies of all the weight sets (test-only allocation)
    if (dtype == AX_BF16) {
        if (hipMalloc(&pw, (size_t)w_count * w_stride_bytes) != hipSuccess) return fail(AX_ERR_DEVICE, "hipMalloc failed");
        if (W2 && hipMalloc(&pw2, (size_t)w_count * w_stride_bytes) != hipSuccess) { (void)hipFree(pw); return fail(AX_ERR_DEVICE, "hipMalloc failed"); }
        for (int i = 0; i < w_count; ++i) {
            const size_t off = (size_t)i * w_stride_bytes;
            ax::launch_pack_weights((const char*)W + off, (char*)pw + off, N, K, s);
            if (W2) ax::launch_pack_weights((const char*)W2 + off, (char*)pw2 + off, N, K, s);
        }
        W = pw;
        if (W2) W2 = pw2;
    }
    auto run = [&](int i) {
        const size_t off = (size_t)(i % w_count) * w_stride_bytes;
        ax::launch_gemm(dt, (ax::Epilogue)epilogue, A, (const char*)W + off, W2 ? (const char*)W2 + off : nullptr, C,
                        M, N, K, s);
    };
    for (int i = 0; i < std::min(iters, 3); ++i) run(i);
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < iters; ++i) run(i);
    (void)hipEventRecord(e1, s);
    hipError_t e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (pw) (void)hipFree(pw);
    if (pw2) (void)hipFree(pw2);
    if (e != hipSuccess) return fail(AX_ERR_DEVICE, "timing: %s", hipGetErrorString(e));
    *avg_us = ms * 1000.f / (float)iters;
    return AX_OK;
}

ax_status ax_dbg_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (!dst || !src || bytes == 0 || bytes % 16 != 0) return fail(AX_ERR_INVALID, "bad argument");
    ax::launch_plain_copy(dst, src, bytes / 16, (hipStream_t)hip_stream);
    HIP_TRY(hipGetLastError());
    return AX_OK;
}

ax_status ax_dbg_peaks(void* buf, size_t bytes, int reps, float* read_gbs, float* copy_gbs,
                       float* mfma_f16_tflops, void* hip_stream) {
    if (!buf || bytes < 64 || bytes % 32 != 0 || reps < 1 || !read_gbs || !copy_gbs || !mfma_f16_tflops)
        return fail(AX_ERR_INVALID, "bad argument");
    hipStream_t s = (hipStream_t)hip_stream;
    TimerEvents ev;
    HIP_TRY(ev.create());
    const hipEvent_t e0 = ev.a, e1 = ev.b;
    char* p = (char*)buf;
    const size_t half = bytes / 2;
    double flops = 0.0;
    float ms[3] = {0.f, 0.f, 0.f};
    for (int which = 0; which < 3; ++which) {
        for (int r = -2; r < reps; ++r) {
            if (r == 0) HIP_TRY(hipEventRecord(e0, s));
            // the sink of the two read-only kernels is never written (see the kernels)
            if (which == 0) ax::launch_read_stream(p, bytes / 16, p, s);
            else if (which == 1) ax::launch_plain_copy(p + half, p, half / 16, s);
            else flops = ax::launch_mfma_loop(4096, p, s);
        }
        HIP_TRY(hipEventRecord(e1, s));
        HIP_TRY(hipEventSynchronize(e1));
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventElapsedTime(&ms[which], e0, e1));
    }
    *read_gbs = (float)((double)bytes * reps / (ms[0] * 1e-3) / 1e9);
    *copy_gbs = (float)((double)half * 2.0 * reps / (ms[1] * 1e-3) / 1e9);
    *mfma_f16_tflops = (float)(flops * reps / (ms[2] * 1e-3) / 1e12);
    return AX_OK;
}

ax_status ax_dbg_cu_fill(void* buf, size_t bytes, float* l2_gbs_per_cu, float* hbm_gbs_per_cu, void* hip_stream) {
    constexpr int CUS = 256;
    constexpr size_t L2_REGION = 64 << 10;                       // per block: 16 MB over the chip, 2 MB per XCD's 4 MB L2
    constexpr int L2_PASSES = 256;
    if (!buf || bytes < CUS * (size_t)(1 << 20) || bytes % (CUS * 16) != 0 || !l2_gbs_per_cu || !hbm_gbs_per_cu)
        return fail(AX_ERR_INVALID, "bad argument (at least 256 MiB, a multiple of 4096 bytes)");
    hipStream_t s = (hipStream_t)hip_stream;
    TimerEvents ev;
    HIP_TRY(ev.create());
    const size_t hbm_region = bytes / CUS;                       // read once: nothing of it is in a cache
    float ms[2] = {0.f, 0.f};
    for (int which = 0; which < 2; ++which) {
        // (one untimed launch first for the L2 figure; none for the memory figure, whose untimed pass would leave
        // up to 256 MB of the buffer in the memory-side cache)
        for (int rep = which == 0 ? -1 : 0; rep < 1; ++rep) {
            if (rep == 0) HIP_TRY(hipEventRecord(ev.a, s));
            // the sink is never written (see the kernel)
            if (which == 0) ax::launch_cu_fill(buf, L2_REGION / 16, CUS, L2_PASSES, buf, s);
            else ax::launch_cu_fill(buf, hbm_region / 16, CUS, 1, buf, s);
        }
        HIP_TRY(hipEventRecord(ev.b, s));
        HIP_TRY(hipEventSynchronize(ev.b));
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventElapsedTime(&ms[which], ev.a, ev.b));
    }
    *l2_gbs_per_cu = (float)((double)L2_REGION * L2_PASSES / (ms[0] * 1e-3) / 1e9);
    *hbm_gbs_per_cu = (float)((double)hbm_region / (ms[1] * 1e-3) / 1e9);
    return AX_OK;
}

ax_status ax_dbg_phase_order(void* buf, size_t bytes, int blocks, int rounds, float* boundary_us, float* barrier_us,
                             void* hip_stream) {
    if (!buf || bytes < 4096 || blocks < 8 || blocks % 8 != 0 || blocks > 256 || rounds < 1 || rounds > 100000 || !boundary_us ||
        !barrier_us)
        return fail(AX_ERR_INVALID, "bad argument");
    hipStream_t s = (hipStream_t)hip_stream;
    TimerEvents ev;
    HIP_TRY(ev.create());
    const hipEvent_t e0 = ev.a, e1 = ev.b;
    char* p = (char*)buf;
    int* err = (int*)(p + 3072);
    float ms[2] = {0.f, 0.f};
    for (int which = 0; which < 2; ++which) {
        for (int rep = -1; rep < 1; ++rep) {                   // one untimed pass, one timed
            HIP_TRY(hipMemsetAsync(p, 0, 4096, s));
            HIP_TRY(hipEventRecord(e0, s));
            if (which == 0) {
                for (int r = 0; r < rounds; ++r) ax::launch_boundary(p, blocks, s);
            } else {
                ax::launch_grid_barrier(p, err, blocks, rounds, s);
            }
            HIP_TRY(hipEventRecord(e1, s));
            HIP_TRY(hipEventSynchronize(e1));
            HIP_TRY(hipGetLastError());
        }
        HIP_TRY(hipEventElapsedTime(&ms[which], e0, e1));
    }
    int timed_out = 0;
    HIP_TRY(hipMemcpy(&timed_out, err, sizeof(int), hipMemcpyDeviceToHost));
    if (timed_out) return fail(AX_ERR_DEVICE, "grid barrier: a workgroup gave up waiting (the launch was not resident as a whole)");
    *boundary_us = ms[0] * 1e3f / (float)rounds;
    *barrier_us = ms[1] * 1e3f / (float)rounds;
    return AX_OK;
}

ax_status ax_dbg_read(ax_model* m, int which, void* host_dst, size_t bytes) {
    if (!ok(m) || !host_dst) return fail(AX_ERR_INVALID, "bad argument");
    const Layout& L = m->lay;
    const size_t off[6] = {L.x, L.qkv, L.q, L.attn, L.ffn, L.h};
    const size_t len[6] = {L.h - L.x, L.q - L.qkv, L.q_bytes, L.attn_bytes, L.ffn_bytes, L.h_bytes};   // hi parts only
    if (which < 0 || which > 5) return fail(AX_ERR_INVALID, "bad buffer id");
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host_dst, m->ws + off[which], std::min(bytes, len[which]), hipMemcpyDeviceToHost));
    return AX_OK;
}

ax_status ax_dbg_check_guards(ax_model* m, int* first_bad) {
    if (!ok(m) || !first_bad) return fail(AX_ERR_INVALID, "bad argument");
    HIP_TRY(hipDeviceSynchronize());
    *first_bad = -1;
    unsigned char host[GUARD_BYTES];
    for (int i = 0; i < m->lay.n_regions; ++i) {
        HIP_TRY(hipMemcpy(host, m->ws + m->lay.guard_at[i], GUARD_BYTES, hipMemcpyDeviceToHost));
        for (int b = 0; b < GUARD_BYTES; ++b)
            if (host[b] != GUARD_FILL) {
                *first_bad = i;
                return AX_OK;
            }
    }
    return AX_OK;
}

ax_status ax_dbg_use_graphs(ax_model* m, int enable) {
    if (!ok(m)) return fail(AX_ERR_INVALID, "bad model handle");
    m->use_graphs = enable != 0;
    return AX_OK;
}

ax_status ax_dbg_profile(ax_model* m, int enable) {
    if (!ok(m)) return fail(AX_ERR_INVALID, "bad model handle");
    m->prof_on = enable != 0;
    return AX_OK;
}

ax_status ax_dbg_profile_read(ax_model* m, double* ms_by_class, int64_t* launches_by_class) {
    if (!ok(m) || !ms_by_class || !launches_by_class) return fail(AX_ERR_INVALID, "bad argument");
    HIP_TRY(hipDeviceSynchronize());
    for (int i = 0; i < AX_DBG_PROFILE_CLASSES; ++i) { ms_by_class[i] = 0.0; launches_by_class[i] = 0; }
    for (auto& sp : m->prof_spans) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
        ms_by_class[sp.cls] += ms;
        ++launches_by_class[sp.cls];
        m->prof_free.push_back(sp.a);
        m->prof_free.push_back(sp.b);
    }
    m->prof_spans.clear();
    return AX_OK;
}

}  // extern "C"
