// Causal "extend" attention over the paged KV cache (grouped-query attention): the T new rows
// of a sequence attend to the P cached positions and to each other; row at position p sees
// keys 0..p (prefix caching relies on exactly this causality, paper Sec. 2.3).
//
//   * attn_simple_kernel: one wavefront per (row, query head), fp32 arithmetic, any head_dim
//     up to 256 and either storage type.  It is the fp32 models' path.
//   * attn_split_kernel + attn_combine_kernel: 16-bit path on the matrix cores (fp16 q, K, V and
//     probabilities, fp32 accumulation; used by bf16-weight models).  The query rows
//     of the G heads that share one KV head are stacked into one matrix (row = t*G + g), cut
//     into tiles of 32 rows; one wavefront owns (tile, KV head, slice of the key range), streams
//     its K/V slice from the pages straight into MFMA operand registers, keeps an online
//     softmax per row and writes an unnormalised partial (O, m, l); the combine kernel merges
//     the slices.  Splitting the key range is what fills 256 CUs when T is small (verify:
//     T = 1 + k) and it is harmless when T is large.
#include "kernels.h"

namespace ax {

typedef _Float16 f16;      // activation and KV-cache type of bf16-weight models
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float ld_f32(const float* p) { return *p; }
__device__ __forceinline__ float ld_f32(const f16* p) { return (float)*p; }
__device__ __forceinline__ void st_f32(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_f32(f16* p, float v) { *p = (f16)v; }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_add(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ------------------------------------------------------------------------------ simple kernel
// grid (n_rows, Hq), 64 threads.  Keys are taken 64 at a time: lane j scores key base + j,
// the wavefront reduces max and sum with shuffles (online softmax), then lane c accumulates
// output channels c, c + 64, ... over the 64 keys (probabilities broadcast by shuffle).
template <typename T, int HD_MAX>
__global__ __launch_bounds__(64) void attn_simple_kernel(const T* __restrict__ q, T* __restrict__ out,
                                                         KVGeom kv, int layer,
                                                         const int* __restrict__ row_pos,
                                                         const int* __restrict__ row_seq,
                                                         const int* __restrict__ seq_bt,
                                                         const int* __restrict__ bt, int Hq) {
    constexpr int NC = HD_MAX / 64;
    const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int hd = kv.head_dim, B = kv.block_tokens;
    const int hk = h / (Hq / kv.n_kv_heads);
    const int pos = row_pos[r];
    const int* tab = bt + seq_bt[row_seq[r]];
    const T* Kp = (const T*)kv.base + kv.plane(layer, 0, hk);
    const T* Vp = (const T*)kv.base + kv.plane(layer, 1, hk);
    const T* qr = q + ((long long)r * Hq + h) * hd;
    const float scale = 1.0f / sqrtf((float)hd);

    __shared__ float sq[HD_MAX];
    for (int c = lane; c < hd; c += 64) sq[c] = ld_f32(qr + c);
    __syncthreads();

    float m = -INFINITY, l = 0.f, o[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) o[i] = 0.f;

    for (int base = 0; base <= pos; base += 64) {
        const int j = base + lane;
        float s = -INFINITY;
        if (j <= pos) {
            const T* kr = Kp + ((long long)tab[j / B] * B + j % B) * hd;
            float d = 0.f;
            for (int c = 0; c < hd; ++c) d = fmaf(sq[c], ld_f32(kr + c), d);
            s = d * scale;
        }
        const float mn = fmaxf(m, wave_max(s));            // finite: key `base` is always visible
        const float p = (j <= pos) ? expf(s - mn) : 0.f;
        const float alpha = expf(m - mn);                  // exp(-inf) = 0 on the first chunk
        l = l * alpha + wave_add(p);
#pragma unroll
        for (int i = 0; i < NC; ++i) o[i] *= alpha;
        const int cnt = min(64, pos - base + 1);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj, 64);
            const int key = base + jj;
            const T* vb = Vp + (long long)tab[key / B] * B * hd + key % B;
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                const int c = lane + 64 * i;
                if (c < hd) o[i] = fmaf(pj, ld_f32(vb + (long long)c * B), o[i]);
            }
        }
        m = mn;
    }
    T* orow = out + ((long long)r * Hq + h) * hd;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = lane + 64 * i;
        if (c < hd) st_f32(orow + c, o[i] / l);
    }
}

// ------------------------------------------------------------------------------ MFMA split kernel
// One wavefront = one (group of NQ q tiles of 32 stacked rows, KV head, key slice).  With NQ > 1
// the K and V operands of a 32-key step are loaded once and used for every q tile of the group:
// a verify step (T = 1 + k rows, (1 + k) * G stacked rows) is then a single group per KV head.
//
// S^T = K * Q^T is computed so that the score tile comes out with lane <-> query row
// (column l % 32) and registers <-> keys: register r of lane l is key (r/4)*8 + (l/32)*4 + r%4
// of the 32-key step.  Row max / sum therefore need the 16 registers of the lane plus one
// exchange with lane ^ 32, and the softmax rescale is a per-lane scalar.  The probabilities
// are already laid out as the B operand of O^T = V^T * P^T: registers 0..7 cover keys
// {4g..4g+3, 8+4g..8+4g+3} of the first 16-key block, registers 8..15 the same of the second
// block (g = l/32).  V pages are token-minor ([head_dim][16]), so the matching A operand of a
// lane (channel d) is two 8-byte loads from its channel's 16-token row.
// One 32-key step of the online softmax for the lane's query row.  s: raw scores q.k of the
// lane's 16 keys (key of register r: kv0 + (r/4)*8 + g*4 + r%4); c = log2(e)/sqrt(hd).  m is the
// reference exponent of the row (scaled, base-2 domain), l the running sum of 2^(s*c - m) over the
// LANE's keys (the caller adds l of lane and lane ^ 32 when it is done).  The
// reference is NOT kept equal to the running maximum: it is only raised when some row of the
// wavefront has a score more than SOFTMAX_SLACK above it (then every row moves to its current
// maximum, the function returns true and the caller multiplies its output accumulators by
// alpha).  In between, probabilities may exceed 1 by at most 2^SOFTMAX_SLACK, far inside the
// range of fp16 operands and fp32 sums, and the per-step rescale of the accumulators - as much
// vector work as the exponentials themselves - runs a handful of times per row instead of on
// every step.  (m, l, o) stay mutually consistent, which is all the slice merge needs.
// The probabilities are packed to fp16 (round toward zero, one instruction per pair) as the two
// PV operands, and l sums exactly those packed values (dot product with ones), so the
// normalisation matches the weights the PV product really uses.  The causal mask is applied only
// on steps that reach past the tile's earliest row (`diagonal`, wavefront-uniform).  v_exp_f32
// is used directly: a result that underflows to 0 is exact enough for a probability.
constexpr float SOFTMAX_SLACK = 8.0f;
__device__ __forceinline__ bool online_softmax_step(f32x16& s, int kv0, int g, int pos_q, bool diagonal, float c,
                                                    float& m, float& l, float& alpha, f16x8 (&pb)[2]) {
    if (diagonal) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kj = kv0 + (r >> 2) * 8 + g * 4 + (r & 3);
            s[r] = (kj <= pos_q) ? s[r] : -INFINITY;
        }
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx *= c;                                                    // c > 0: max commutes with the scaling
    // mx covers the lane's 16 keys, i.e. half of its row's 32: the test below is the same over
    // half rows as over whole rows, so the two halves only meet (one cross-lane exchange) when the
    // reference really moves
    const bool raise = __any(mx > m + SOFTMAX_SLACK);           // m = -inf: any visible key raises it
    alpha = 1.0f;
    if (raise) {
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mn = fmaxf(m, mx);
        alpha = (mn == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - mn);   // m = -inf -> 0
        l *= alpha;
        m = mn;
    }
    const float mu = (m == -INFINITY) ? 0.f : m;               // row with nothing visible yet
    const f16x2 ones = {(f16)1.0f, (f16)1.0f};
    float ps = 0.f;
    u32x4 pw[2];
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[r], c, -mu));       // masked: -inf -> 0
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[r + 1], c, -mu));
        const auto h = __builtin_amdgcn_cvt_pkrtz(p0, p1);
        ps = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, h), ones, ps, false);
        pw[r >> 3][(r & 7) >> 1] = __builtin_bit_cast(unsigned, h);
    }
    pb[0] = __builtin_bit_cast(f16x8, pw[0]);
    pb[1] = __builtin_bit_cast(f16x8, pw[1]);
    l += ps;                                                    // the lane's half of the row; halves are added at the end
    return raise;
}

// Which (q-tile group, KV head, key slice) a workgroup works on.  Workgroups are dealt to the 8 XCDs round robin
// in launch order (x fastest), and each XCD has its own L2: with the plain blockIdx mapping the q-tile groups that
// read the SAME keys (same KV head, same slice) have consecutive ids and land on 8 different L2s, so every K/V
// byte crossed HBM once per group (measured 7.9x the cache's bytes on a 256-row extend, 2x on a verify step).
// Renumbered: XCD c takes the c-th eighth of the (head, slice, group) order, group fastest - all groups of one
// (head, slice) share one L2 and run at the same time, and so do the slices of one head, which all read that
// head's q rows (with 8 KV heads: one head per XCD; K, V and q each cross HBM once).
struct AttnWork { int tile, hk, split; };
__device__ __forceinline__ AttnWork attn_work() {
    const unsigned nx = gridDim.x, nz = gridDim.z, total = nx * gridDim.y * nz;
    unsigned id = blockIdx.x + nx * (blockIdx.y + gridDim.y * blockIdx.z);
    if ((total & 7u) == 0) id = (id & 7u) * (total >> 3) + (id >> 3);
    return {(int)(id % nx), (int)(id / (nx * nz)), (int)((id / nx) % nz)};
}

struct AttnArgs {
    const f16* q;
    f16* out;
    long long q_lo_off, out_lo_off;   // split activations: lo parts of q / out this many elements behind (0 = not split)
    KVGeom kv;
    int layer, Hq, n_splits;
    const int* tile_info;      // per q-tile group, 8 ints: seq, first stacked row, P, T, row0, block-table offset,
                               // key limit (0 = none: causal bound of the rows), first key
    const int* bt;
    float* partials;
    // shared-prefix pass of a many-sequence call (see launch_attention); unused otherwise
    const float* shared_partials;
    int shared_splits, shared_nq, shared_len;
};

// Everything a step needs from memory is requested as early as possible, because at verify
// sizes the kernel is a chain of dependent memory latencies, not a bandwidth problem: the tile
// record is one 32-byte load, the block-table entries of the whole key slice are fetched by
// one wavefront-wide load (and handed out with shuffles), and the K/V operands of step s + 1
// are in flight while step s is multiplied.
// QS: q comes as hi and lo parts (split activations): the score product takes both against the same K operand.
template <int HD, int NQ, bool QS = false>
__global__ __launch_bounds__(64) void attn_split_kernel(AttnArgs a) {
    constexpr int KQ = HD / 16;          // MFMA k-steps of the score product
    constexpr int NP = QS ? 2 : 1;
    constexpr int DT = HD / 32;          // 32-channel tiles of the output
    constexpr int PS = HD * 32 + 64;     // floats of one partial: O^T [HD][32], m[32], l[32]
    const AttnWork wk = attn_work();
    const int tile = wk.tile, hk = wk.hk, split = wk.split;
    const int lane = threadIdx.x, ql = lane & 31, g = lane >> 5;
    const int Hq = a.Hq, Hkv = a.kv.n_kv_heads, G = Hq / Hkv;
    const int4 ti0 = *(const int4*)(a.tile_info + tile * 8), ti1 = *(const int4*)(a.tile_info + tile * 8 + 4);
    const int r0 = ti0.y, P = ti0.z, T = ti0.w, row0 = ti1.x;
    const int n_stacked = T * G;
    const int* tab = a.bt + ti1.y;
    const int kv_len = P + T, last_blk = (kv_len - 1) >> 4;

    // keys this group can see at all: up to the position of its last valid row.  (Keys past the end of the
    // sequence, reached only by its last step, re-read the last valid K row - see fetch - and their scores are
    // replaced by -inf, so K is never read from unwritten slots; V is, and process() zeroes those operands.)
    const int r_last = min(r0 + NQ * 32 - 1, n_stacked - 1);
    const int kv_end = P + r_last / G + 1;
    const int first = ti1.w >> 5;                        // first key step (keys before it belong to the shared pass)
    const int steps = (kv_end + 31) / 32;
    const int per = (steps - first + a.n_splits - 1) / a.n_splits;
    const int s_lo = first + split * per, s_hi = min(steps, s_lo + per);

    // this lane's query rows (clamped rows compute garbage that is never written)
    int pos_q[NQ], pos_min[NQ];          // pos_min: earliest position among the tile's rows (uniform)
    f16x8 qf[NQ][NP][KQ];
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const int rq = min(r0 + t * 32 + ql, n_stacked - 1);
        const int tq = rq / G, gq = rq % G;
        pos_q[t] = P + tq;
        pos_min[t] = P + min(r0 + t * 32, n_stacked - 1) / G;
        const f16* qrow = a.q + ((long long)(row0 + tq) * Hq + hk * G + gq) * HD;
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int kk = 0; kk < KQ; ++kk) qf[t][p][kk] = *(const f16x8*)(qrow + (p ? a.q_lo_off : 0) + kk * 16 + g * 8);
    }

    const f16* Kp = (const f16*)a.kv.base + a.kv.plane(a.layer, 0, hk);
    const f16* Vp = (const f16*)a.kv.base + a.kv.plane(a.layer, 1, hk);

    const float c = 1.4426950408889634f / sqrtf((float)HD);   // log2(e) / sqrt(hd)
    float m[NQ], l[NQ];
    f32x16 o[NQ][DT];
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        m[t] = -INFINITY;
        l[t] = 0.f;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[t][d][r] = 0.f;
    }

    f16x8 kf[2][KQ];                     // K / V operands of the current and the next step
    f16x4 vq[2][DT][4];
    int tabv = 0;                        // block ids of steps [chunk, chunk + 32): lane i holds block 2*chunk + i
    auto fetch = [&](int buf, int st, int chunk) {
        const int kv0 = st * 32;
        const int key = min(kv0 + ql, kv_len - 1);
        const int kblk = __shfl(tabv, min(key >> 4, last_blk) - 2 * chunk, 64);
        const f16* krow = Kp + ((long long)kblk * 16 + (key & 15)) * HD + g * 8;
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) kf[buf][kk] = *(const f16x8*)(krow + kk * 16);
        const int b0 = __shfl(tabv, min(kv0 >> 4, last_blk) - 2 * chunk, 64);
        const int b1 = __shfl(tabv, min((kv0 >> 4) + 1, last_blk) - 2 * chunk, 64);
#pragma unroll
        for (int d = 0; d < DT; ++d) {
            const f16* v0 = Vp + ((long long)b0 * HD + d * 32 + ql) * 16 + g * 4;
            const f16* v1 = Vp + ((long long)b1 * HD + d * 32 + ql) * 16 + g * 4;
            vq[buf][d][0] = *(const f16x4*)v0;
            vq[buf][d][1] = *(const f16x4*)(v0 + 8);
            vq[buf][d][2] = *(const f16x4*)v1;
            vq[buf][d][3] = *(const f16x4*)(v1 + 8);
        }
    };
    auto process = [&](int buf, int st) {
        const int kv0 = st * 32;
        if (kv0 + 32 > kv_len) {
            // the sequence ends inside this step (its last one): slots of the last block past the end were never
            // written by this sequence and may hold anything - their V operands become exact zeros, so that a
            // probability of 0 times whatever lies in caller memory cannot turn into a NaN
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (kv0 + qd * 8 + g * 4 + i >= kv_len) vq[buf][d][qd][i] = (f16)0.f;
        }
#pragma unroll
        for (int t = 0; t < NQ; ++t) {
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KQ; ++kk)
#pragma unroll
                for (int p = 0; p < NP; ++p) s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[buf][kk], qf[t][p][kk], s, 0, 0, 0);
            float alpha;
            f16x8 pb[2];
            if (online_softmax_step(s, kv0, g, pos_q[t], kv0 + 31 > pos_min[t], c, m[t], l[t], alpha, pb)) {
#pragma unroll
                for (int d = 0; d < DT; ++d)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[t][d][r] *= alpha;
            }
#pragma unroll
            for (int d = 0; d < DT; ++d) {
                const f16x4 *v = vq[buf][d];
                const f16x8 va = {v[0][0], v[0][1], v[0][2], v[0][3], v[1][0], v[1][1], v[1][2], v[1][3]};
                const f16x8 vb = {v[2][0], v[2][1], v[2][2], v[2][3], v[3][0], v[3][1], v[3][2], v[3][3]};
                o[t][d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, pb[0], o[t][d], 0, 0, 0);
                o[t][d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vb, pb[1], o[t][d], 0, 0, 0);
            }
        }
    };

    for (int chunk = s_lo; chunk < s_hi; chunk += 32) {          // 32 steps = 64 blocks = one table load
        tabv = tab[min(2 * chunk + lane, last_blk)];
        const int c_hi = min(s_hi, chunk + 32);
        fetch(0, chunk, chunk);
        for (int st = chunk; st < c_hi; st += 2) {
            if (st + 1 < c_hi) fetch(1, st + 1, chunk);
            process(0, st);
            if (st + 1 < c_hi) {
                if (st + 2 < c_hi) fetch(0, st + 2, chunk);
                process(1, st + 1);
            }
        }
    }

    // partials of the group: NQ consecutive (O^T, m, l) records per (group, KV head, slice);
    // rows past the end of the sequence are not written (and never read)
    float l_row[NQ];
#pragma unroll
    for (int t = 0; t < NQ; ++t) l_row[t] = l[t] + __shfl_xor(l[t], 32, 64);    // both halves of each row
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        if (r0 + t * 32 + ql >= n_stacked) continue;
        float* part = a.partials + (((long long)(tile * Hkv + hk) * a.n_splits + split) * NQ + t) * PS;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ch = d * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
                part[ch * 32 + ql] = o[t][d][r];
            }
        if (g == 0) {
            part[HD * 32 + ql] = m[t];
            part[HD * 32 + 32 + ql] = l_row[t];
        }
    }
}

// ------------------------------------------------------------------------------ MFMA block kernel
// Long extends (many q tiles per KV head): a block of 4 wavefronts owns 4 consecutive q tiles
// (128 stacked rows) of one KV head and one key slice.  The K/V operands of a 32-key step are
// fetched once per block (one 16-byte chunk of K and one of V per thread and 64 channels of
// head_dim), staged through LDS and shared by the four tiles; global loads run D steps ahead in
// a register ring, LDS is double buffered, one barrier per step.  Everything after the operand
// fetch is the per-wavefront online softmax of attn_split_kernel; the partial records are those
// of a group of NQ = 4 tiles, merged by attn_combine_kernel<HD, 4>.
//
// LDS layout of a stage: K rows [32 keys][HD + 8] (padded, 16-byte operand reads are conflict
// free); V rows [2 blocks * HD channels][16 tokens in operand order + 8 pad], where operand order
// puts tokens {0-3, 8-11, 4-7, 12-15} so that a lane's PV operand (tokens 4g..4g+3 and
// 8+4g..8+4g+3 of its channel) is one 16-byte read.
template <int HD, int NQ, bool QS = false>
__global__ __launch_bounds__(64 * NQ) void attn_block_kernel(AttnArgs a) {
    constexpr int KQ = HD / 16, DT = HD / 32, PS = HD * 32 + 64, NT = 64 * NQ;
    constexpr int NP = QS ? 2 : 1;       // q in hi and lo parts (split activations)
    constexpr int D = 4;                              // prefetch distance in key steps (even)
    constexpr int KLS = HD + 8, VLS = 24;             // padded LDS row lengths (fp16 elements)
    constexpr int TCH = 32 * HD / 8;                  // 16-byte chunks of K (and of V) per step
    constexpr int CH = (TCH + NT - 1) / NT;           // ... per thread (threads past TCH idle)
    __shared__ __attribute__((aligned(16))) f16 sK[2][32 * KLS];
    __shared__ __attribute__((aligned(16))) f16 sV[2][2 * HD * VLS];

    const AttnWork wk = attn_work();
    const int tile = wk.tile, hk = wk.hk, split = wk.split;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ql = lane & 31, g = lane >> 5;
    const int Hq = a.Hq, Hkv = a.kv.n_kv_heads, G = Hq / Hkv;
    const int4 ti0 = *(const int4*)(a.tile_info + tile * 8), ti1 = *(const int4*)(a.tile_info + tile * 8 + 4);
    const int r0 = ti0.y, P = ti0.z, T = ti0.w, row0 = ti1.x;
    const int n_stacked = T * G;
    const int* tab = a.bt + ti1.y;
    const int klimit = ti1.z;                                  // > 0: keys [0, klimit) only (shared pass)
    const int kv_len = klimit > 0 ? klimit : P + T, last_blk = (kv_len - 1) >> 4;

    const int r_last = min(r0 + NQ * 32 - 1, n_stacked - 1);
    const int kv_end = klimit > 0 ? klimit : P + r_last / G + 1;
    const int steps = (kv_end + 31) / 32;
    const int per = (steps + a.n_splits - 1) / a.n_splits;
    const int s_lo = split * per, s_hi = min(steps, s_lo + per);

    // this wavefront's q tile
    const int rq = min(r0 + wave * 32 + ql, n_stacked - 1);
    const int tq = rq / G, gq = rq % G;
    const int pos_q = P + tq;
    const f16* qrow = a.q + ((long long)(row0 + tq) * Hq + hk * G + gq) * HD;
    f16x8 qf[NP][KQ];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) qf[p][kk] = *(const f16x8*)(qrow + (p ? a.q_lo_off : 0) + kk * 16 + g * 8);

    const f16* Kp = (const f16*)a.kv.base + a.kv.plane(a.layer, 0, hk);
    const f16* Vp = (const f16*)a.kv.base + a.kv.plane(a.layer, 1, hk);
    const float c = 1.4426950408889634f / sqrtf((float)HD);
    const int pos_tile_min = P + (r0 + wave * 32) / G;         // earliest position among this tile's rows
    float m = -INFINITY, l = 0.f, alpha_out = 1.f;
    f16x8 pb_out[2];
    f32x16 o[DT];
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] = 0.f;

    // operand chunks of this thread: K chunk i covers key (cidx / (HD/8)), columns 8*(cidx % (HD/8));
    // V chunk i covers block (cidx / (2*HD)), channel ((cidx / 2) % HD), tokens 8*(cidx % 2)..+7.
    // The 64 chunks of a wavefront lie inside ONE 16-token block of the step (8 or 4 whole keys of K,
    // half or a quarter of a V block), so which of the step's two blocks a chunk belongs to is
    // wavefront-uniform: the block ids are read out of the table register into scalars, the block's
    // base address is scalar arithmetic, and what is left per lane is a constant offset computed once.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    unsigned k_off[CH], v_off[CH];
    bool k_second[CH], v_second[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int cidx = min(tid + NT * i, TCH - 1), c0 = min(wave_u * 64 + NT * i, TCH - 1);
        k_off[i] = (unsigned)(((cidx / (HD / 8)) & 15) * HD + (cidx % (HD / 8)) * 8) * 2u;      // bytes
        v_off[i] = (unsigned)(((cidx / 2) % HD) * 16 + (cidx % 2) * 8) * 2u;
        k_second[i] = ((c0 / (HD / 8)) >> 4) != 0;
        v_second[i] = (c0 / (2 * HD)) != 0;
    }
    u32x4 rk[D][CH], rv[D][CH];
    // keys past the end of the sequence (last step only) read slots of the last block that were never
    // written, or the last block twice: their scores are replaced by -inf whatever they are, and
    // process() zeroes their V operands
    auto gload = [&](int slot, int st, int tabv, int chunk) {
        const int rel = 2 * (st - chunk), lim = last_blk - 2 * chunk;     // table lanes of the step's two blocks
        const int b0 = __builtin_amdgcn_readlane(tabv, min(rel, lim)), b1 = __builtin_amdgcn_readlane(tabv, min(rel + 1, lim));
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (TCH % NT != 0 && wave_u * 64 + NT * i >= TCH) continue;     // more threads than chunks: the rest load nothing
            const char* kb = (const char*)(Kp + (long long)(k_second[i] ? b1 : b0) * 16 * HD);
            const char* vb = (const char*)(Vp + (long long)(v_second[i] ? b1 : b0) * 16 * HD);
            rk[slot][i] = *(const u32x4*)(kb + k_off[i]);
            rv[slot][i] = *(const u32x4*)(vb + v_off[i]);
        }
    };
    auto lstore = [&](int slot, int buf) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int cidx = tid + NT * i;
            if (TCH % NT != 0 && cidx >= TCH) continue;
            *(u32x4*)(sK[buf] + (cidx / (HD / 8)) * KLS + (cidx % (HD / 8)) * 8) = rk[slot][i];
            // tokens 8h..8h+3 -> operand position 4h, tokens 8h+4..8h+7 -> operand position 8 + 4h
            const int vrow = (cidx / (2 * HD)) * HD + (cidx / 2) % HD, h = cidx % 2;
            uint2* dst = (uint2*)(sV[buf] + vrow * VLS);
            dst[h] = make_uint2(rv[slot][i][0], rv[slot][i][1]);
            dst[2 + h] = make_uint2(rv[slot][i][2], rv[slot][i][3]);
        }
    };
    auto process = [&](int buf, int st) {
        const int kv0 = st * 32;
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) {
            const f16x8 kf = *(const f16x8*)(sK[buf] + ql * KLS + kk * 16 + g * 8);
#pragma unroll
            for (int p = 0; p < NP; ++p) s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[p][kk], s, 0, 0, 0);
        }
        if (online_softmax_step(s, kv0, g, pos_q, kv0 + 31 > pos_tile_min, c, m, l, alpha_out, pb_out)) {
            const float alpha = alpha_out;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
        }
        const f16x8* pb = pb_out;
        const bool ragged = kv0 + 32 > kv_len;          // block-uniform: the sequence ends inside this step
#pragma unroll
        for (int d = 0; d < DT; ++d) {
            f16x8 va = *(const f16x8*)(sV[buf] + (d * 32 + ql) * VLS + g * 8);
            f16x8 vb = *(const f16x8*)(sV[buf] + (HD + d * 32 + ql) * VLS + g * 8);
            if (ragged) {
                // slots past the end of the sequence hold whatever the pool memory held: exact zeros instead, so
                // that their probability of 0 cannot meet a NaN or an infinity (element i of va is token
                // (i / 4) * 8 + 4 g + i % 4 of the step's first block, of vb the same of its second block)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int key = kv0 + (i >> 2) * 8 + g * 4 + (i & 3);
                    if (key >= kv_len) va[i] = (f16)0.f;
                    if (key + 16 >= kv_len) vb[i] = (f16)0.f;
                }
            }
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, pb[0], o[d], 0, 0, 0);
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vb, pb[1], o[d], 0, 0, 0);
        }
    };

    for (int chunk = s_lo; chunk < s_hi; chunk += 32) {          // 32 steps = 64 blocks = one table load
        const int tabv = tab[min(2 * chunk + lane, last_blk)];
        const int c_hi = min(s_hi, chunk + 32), n = c_hi - chunk;
#pragma unroll
        for (int u = 0; u < D; ++u)
            if (u < n) gload(u, chunk + u, tabv, chunk);
        lstore(0, 0);
        __syncthreads();
        int b = 0;
        for (; b + 2 * D <= n; b += D) {                         // steady state, branch free
#pragma unroll
            for (int u = 0; u < D; ++u) {
                gload(u, chunk + b + u + D, tabv, chunk);
                process(u & 1, chunk + b + u);
                lstore((u + 1) % D, (u + 1) & 1);
                __syncthreads();
            }
        }
        for (; b < n; b += D) {                                  // drain
#pragma unroll
            for (int u = 0; u < D; ++u) {
                const int i = b + u;
                if (i < n) {
                    if (i + D < n) gload(u, chunk + i + D, tabv, chunk);
                    process(u & 1, chunk + i);
                    if (i + 1 < n) lstore((u + 1) % D, (u + 1) & 1);
                    __syncthreads();
                }
            }
        }
    }

    const float l_row = l + __shfl_xor(l, 32, 64);               // both halves of the row
    if (r0 + wave * 32 + ql < n_stacked) {
        float* part = a.partials + (((long long)(tile * Hkv + hk) * a.n_splits + split) * NQ + wave) * PS;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ch = d * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
                part[ch * 32 + ql] = o[d][r];
            }
        if (g == 0) {
            part[HD * 32 + ql] = m;
            part[HD * 32 + 32 + ql] = l_row;
        }
    }
}

// Merges the key slices of one q tile.  grid (n_groups * Hkv * NQ, HD / 4), 256 threads =
// 32 query rows x 8 slice groups; a block produces 4 output channels.  A thread loads the
// (m, l, 4 channels) of its slices s = sg, sg + 8, ... in one go (up to 16 slices in registers),
// the row maximum and then the weighted sums meet in LDS.  With a shared-prefix pass the slices
// of that pass follow the tile's own: they live in the records of the shared pass's tile group
// that holds the row (rows of all sequences stacked: global row * G + g).
template <int HD, int NQ>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
    constexpr int PS = HD * 32 + 64;
    constexpr int MAXS = 16;                                   // slices per thread held in registers
    __shared__ float red[8][6][32];
    const int Hkv = a.kv.n_kv_heads, G = a.Hq / Hkv;
    const int t = blockIdx.x % NQ, hk = (blockIdx.x / NQ) % Hkv, tile = blockIdx.x / (NQ * Hkv);
    const int ch0 = blockIdx.y * 4;
    const int ql = threadIdx.x & 31, sg = threadIdx.x >> 5;
    const int4 ti0 = *(const int4*)(a.tile_info + tile * 8);
    const int row0 = a.tile_info[tile * 8 + 4];
    const int r_first = ti0.y + t * 32, n_stacked = ti0.w * G;
    if (r_first >= n_stacked) return;                          // whole q tile past the end (block-uniform)
    const int r = r_first + ql;
    const bool valid = r < n_stacked;
    const int own_splits = a.n_splits, n_splits = own_splits + a.shared_splits;
    const float* base = a.partials + ((long long)(tile * Hkv + hk) * own_splits * NQ + t) * PS + ql;
    const long long stride = (long long)NQ * PS;               // between slices
    const float* sbase = nullptr;                              // the row's record in the shared pass, slice 0
    long long sstride = 0;
    if (a.shared_splits > 0) {
        const int rc = min(r, n_stacked - 1), R = (row0 + rc / G) * G + rc % G, gsz = 32 * a.shared_nq;
        sbase = a.shared_partials + ((long long)((R / gsz) * Hkv + hk) * a.shared_splits * a.shared_nq + (R % gsz) / 32) * PS + (R & 31);
        sstride = (long long)a.shared_nq * PS;
    }
    auto slice = [&](int s) { return s < own_splits ? base + s * stride : sbase + (s - own_splits) * sstride; };

    float mv[MAXS], lv[MAXS], ov[MAXS][4];
    float mloc = -INFINITY;
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const int s = sg + 8 * i;
        mv[i] = -INFINITY;
        lv[i] = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) ov[i][c] = 0.f;
        if (valid && s < n_splits) {
            const float* p = slice(s);
            mv[i] = p[HD * 32];
            lv[i] = p[HD * 32 + 32];
#pragma unroll
            for (int c = 0; c < 4; ++c) ov[i][c] = p[(ch0 + c) * 32];
        }
    }
#pragma unroll
    for (int i = 0; i < MAXS; ++i) mloc = fmaxf(mloc, mv[i]);
    if (valid)                                                 // more than 128 slices: the rest from memory
        for (int s = sg + 8 * MAXS; s < n_splits; s += 8) mloc = fmaxf(mloc, slice(s)[HD * 32]);
    red[sg][0][ql] = mloc;
    __syncthreads();
    float M = red[0][0][ql];
#pragma unroll
    for (int i = 1; i < 8; ++i) M = fmaxf(M, red[i][0][ql]);   // finite: slice 0 always sees key 0
    __syncthreads();

    float l = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const float w = exp2f(mv[i] - M);                      // absent slices: 2^-inf = 0
        l += w * lv[i];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += w * ov[i][c];
    }
    if (valid)
        for (int s = sg + 8 * MAXS; s < n_splits; s += 8) {
            const float* p = slice(s);
            const float w = exp2f(p[HD * 32] - M);
            l += w * p[HD * 32 + 32];
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] += w * p[(ch0 + c) * 32];
        }
    red[sg][1][ql] = l;
#pragma unroll
    for (int c = 0; c < 4; ++c) red[sg][2 + c][ql] = acc[c];
    __syncthreads();
    if (sg >= 4 || !valid) return;                   // 128 threads finish: (channel sg, row ql)
    float L = 0.f, o = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { L += red[i][1][ql]; o += red[i][2 + sg][ql]; }
    f16* dst = a.out + ((long long)(row0 + r / G) * a.Hq + hk * G + r % G) * HD + ch0 + sg;
    const float res = o / L;
    const f16 hi = (f16)res;
    *dst = hi;
    if (a.out_lo_off) dst[a.out_lo_off] = (f16)(res - (float)hi);
}

// Slice merge for launches with many tile records and few slices each (the block kernel's groups
// of 4 or 8 tiles; single-tile launches over many sequences, with their shared-prefix slices).
// One block per (group, KV head, tile): 256 threads = 32 query rows x 8 channel groups, a thread
// owns HD/8 consecutive channels of its row and walks the slices itself, so nothing meets in
// LDS and every load of a pass is independent.  Pass 1: the row's reference exponents of all
// slices -> maximum.  Pass 2: weights 2^(m_s - M), weighted sums, one 16-byte (HD = 64) or
// 32-byte store of the normalised fp16 outputs.
template <int HD, int NQ>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
    constexpr int PS = HD * 32 + 64, CPT = HD / 8, SU = 4;
    const int Hkv = a.kv.n_kv_heads, G = a.Hq / Hkv;
    const int t = blockIdx.x % NQ, hk = (blockIdx.x / NQ) % Hkv, tile = blockIdx.x / (NQ * Hkv);
    const int ql = threadIdx.x & 31, cg = threadIdx.x >> 5;
    const int4 ti0 = *(const int4*)(a.tile_info + tile * 8);
    const int row0 = a.tile_info[tile * 8 + 4];
    const int r = ti0.y + t * 32 + ql, n_stacked = ti0.w * G;
    if (r >= n_stacked) return;
    const int own_splits = a.n_splits, n_splits = own_splits + a.shared_splits;
    const float* base = a.partials + ((long long)(tile * Hkv + hk) * own_splits * NQ + t) * PS + ql;
    const long long stride = (long long)NQ * PS;               // between slices
    const float* sbase = nullptr;                              // the row's record in a shared-prefix pass, slice 0
    long long sstride = 0;
    if (a.shared_splits > 0) {
        const int R = (row0 + r / G) * G + r % G, gsz = 32 * a.shared_nq;
        sbase = a.shared_partials + ((long long)((R / gsz) * Hkv + hk) * a.shared_splits * a.shared_nq + (R % gsz) / 32) * PS + (R & 31);
        sstride = (long long)a.shared_nq * PS;
    }
    auto slice = [&](int s) { return s < own_splits ? base + s * stride : sbase + (s - own_splits) * sstride; };

    float M = -INFINITY;
    for (int s0 = 0; s0 < n_splits; s0 += 8) {
        float mv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) mv[i] = s0 + i < n_splits ? slice(s0 + i)[HD * 32] : -INFINITY;
#pragma unroll
        for (int i = 0; i < 8; ++i) M = fmaxf(M, mv[i]);
    }                                                          // finite: slice 0 always sees its first key
    float L = 0.f, acc[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) acc[c] = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += SU) {
        float mv[SU], lv[SU], ov[SU][CPT];
#pragma unroll
        for (int i = 0; i < SU; ++i) {
            const float* p = slice(min(s0 + i, n_splits - 1));
            mv[i] = s0 + i < n_splits ? p[HD * 32] : -INFINITY;            // absent slice: weight 0
            lv[i] = p[HD * 32 + 32];
#pragma unroll
            for (int c = 0; c < CPT; ++c) ov[i][c] = p[(cg * CPT + c) * 32];
        }
#pragma unroll
        for (int i = 0; i < SU; ++i) {
            const float w = exp2f(mv[i] - M);
            L += w * lv[i];
#pragma unroll
            for (int c = 0; c < CPT; ++c) acc[c] += w * ov[i][c];
        }
    }
    const float inv = 1.0f / L;
    f16* dst = a.out + ((long long)(row0 + r / G) * a.Hq + hk * G + r % G) * HD + cg * CPT;
#pragma unroll
    for (int c0 = 0; c0 < CPT; c0 += 8) {
        f16x8 v, lo;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float ov = acc[c0 + c] * inv;
            v[c] = (f16)ov;
            lo[c] = (f16)(ov - (float)v[c]);
        }
        *(f16x8*)(dst + c0) = v;
        if (a.out_lo_off) *(f16x8*)(dst + a.out_lo_off + c0) = lo;
    }
}

size_t attention_partial_floats(int n_tiles, int n_kv_heads, int head_dim, int n_splits) {
    return (size_t)n_tiles * n_kv_heads * n_splits * ((size_t)head_dim * 32 + 64);
}

template <int HD, int NQ>
static void launch_attn_mfma(const AttnArgs& a, int n_groups, hipStream_t s) {
    dim3 grid(n_groups, a.kv.n_kv_heads, a.n_splits), cgrid(n_groups * a.kv.n_kv_heads * NQ, HD / 4);
    if (a.q_lo_off) attn_split_kernel<HD, NQ, true><<<grid, 64, 0, s>>>(a);
    else attn_split_kernel<HD, NQ, false><<<grid, 64, 0, s>>>(a);
    // few records with many slices (one session): blocks of 4 channels that spread the slices over
    // threads; many records with few slices (many sessions): one block per record
    if (n_groups * a.kv.n_kv_heads >= 64 && a.n_splits + a.shared_splits <= 32)
        attn_merge_kernel<HD, NQ><<<n_groups * a.kv.n_kv_heads * NQ, 256, 0, s>>>(a);
    else
        attn_combine_kernel<HD, NQ><<<cgrid, 256, 0, s>>>(a);
}

template <int HD, int NQ>
static void launch_attn_block(const AttnArgs& a, dim3 grid, hipStream_t s) {
    if (a.q_lo_off) attn_block_kernel<HD, NQ, true><<<grid, 64 * NQ, 0, s>>>(a);
    else attn_block_kernel<HD, NQ, false><<<grid, 64 * NQ, 0, s>>>(a);
}

void launch_attention(DType dt, const void* q, void* out, KVGeom kv, int layer, const StepView& sv,
                      int n_q_heads, float* partials, int n_splits, hipStream_t s, long long q_lo_off,
                      long long out_lo_off) {
    if (dt == F32) {
        dim3 grid(sv.n_rows, n_q_heads);
        attn_simple_kernel<float, 256><<<grid, 64, 0, s>>>((const float*)q, (float*)out, kv, layer,
                                                           sv.row_pos, sv.row_seq, sv.seq_bt, sv.bt,
                                                           n_q_heads);
        return;
    }
    AttnArgs a{};
    a.q = (const f16*)q; a.out = (f16*)out; a.kv = kv; a.layer = layer; a.Hq = n_q_heads; a.n_splits = n_splits;
    a.tile_info = sv.tile_info; a.bt = sv.bt; a.partials = partials;
    a.q_lo_off = q_lo_off; a.out_lo_off = out_lo_off;
    const int hd = kv.head_dim;
    if (sv.tile_nq >= 4) {                                     // long extends: 4 or 8 tiles per block, K/V through LDS
        dim3 grid(sv.n_tiles, kv.n_kv_heads, n_splits);
        const unsigned mgrid = (unsigned)(sv.n_tiles * kv.n_kv_heads * sv.tile_nq);
        if (sv.tile_nq == 4) {
            if (hd == 64) {
                launch_attn_block<64, 4>(a, grid, s);
                attn_merge_kernel<64, 4><<<mgrid, 256, 0, s>>>(a);
            } else {
                launch_attn_block<128, 4>(a, grid, s);
                attn_merge_kernel<128, 4><<<mgrid, 256, 0, s>>>(a);
            }
        } else {
            if (hd == 64) {
                launch_attn_block<64, 8>(a, grid, s);
                attn_merge_kernel<64, 8><<<mgrid, 256, 0, s>>>(a);
            } else {
                launch_attn_block<128, 8>(a, grid, s);
                attn_merge_kernel<128, 8><<<mgrid, 256, 0, s>>>(a);
            }
        }
    } else {
        if (sv.n_tiles_shared > 0) {
            // Many sequences that share a cached prefix (the same leading blocks): the keys of the
            // prefix are applied ONCE to the rows of all sequences - a pass of the block kernel over
            // one virtual sequence made of every row of the call, keys [0, shared_len), no causal
            // mask needed - instead of being pulled from L2 once per sequence; the per-sequence
            // wavefronts below start at shared_len, and the merge adds the shared pass's slices.
            AttnArgs sh = a;
            sh.tile_info = sv.tile_info + (size_t)sv.n_tiles * 8;
            sh.n_splits = sv.shared_splits;
            sh.partials = partials + attention_partial_floats(sv.n_tiles, kv.n_kv_heads, hd, n_splits);
            dim3 grid(sv.n_tiles_shared, kv.n_kv_heads, sv.shared_splits);
            if (sv.shared_nq == 4) {
                if (hd == 64) launch_attn_block<64, 4>(sh, grid, s); else launch_attn_block<128, 4>(sh, grid, s);
            } else {
                if (hd == 64) launch_attn_block<64, 8>(sh, grid, s); else launch_attn_block<128, 8>(sh, grid, s);
            }
            a.shared_partials = sh.partials;
            a.shared_splits = sv.shared_splits;
            a.shared_nq = sv.shared_nq;
            a.shared_len = sv.shared_len;
        }
        if (hd == 64) launch_attn_mfma<64, 1>(a, sv.n_tiles, s); else launch_attn_mfma<128, 1>(a, sv.n_tiles, s);
    }
}

}  // namespace ax
