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
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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
// One wavefront = one (q tile of 32 stacked rows, KV head, key slice).
//
// S^T = K * Q^T is computed so that the score tile comes out with lane <-> query row
// (column l % 32) and registers <-> keys: register r of lane l is key (r/4)*8 + (l/32)*4 + r%4
// of the 32-key step.  Row max / sum therefore need the 16 registers of the lane plus one
// exchange with lane ^ 32, and the softmax rescale is a per-lane scalar.  The probabilities
// are already laid out as the B operand of O^T = V^T * P^T: registers 0..7 cover keys
// {4g..4g+3, 8+4g..8+4g+3} of the first 16-key block, registers 8..15 the same of the second
// block (g = l/32).  V pages are token-minor ([head_dim][16]), so the matching A operand of a
// lane (channel d) is two 8-byte loads from its channel's 16-token row.
template <int HD>
__global__ __launch_bounds__(64) void attn_split_kernel(const f16* __restrict__ q, KVGeom kv, int layer,
                                                        const int* __restrict__ seq_P,
                                                        const int* __restrict__ seq_T,
                                                        const int* __restrict__ seq_row0,
                                                        const int* __restrict__ seq_bt,
                                                        const int* __restrict__ bt,
                                                        const int* __restrict__ tile_seq,
                                                        const int* __restrict__ tile_r0, int Hq,
                                                        float* __restrict__ partials, int n_splits) {
    constexpr int KQ = HD / 16;          // MFMA k-steps of the score product
    constexpr int DT = HD / 32;          // 32-channel tiles of the output
    const int tile = blockIdx.x, hk = blockIdx.y, split = blockIdx.z;
    const int lane = threadIdx.x, ql = lane & 31, g = lane >> 5;
    const int Hkv = kv.n_kv_heads, G = Hq / Hkv;
    const int sq = tile_seq[tile], r0 = tile_r0[tile];
    const int P = seq_P[sq], T = seq_T[sq], row0 = seq_row0[sq];
    const int n_stacked = T * G;
    const int* tab = bt + seq_bt[sq];
    const int kv_len = P + T;

    // keys this tile can see at all: up to the position of its last valid row
    const int r_last = min(r0 + 31, n_stacked - 1);
    const int kv_end = P + r_last / G + 1;
    const int steps = (kv_end + 31) / 32;
    const int per = (steps + n_splits - 1) / n_splits;
    const int s_lo = split * per, s_hi = min(steps, s_lo + per);

    // this lane's query row (clamped rows compute garbage that is never written)
    const int rq = min(r0 + ql, n_stacked - 1);
    const int tq = rq / G, gq = rq % G;
    const int pos_q = P + tq;
    const f16* qrow = q + ((long long)(row0 + tq) * Hq + hk * G + gq) * HD;
    f16x8 qf[KQ];
#pragma unroll
    for (int kk = 0; kk < KQ; ++kk) qf[kk] = *(const f16x8*)(qrow + kk * 16 + g * 8);

    const f16* Kp = (const f16*)kv.base + kv.plane(layer, 0, hk);
    const f16* Vp = (const f16*)kv.base + kv.plane(layer, 1, hk);

    const float c = 1.4426950408889634f / sqrtf((float)HD);   // log2(e) / sqrt(hd)
    float m = -INFINITY, l = 0.f;
    f32x16 o[DT];
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] = 0.f;

    for (int st = s_lo; st < s_hi; ++st) {
        const int kv0 = st * 32;
        // K rows: this lane supplies key kv0 + ql (clamped into the sequence)
        const int key = min(kv0 + ql, kv_len - 1);
        const f16* krow = Kp + ((long long)tab[key >> 4] * 16 + (key & 15)) * HD + g * 8;
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) {
            const f16x8 kf = *(const f16x8*)(krow + kk * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[kk], s, 0, 0, 0);
        }
        // V operands: channel (d*32 + ql) of blocks kv0/16 and kv0/16 + 1
        const int b0 = tab[min(kv0 >> 4, (kv_len - 1) >> 4)];
        const int b1 = tab[min((kv0 >> 4) + 1, (kv_len - 1) >> 4)];
        f16x8 vf[DT][2];
#pragma unroll
        for (int d = 0; d < DT; ++d) {
            const f16* v0 = Vp + ((long long)b0 * HD + d * 32 + ql) * 16 + g * 4;
            const f16* v1 = Vp + ((long long)b1 * HD + d * 32 + ql) * 16 + g * 4;
            const f16x4 a0 = *(const f16x4*)v0, a1 = *(const f16x4*)(v0 + 8);
            const f16x4 c0 = *(const f16x4*)v1, c1 = *(const f16x4*)(v1 + 8);
            vf[d][0] = (f16x8){a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
            vf[d][1] = (f16x8){c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
        }
        // causal mask + online softmax (base-2 exponentials)
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kj = kv0 + (r >> 2) * 8 + g * 4 + (r & 3);
            s[r] = (kj <= pos_q) ? s[r] * c : -INFINITY;
            mx = fmaxf(mx, s[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mn = fmaxf(m, mx);
        const float mu = (mn == -INFINITY) ? 0.f : mn;        // row with nothing visible yet
        const float alpha = exp2f(m - mu);                    // m = -inf -> 0
        float ps = 0.f;
        f16x8 pb[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float p = exp2f(s[r] - mu);                 // masked -> 0
            ps += p;
            pb[r >> 3][r & 7] = (f16)p;
        }
        ps += __shfl_xor(ps, 32, 64);
        l = l * alpha + ps;
        m = mn;
#pragma unroll
        for (int d = 0; d < DT; ++d) {
#pragma unroll
            for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[d][0], pb[0], o[d], 0, 0, 0);
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[d][1], pb[1], o[d], 0, 0, 0);
        }
    }

    // partial layout per (tile, hk, split): O^T [HD][32] floats, then m[32], l[32] (base-2 domain)
    float* part = partials + ((long long)(tile * Hkv + hk) * n_splits + split) * (HD * 32 + 64);
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ch = d * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
            part[ch * 32 + ql] = o[d][r];
        }
    if (g == 0) {
        part[HD * 32 + ql] = m;
        part[HD * 32 + 32 + ql] = l;
    }
}

// Merges the key slices of one (tile, KV head).  grid (n_tiles * Hkv, HD / 4), 256 threads =
// 32 query rows x 8 slice groups; a block produces 4 output channels.  Each thread folds the
// slices s = sg, sg + 8, ... (weights 2^(m_s - M)), the 8 groups meet in LDS.
template <int HD>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float* __restrict__ partials,
                                                           f16* __restrict__ out,
                                                           const int* __restrict__ seq_T,
                                                           const int* __restrict__ seq_row0,
                                                           const int* __restrict__ tile_seq,
                                                           const int* __restrict__ tile_r0, int Hq,
                                                           int Hkv, int n_splits) {
    constexpr int PS = HD * 32 + 64;                 // floats per partial
    __shared__ float red[8][6][32];
    const int tile = blockIdx.x / Hkv, hk = blockIdx.x % Hkv, ch0 = blockIdx.y * 4;
    const int ql = threadIdx.x & 31, sg = threadIdx.x >> 5;
    const float* base = partials + (long long)(tile * Hkv + hk) * n_splits * PS;

    float mloc = -INFINITY;
    for (int s = sg; s < n_splits; s += 8) mloc = fmaxf(mloc, base[(long long)s * PS + HD * 32 + ql]);
    red[sg][0][ql] = mloc;
    __syncthreads();
    float M = red[0][0][ql];
#pragma unroll
    for (int i = 1; i < 8; ++i) M = fmaxf(M, red[i][0][ql]);   // finite: slice 0 always sees key 0
    __syncthreads();

    float l = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = sg; s < n_splits; s += 8) {
        const float* p = base + (long long)s * PS;
        const float w = exp2f(p[HD * 32 + ql] - M);
        l += w * p[HD * 32 + 32 + ql];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += w * p[(ch0 + c) * 32 + ql];
    }
    red[sg][1][ql] = l;
#pragma unroll
    for (int c = 0; c < 4; ++c) red[sg][2 + c][ql] = acc[c];
    __syncthreads();
    if (sg >= 4) return;                             // 128 threads finish: (channel sg, row ql)
    const int G = Hq / Hkv;
    const int sq = tile_seq[tile], r = tile_r0[tile] + ql;
    if (r >= seq_T[sq] * G) return;
    float L = 0.f, o = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { L += red[i][1][ql]; o += red[i][2 + sg][ql]; }
    out[((long long)(seq_row0[sq] + r / G) * Hq + hk * G + r % G) * HD + ch0 + sg] = (f16)(o / L);
}

size_t attention_partial_floats(int n_tiles, int n_kv_heads, int head_dim, int n_splits) {
    return (size_t)n_tiles * n_kv_heads * n_splits * ((size_t)head_dim * 32 + 64);
}

void launch_attention(DType dt, const void* q, void* out, KVGeom kv, int layer, const StepView& sv,
                      int n_q_heads, float* partials, int n_splits, hipStream_t s) {
    if (dt == F32) {
        dim3 grid(sv.n_rows, n_q_heads);
        attn_simple_kernel<float, 256><<<grid, 64, 0, s>>>((const float*)q, (float*)out, kv, layer,
                                                           sv.row_pos, sv.row_seq, sv.seq_bt, sv.bt,
                                                           n_q_heads);
        return;
    }
    dim3 grid(sv.n_tiles, kv.n_kv_heads, n_splits), cgrid(sv.n_tiles * kv.n_kv_heads, kv.head_dim / 4);
    if (kv.head_dim == 64) {
        attn_split_kernel<64><<<grid, 64, 0, s>>>((const f16*)q, kv, layer, sv.seq_P, sv.seq_T,
                                                  sv.seq_row0, sv.seq_bt, sv.bt, sv.tile_seq,
                                                  sv.tile_r0, n_q_heads, partials, n_splits);
        attn_combine_kernel<64><<<cgrid, 256, 0, s>>>(partials, (f16*)out, sv.seq_T, sv.seq_row0,
                                                      sv.tile_seq, sv.tile_r0, n_q_heads,
                                                      kv.n_kv_heads, n_splits);
    } else {
        attn_split_kernel<128><<<grid, 64, 0, s>>>((const f16*)q, kv, layer, sv.seq_P, sv.seq_T,
                                                   sv.seq_row0, sv.seq_bt, sv.bt, sv.tile_seq,
                                                   sv.tile_r0, n_q_heads, partials, n_splits);
        attn_combine_kernel<128><<<cgrid, 256, 0, s>>>(partials, (f16*)out, sv.seq_T, sv.seq_row0,
                                                       sv.tile_seq, sv.tile_r0, n_q_heads,
                                                       kv.n_kv_heads, n_splits);
    }
}

}  // namespace ax
