// Small memory-bound kernels of the extend forward: embedding gather, RMSNorm, rotary + paged
// KV append, vocabulary argmax, greedy draft acceptance, copy-on-write block copy.
#include "kernels.h"

namespace ax {

typedef __bf16 bf16;
typedef _Float16 f16;     // activation and KV-cache type of bf16-weight models

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
__device__ __forceinline__ float to_f32(f16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // RNE
template <> __device__ __forceinline__ f16 from_f32<f16>(float v) { return (f16)v; }     // RNE

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---------------------------------------------------------------- embedding gather
template <typename T>
__global__ void embed_kernel(const T* __restrict__ emb, const int* __restrict__ row_tok,
                             float* __restrict__ x, int d) {
    const int r = blockIdx.x;
    const T* src = emb + (long long)row_tok[r] * d;
    float* dst = x + (long long)r * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) dst[c] = to_f32(src[c]);
}

void launch_embed(DType dt, const void* emb, const int* row_tok, float* x, int n_rows, int d,
                  hipStream_t s) {
    if (dt == F32)
        embed_kernel<float><<<n_rows, 256, 0, s>>>((const float*)emb, row_tok, x, d);
    else
        embed_kernel<bf16><<<n_rows, 256, 0, s>>>((const bf16*)emb, row_tok, x, d);
}

// Embedding gather that also prepares the first RMSNorm of bf16-weight models: the fp16 copy
// scaled by the norm gain and the row's sum of squares (in partial 0; the other partials are
// zeroed so that the row looks like the output of a GEMM with `nparts` column blocks).
__global__ void embed_norm_kernel(const bf16* __restrict__ emb, const int* __restrict__ row_tok,
                                  const bf16* __restrict__ gain, float* __restrict__ x,
                                  f16* __restrict__ a, long long a_lo_off, float* __restrict__ ssq, int nparts, int d) {
    __shared__ float part[4];
    const int r = blockIdx.x;
    const bf16* src = emb + (long long)row_tok[r] * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) {
        const float v = (float)src[c];
        x[(long long)r * d + c] = v;
        const float av = v * (float)gain[c];
        const f16 hi = (f16)av;
        a[(long long)r * d + c] = hi;
        if (a_lo_off) a[(long long)r * d + c + a_lo_off] = (f16)(av - (float)hi);     // split activations: the rounding remainder
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    for (int p = threadIdx.x; p < nparts; p += 256)
        ssq[(long long)r * nparts + p] = p == 0 ? part[0] + part[1] + part[2] + part[3] : 0.f;
}

void launch_embed_norm(const void* emb, const int* row_tok, const void* gain, float* x, void* a, long long a_lo_off,
                       float* ssq, int nparts, int n_rows, int d, hipStream_t s) {
    embed_norm_kernel<<<n_rows, 256, 0, s>>>((const bf16*)emb, row_tok, (const bf16*)gain, x, (f16*)a, a_lo_off, ssq,
                                             nparts, d);
}

// ---------------------------------------------------------------- RMSNorm
// One 256-thread block per row: sum of squares in fp32 (wavefront shuffles, then LDS across the
// four wavefronts), then x * rsqrt(mean + eps) * gain.
template <typename TG, typename T>
__global__ void rmsnorm_kernel(const float* __restrict__ x, const TG* __restrict__ gain,
                               T* __restrict__ h, const int* __restrict__ rows, int d, float eps) {
    __shared__ float part[4];
    const int i = blockIdx.x;
    const int r = rows ? rows[i] : i;
    const float* xr = x + (long long)r * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) {
        float v = xr[c];
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    T* hr = h + (long long)i * d;
    for (int c = threadIdx.x; c < d; c += 256) hr[c] = from_f32<T>(xr[c] * inv * to_f32(gain[c]));
}

void launch_rmsnorm(DType dt, const float* x, const void* gain, void* h, const int* rows,
                    int n_rows, int d, float eps, hipStream_t s) {
    if (dt == F32)
        rmsnorm_kernel<float, float><<<n_rows, 256, 0, s>>>(x, (const float*)gain, (float*)h, rows, d, eps);
    else
        rmsnorm_kernel<bf16, f16><<<n_rows, 256, 0, s>>>(x, (const bf16*)gain, (f16*)h, rows, d, eps);
}

// ---------------------------------------------------------------- rotary + paged KV append
// grid (n_rows, Hq + 2*Hkv); one block per (row, head).  Pair (j, j + hd/2) is rotated by
// the angle pos * base^(-2j/hd); cos / sin come from a host-built table [max_pos][hd/2].
template <typename T>
__global__ void rope_kv_kernel(const float* __restrict__ qkv, T* __restrict__ q_out, KVGeom kv,
                               int layer, const int* __restrict__ row_pos,
                               const int* __restrict__ row_seq, const int* __restrict__ seq_bt,
                               const int* __restrict__ bt, const float* __restrict__ rope_cos,
                               const float* __restrict__ rope_sin, int Hq) {
    const int r = blockIdx.x, head = blockIdx.y;
    const int hd = kv.head_dim, half = hd >> 1, Hkv = kv.n_kv_heads, B = kv.block_tokens;
    const int pos = row_pos[r];
    const float* src = qkv + (long long)r * (Hq + 2 * Hkv) * hd + (long long)head * hd;
    T* pool = (T*)kv.base;
    if (head < Hq + Hkv) {
        const float* cs = rope_cos + (long long)pos * half;
        const float* sn = rope_sin + (long long)pos * half;
        T* dst;
        if (head < Hq) {
            dst = q_out + ((long long)r * Hq + head) * hd;
        } else {
            const int blk = bt[seq_bt[row_seq[r]] + pos / B];
            dst = pool + kv.plane(layer, 0, head - Hq) + ((long long)blk * B + pos % B) * hd;
        }
        for (int j = threadIdx.x; j < half; j += blockDim.x) {
            const float a = src[j], b = src[j + half], c = cs[j], sgn = sn[j];
            dst[j] = from_f32<T>(a * c - b * sgn);
            dst[j + half] = from_f32<T>(b * c + a * sgn);
        }
    } else {
        const int blk = bt[seq_bt[row_seq[r]] + pos / B];
        T* dst = pool + kv.plane(layer, 1, head - Hq - Hkv) + (long long)blk * B * hd + pos % B;
        for (int c = threadIdx.x; c < hd; c += blockDim.x) dst[(long long)c * B] = from_f32<T>(src[c]);
    }
}

void launch_rope_kv(DType dt, const float* qkv, void* q_out, KVGeom kv, int layer,
                    const StepView& sv, const float* rope_cos, const float* rope_sin,
                    int n_q_heads, hipStream_t s) {
    dim3 grid(sv.n_rows, n_q_heads + 2 * kv.n_kv_heads);
    if (dt == F32)
        rope_kv_kernel<float><<<grid, 64, 0, s>>>(qkv, (float*)q_out, kv, layer, sv.row_pos, sv.row_seq,
                                                  sv.seq_bt, sv.bt, rope_cos, rope_sin, n_q_heads);
    else
        rope_kv_kernel<f16><<<grid, 64, 0, s>>>(qkv, (f16*)q_out, kv, layer, sv.row_pos, sv.row_seq,
                                                 sv.seq_bt, sv.bt, rope_cos, rope_sin, n_q_heads);
}

// ---------------------------------------------------------------- vocabulary argmax
// Two stages.  Order is (value descending, index ascending): ties go to the lowest id.
__device__ __forceinline__ void argmax_merge(float& bv, int& bi, float v, int i) {
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

__device__ __forceinline__ void argmax_wave(float& bv, int& bi) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float v = __shfl_xor(bv, o, 64);
        int i = __shfl_xor(bi, o, 64);
        argmax_merge(bv, bi, v, i);
    }
}

__global__ void argmax_stage1(const float* __restrict__ logits, int V, float* __restrict__ pv,
                              int* __restrict__ pi) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int r = blockIdx.y, part = blockIdx.x;
    const int span = (V + ARGMAX_PARTS - 1) / ARGMAX_PARTS;
    const int lo = part * span, hi = min(V, lo + span);
    const float* row = logits + (long long)r * V;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int c = lo + threadIdx.x; c < hi; c += 256) argmax_merge(bv, bi, row[c], c);
    argmax_wave(bv, bi);
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) argmax_merge(bv, bi, sv[w], si[w]);
        pv[r * ARGMAX_PARTS + part] = bv;
        pi[r * ARGMAX_PARTS + part] = bi;
    }
}

__global__ void argmax_stage2(const float* __restrict__ pv, const int* __restrict__ pi,
                              int* __restrict__ out) {
    const int r = blockIdx.x;
    float bv = pv[r * ARGMAX_PARTS + threadIdx.x];
    int bi = pi[r * ARGMAX_PARTS + threadIdx.x];
    argmax_wave(bv, bi);
    if (threadIdx.x == 0) out[r] = bi;
}

void launch_argmax(const float* logits, int rows, int V, int* out, int* scratch, hipStream_t s) {
    static_assert(ARGMAX_PARTS == 64, "stage 2 is one wavefront");
    float* pv = (float*)scratch;
    int* pi = scratch + (size_t)rows * ARGMAX_PARTS;
    argmax_stage1<<<dim3(ARGMAX_PARTS, rows), 256, 0, s>>>(logits, V, pv, pi);
    argmax_stage2<<<rows, 64, 0, s>>>(pv, pi, out);
}

// ---------------------------------------------------------------- greedy draft acceptance
// One wavefront per sequence: its rows are [pending, drafts...], g holds the greedy token after
// each row.  Lane i < k votes drafts[i] == g[i]; the accepted length is the position of the
// first lane whose vote is false (ballot + find-first-set).
__global__ void accept_kernel(const int* __restrict__ g, const int* __restrict__ row_tok,
                              const int* __restrict__ seq_row0, const int* __restrict__ seq_T,
                              int* __restrict__ result) {
    const int lane = threadIdx.x, s = blockIdx.x;
    const int row0 = seq_row0[s], k = seq_T[s] - 1;
    int a = 0;
    for (int base = 0; base < k; base += 64) {           // k > 64 only in principle
        const int i = base + lane;
        const bool ok = (i < k) && (row_tok[row0 + 1 + i] == g[row0 + i]);
        const unsigned long long mism = ~__ballot(ok);
        const int first_bad = __ffsll((long long)mism) - 1;   // 0..63, or -1 if none
        if (first_bad >= 0) { a = base + first_bad; break; }
        a = base + 64;
    }
    if (a > k) a = k;
    if (lane == 0) { result[2 * s] = a; result[2 * s + 1] = g[row0 + a]; }
}

void launch_accept(const int* g, const StepView& sv, int* result, hipStream_t s) {
    accept_kernel<<<sv.n_seq, 64, 0, s>>>(g, sv.row_tok, sv.seq_row0, sv.seq_T, result);
}

// Stage 2 of the argmax and the acceptance in one launch (a verify step is a chain of launches
// that each cost a few microseconds whatever they do).  Block = one sequence, 16 wavefronts:
// wavefront w finishes rows w, w + 16, .. from their stage-1 candidates, the greedy tokens meet
// in LDS, wavefront 0 votes as accept_kernel does.
__global__ __launch_bounds__(1024) void argmax_accept_kernel(const float* __restrict__ pv, const int* __restrict__ pi,
                                                             int* __restrict__ g, const int* __restrict__ row_tok,
                                                             const int* __restrict__ seq_row0,
                                                             const int* __restrict__ seq_T, int* __restrict__ result,
                                                             int* __restrict__ result_host) {
    __shared__ int s_g[ACCEPT_MAX_ROWS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, s = blockIdx.x;
    const int row0 = seq_row0[s], T = seq_T[s], k = T - 1;
    for (int i = wave; i < T; i += 16) {
        float bv = pv[(long long)(row0 + i) * ARGMAX_PARTS + lane];
        int bi = pi[(long long)(row0 + i) * ARGMAX_PARTS + lane];
        argmax_wave(bv, bi);
        if (lane == 0) { s_g[i] = bi; g[row0 + i] = bi; }
    }
    __syncthreads();
    if (wave != 0) return;
    int a = 0;
    for (int base = 0; base < k; base += 64) {
        const int i = base + lane;
        const bool ok = (i < k) && (row_tok[row0 + 1 + i] == s_g[i]);
        const unsigned long long mism = ~__ballot(ok);
        const int first_bad = __ffsll((long long)mism) - 1;
        if (first_bad >= 0) { a = base + first_bad; break; }
        a = base + 64;
    }
    if (a > k) a = k;
    if (lane == 0) {
        const int next = s_g[a];
        result[2 * s] = a;
        result[2 * s + 1] = next;
        if (result_host) { result_host[2 * s] = a; result_host[2 * s + 1] = next; }
    }
}

void launch_argmax_partials(const float* logits, int rows, int V, int* scratch, hipStream_t s) {
    argmax_stage1<<<dim3(ARGMAX_PARTS, rows), 256, 0, s>>>(logits, V, (float*)scratch, scratch + (size_t)rows * ARGMAX_PARTS);
}

void launch_argmax_accept(const int* scratch, int rows, int* g, const StepView& sv, int* result, int* result_host,
                          hipStream_t s) {
    argmax_accept_kernel<<<sv.n_seq, 1024, 0, s>>>((const float*)scratch, scratch + (size_t)rows * ARGMAX_PARTS, g,
                                                   sv.row_tok, sv.seq_row0, sv.seq_T, result, result_host);
}

// ---------------------------------------------------------------- copy-on-write block copy
// grid = 2 * n_layers * Hkv planes; each block copies B*hd elements of one plane as 16-byte
// words (B*hd*itemsize is a multiple of 16 for every supported shape).
__global__ void block_copy_kernel(char* __restrict__ base, long long plane_bytes,
                                  long long block_bytes, int src, int dst) {
    const uint4* s = (const uint4*)(base + blockIdx.x * plane_bytes + (long long)src * block_bytes);
    uint4* d = (uint4*)(base + blockIdx.x * plane_bytes + (long long)dst * block_bytes);
    for (int i = threadIdx.x; i < block_bytes / 16; i += blockDim.x) d[i] = s[i];
}

// ---------------------------------------------------------------- KV image <-> pages
// An image holds a sequence's blocks in logical order; block record b is
// [plane (layer, K|V, kv head)][block_tokens * hd elements] exactly as a block lies in the pool.
// grid = (planes, blocks of the sequence); 16-byte words.  On export the slots of the last
// block at or beyond `last_fill` are written as zero, so an image is a function of the cached
// values only.
template <bool TO_IMAGE>
__global__ void kv_image_kernel(char* __restrict__ pool, long long plane_bytes, int block_bytes,
                                const int* __restrict__ ids, char* __restrict__ image, int n_kv_heads,
                                int hd, int isz, int last_fill) {
    const int p = blockIdx.x, b = blockIdx.y, n_planes = gridDim.x;
    char* pg = pool + p * plane_bytes + (long long)ids[b] * block_bytes;
    char* im = image + ((long long)b * n_planes + p) * block_bytes;
    if (TO_IMAGE && b == (int)gridDim.y - 1 && last_fill < 16) {
        const bool is_v = (p / n_kv_heads) & 1;             // V pages are [hd][slot], K pages [slot][hd]
        const int n_el = block_bytes / isz;
        for (int e = threadIdx.x; e < n_el; e += blockDim.x) {
            const int slot = is_v ? (e & 15) : e / hd;
            if (isz == 2) ((unsigned short*)im)[e] = slot < last_fill ? ((const unsigned short*)pg)[e] : (unsigned short)0;
            else ((unsigned*)im)[e] = slot < last_fill ? ((const unsigned*)pg)[e] : 0u;
        }
        return;
    }
    const uint4* src = (const uint4*)(TO_IMAGE ? pg : im);
    uint4* dst = (uint4*)(TO_IMAGE ? im : pg);
    for (int i = threadIdx.x; i < block_bytes / 16; i += blockDim.x) dst[i] = src[i];
}

void launch_kv_image(bool to_image, DType dt, KVGeom kv, int n_layers, const int* ids, int n_seq_blocks,
                     void* image, int last_fill, hipStream_t s) {
    const int isz = dt == F32 ? 4 : 2;
    const int block_bytes = kv.block_tokens * kv.head_dim * isz;
    const long long plane_bytes = kv.n_blocks * (long long)block_bytes;
    dim3 grid((unsigned)(2 * n_layers * kv.n_kv_heads), (unsigned)n_seq_blocks);
    if (to_image)
        kv_image_kernel<true><<<grid, 128, 0, s>>>((char*)kv.base, plane_bytes, block_bytes, ids, (char*)image,
                                                   kv.n_kv_heads, kv.head_dim, isz, last_fill);
    else
        kv_image_kernel<false><<<grid, 128, 0, s>>>((char*)kv.base, plane_bytes, block_bytes, ids, (char*)image,
                                                    kv.n_kv_heads, kv.head_dim, isz, last_fill);
}

__global__ void plain_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

void launch_plain_copy(void* dst, const void* src, size_t n16, hipStream_t s) {
    plain_copy_kernel<<<4096, 256, 0, s>>>((const uint4*)src, (uint4*)dst, n16);
}

void launch_block_copy(DType dt, KVGeom kv, int n_layers, int src, int dst, hipStream_t s) {
    const long long isz = dt == F32 ? 4 : 2;
    const long long block_bytes = (long long)kv.block_tokens * kv.head_dim * isz;
    const long long plane_bytes = kv.n_blocks * block_bytes;
    block_copy_kernel<<<2 * n_layers * kv.n_kv_heads, 64, 0, s>>>((char*)kv.base, plane_bytes,
                                                                  block_bytes, src, dst);
}

}  // namespace ax
