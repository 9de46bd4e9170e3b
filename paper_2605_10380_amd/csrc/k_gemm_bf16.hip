// GEMMs of bf16-weight models on the gfx950 matrix cores: C = A[M,K] * W[N,K]^T, fp32
// accumulation.  The caller's weights are bf16; the kernels read the library's own 16-bit copy,
// made once at model creation: each bf16 widened to fp16 (exact for every |w| >= 2^-14, absolute
// error below 2^-25 beneath that) and laid out in MFMA operand order (see "weight layout" below).
// Activations are fp16 and the product runs on the fp16 MFMA, which has the same rate as the
// bf16 one.  Reason: bf16 activations (8 significant bits) put the logits of a 16-layer decoder
// ~0.05 away from the exact result; fp16 activations (11 bits) keep them within 0.01.
//
//   * skinny kernel (M <= 16, the O projection and narrow stores to 32: verify steps, pure weight streaming): one block owns 16 output
//     columns, its wavefronts split K, W goes HBM -> registers -> v_mfma_f32_16x16x32_f16
//     with no LDS in the streaming loop; the per-wavefront partial sums meet in LDS.
//   * tile kernel   (more rows): 8 wavefronts, LDS-staged 64 x 128 x 64 tiles,
//     v_mfma_f32_32x32x16_f16, global loads several K slices ahead.
//   * stream kernel (SwiGLU from 193-257 rows, logits from 17 rows, QKV / down projection of many rows, and - over K
//     slices - the SwiGLU GEMM of 17-192 rows and the down projection of 129 rows up): activations through LDS,
//     weights straight into MFMA operands.  The launcher states each crossover with the figures behind it.
//
// RMSNorm is folded into the GEMMs around it.  The GEMM that produces the residual stream x
// also writes a = fp16(x * gain_next) and, per row and per block of columns, a partial sum of
// x^2.  The GEMM that consumes a multiplies its accumulators by 1 / sqrt(mean(x^2) + eps) in
// the epilogue: (x * g / rms) W^T = (1 / rms) * ((x * g) W^T).  No separate norm kernel runs.
//
// Epilogues: fp32 store (optionally rms-scaled), residual add (+ norm preparation), SwiGLU
// (two weight matrices share the A operand), and QKV (rms scale, rotary embedding, q to the
// activation buffer, k and v straight into the KV pages).
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "kernels.h"

namespace ax {

typedef __bf16 bf16;
typedef _Float16 f16;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

void launch_gemm_f32(Epilogue epi, const float* A, const float* W, const float* W2, float* C,
                     int M, int N, int K, hipStream_t s);

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

// 8 bf16 (one 16-byte fragment) -> 8 fp16.  A bf16 is the top half of an fp32, so each half of
// a dword becomes an fp32 by a shift or a mask; bf16 has fewer significant bits than fp16, so
// the round-toward-zero pack is exact in fp16's normal range.
__device__ __forceinline__ f16x8 bf16x8_to_f16x8(u32x4 raw) {
    f16x8 out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = __uint_as_float(raw[i] << 16), hi = __uint_as_float(raw[i] & 0xffff0000u);
        const f16x2 h = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(lo, hi));
        out[2 * i] = h[0];
        out[2 * i + 1] = h[1];
    }
    return out;
}
__device__ __forceinline__ f16x8 load_w(const bf16* p) { return *(const f16x8*)p; }     // packed weights are already fp16

// Split activations (see GemmArgs): v goes out as hi = fp16(v) and, lo_off elements further on, lo = fp16(v - hi).
__device__ __forceinline__ void store_split(f16* p, long long lo_off, float v) {
    const f16 hi = (f16)v;
    *p = hi;
    if (lo_off) p[lo_off] = (f16)(v - (float)hi);
}
__device__ __forceinline__ void store_split4(f16* p, long long lo_off, const float (&v)[4]) {
    f16x4 hi, lo;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        hi[r] = (f16)v[r];
        lo[r] = (f16)(v[r] - (float)hi[r]);
    }
    *(f16x4*)p = hi;
    if (lo_off) *(f16x4*)(p + lo_off) = lo;
}

// ------------------------------------------------------------------------------ weight layout
// bf16 weight matrices are not read as given.  ax_model_create repacks every [N, K] matrix once,
// widening each bf16 to fp16 on the way (the round-toward-zero pack above: exact in fp16's normal
// range; the kernels multiply on the fp16 MFMA), into panels of 16 rows; a panel is cut into chunks of 32 k, and a chunk (1 KB) is stored in
// the order the 16x16x32 MFMA takes it: 4 k-groups of 8, inside a group the 16 rows, each with
// its 8 consecutive k (16 bytes).  A wavefront's weight load for one MFMA step is then 1 KB of
// contiguous memory instead of 16 pieces of 64 bytes from 16 rows - measured 7-19 % faster
// streaming in the skinny kernels and ~1.4x in the tile kernels that feed MFMA operands straight
// from global memory.  Element (n, k) sits at
//     (n / 16) * 16 K  +  (k / 32) * 512  +  ((k % 32) / 8) * 128  +  (n % 16) * 8  +  k % 8.
// N % 16 == 0 and K % 32 == 0 (guaranteed by the model configuration checks).
__device__ __forceinline__ long long packed_row(int n, int K) { return (long long)(n >> 4) * 16 * K + (n & 15) * 8; }
constexpr int PK_KG = 128;        // elements between k-groups of 8 inside a chunk
constexpr int PK_CHUNK = 512;     // elements per chunk of 32 k  (so k advances by 32 -> +512: "k * 16")

// out-of-place repack: one thread per 16-byte unit of the destination (coalesced writes)
// A bf16 weight beyond fp16's range (|w| > 65504, infinities, NaNs) does not survive: `bad` reports it.
__global__ void pack_weights_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int N, int K, int* __restrict__ bad) {
    const long long units = (long long)N * K / 8, stride = (long long)gridDim.x * blockDim.x;
    const int upp = 2 * K;                                   // 16-byte units per panel
    bool lost = false;
    for (long long u = (long long)blockIdx.x * blockDim.x + threadIdx.x; u < units; u += stride) {
        const int panel = (int)(u / upp), w = (int)(u % upp);
        const int c = w >> 6, kg = (w >> 4) & 3, r = w & 15;
        const u32x4 raw = src[((long long)(panel * 16 + r) * K + c * 32 + kg * 8) / 8];
#pragma unroll
        for (int i = 0; i < 4; ++i)       // checked on the exact values: the narrowing itself rounds toward zero and would saturate
            lost |= !(__builtin_fabsf(__uint_as_float(raw[i] << 16)) <= 65504.0f) ||
                    !(__builtin_fabsf(__uint_as_float(raw[i] & 0xffff0000u)) <= 65504.0f);
        dst[u] = __builtin_bit_cast(u32x4, bf16x8_to_f16x8(raw));
    }
    if (bad && lost) *bad = 1;                               // every writer stores the same value
}

void launch_pack_weights(const void* src, void* dst, int N, int K, hipStream_t s, int* bad) {
    pack_weights_kernel<<<2048, 256, 0, s>>>((const u32x4*)src, (u32x4*)dst, N, K, bad);
}

// 1 / rms of A rows from the column-block partial sums of x^2 their producer left behind.
// A kernel of this size is a chain of memory round trips, so every helper here requests all
// the partials it will need before it adds anything up: the index is clamped instead of
// branched on (no load sits behind a branch), values past the end are dropped when summing.
//
// One row's partials spread over a group of G lanes (gl = lane within the group), 4 G per round.
template <int G>
__device__ __forceinline__ float ssq_lane_sum(const float* __restrict__ src, int nparts, int gl) {
    float v = 0.f;
    for (int base = 0; base < nparts; base += 4 * G) {
        float t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = src[min(base + u * G + gl, nparts - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u) v += base + u * G + gl < nparts ? t[u] : 0.f;
    }
    return v;
}
// One row by one wavefront; every lane gets the result.
__device__ __forceinline__ float wave_inv_rms(const float* __restrict__ ssq, int row, int nparts,
                                              int d_norm, float eps, int lane) {
    float v = ssq_lane_sum<64>(ssq + (long long)row * nparts, nparts, lane);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return 1.0f / sqrtf(v / (float)d_norm + eps);
}

// Block-wide: 1 / rms of `rows` A-rows into s_inv[0..rows).  Half a wavefront (32 lanes) owns a
// row and a thread works on INV_BATCH rows at a time (a power of two up to 16): their
// 4 x INV_BATCH loads are in flight together, so the table costs one memory round trip per
// INV_BATCH rows of a thread (and per 128 partials of a row), not one per load.
// The INV_BATCH per-lane sums are then added across the 32 lanes with a transposing butterfly:
// at each stage a lane hands half of its values to its partner and keeps the other half, so the
// batch costs INV_BATCH - 1 + (5 - log2 INV_BATCH) cross-lane exchanges instead of 5 per row and
// ends with each row's total in its own lanes - one division and square root per thread, not one
// per row.  (Five exchanges and a square root per row, one row after the other, were ~4 us of a
// 128-row block's prologue.)  The caller synchronises before reading s_inv.
template <int INV_BATCH>
__device__ __forceinline__ void block_inv_rms(const GemmArgs& g, int first_row, int rows, float* s_inv) {
    static_assert(INV_BATCH == 1 || INV_BATCH == 2 || INV_BATCH == 4 || INV_BATCH == 8 || INV_BATCH == 16, "power of two up to 16");
    constexpr int LOG = INV_BATCH == 16 ? 4 : INV_BATCH == 8 ? 3 : INV_BATCH == 4 ? 2 : INV_BATCH == 2 ? 1 : 0;
    const int hw = threadIdx.x >> 5, hl = threadIdx.x & 31, nhw = blockDim.x >> 5;
    for (int base = 0; base < rows; base += INV_BATCH * nhw) {
        long long src[INV_BATCH];
        float v[INV_BATCH];
#pragma unroll
        for (int p = 0; p < INV_BATCH; ++p) {
            const int gm = min(first_row + min(base + p * nhw + hw, rows - 1), g.M - 1);
            src[p] = (long long)(g.a_rows ? g.a_rows[gm] : gm) * g.nparts;
            v[p] = 0.f;
        }
        for (int q0 = 0; q0 < g.nparts; q0 += 128) {
            float t[INV_BATCH][4];
#pragma unroll
            for (int p = 0; p < INV_BATCH; ++p)
#pragma unroll
                for (int u = 0; u < 4; ++u) t[p][u] = g.ssq[src[p] + min(q0 + u * 32 + hl, g.nparts - 1)];
#pragma unroll
            for (int p = 0; p < INV_BATCH; ++p)
#pragma unroll
                for (int u = 0; u < 4; ++u) v[p] += q0 + u * 32 + hl < g.nparts ? t[p][u] : 0.f;
        }
        // stage st: partner = lane ^ (16 >> st); the lane with that bit set keeps the upper half of
        // the remaining values, so after LOG stages it holds the row whose index (within the batch)
        // is the top LOG bits of its lane number
#pragma unroll
        for (int st = 0; st < LOG; ++st) {
            const int n = INV_BATCH >> st, o = 16 >> st;
            const bool upper = (hl & o) != 0;
#pragma unroll
            for (int j = 0; j < n / 2; ++j) {
                const float send = upper ? v[j] : v[j + n / 2];
                const float keep = upper ? v[j + n / 2] : v[j];
                v[j] = keep + __shfl_xor(send, o, 64);
            }
        }
#pragma unroll
        for (int o = 16 >> LOG; o > 0; o >>= 1) v[0] += __shfl_xor(v[0], o, 64);
        const int r = base + (hl >> (5 - LOG)) * nhw + hw;
        if ((hl & ((32 >> LOG) - 1)) == 0 && r < rows) s_inv[r] = 1.0f / sqrtf(v[0] / (float)g.d_norm + g.eps);
    }
}

// The same for rows that left at most 4 partial sums behind (their producer was a K-split GEMM's
// reduce kernel, or the embedding): four lanes per row, one load each, the rows of up to four
// passes in flight together - cheap enough in registers to sit behind the operand loads of a
// kernel's prologue, where its cold misses overlap theirs.
__device__ __forceinline__ void block_inv_rms_few(const GemmArgs& g, int first_row, int rows, float* s_inv) {
    const int p = threadIdx.x & 3, per_pass = blockDim.x >> 2;
    for (int base = 0; base < rows; base += 4 * per_pass) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int gm = min(first_row + min(base + u * per_pass + (int)(threadIdx.x >> 2), rows - 1), g.M - 1);
            v[u] = g.ssq[(long long)(g.a_rows ? g.a_rows[gm] : gm) * g.nparts + min(p, g.nparts - 1)];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float t = p < g.nparts ? v[u] : 0.f;
            t += __shfl_xor(t, 1, 64);
            t += __shfl_xor(t, 2, 64);
            const int r = base + u * per_pass + (int)(threadIdx.x >> 2);
            if (p == 0 && r < rows) s_inv[r] = 1.0f / sqrtf(t / (float)g.d_norm + g.eps);
        }
    }
}

// ------------------------------------------------------------------------------ tile kernel
// MFMA 32x32x16 operand layout (wave64): lane l supplies row/col (l % 32) and the 8 k values
// 8*(l/32) .. +7; result register r of lane l is C[(r/4)*8 + (l/32)*4 + r%4][l % 32].
// Block = WM x WN wavefronts, wavefront tile = (TM*32) x (TN*32).  (The QKV projection runs
// as a plain store GEMM followed by qkv_reduce_rope_kernel.)
// SPLIT: the A operand comes as hi and lo parts (split activations): both are staged and multiplied against the
// same B fragments.
template <int EPI, int TM, int TN, int WM = 2, int WN = 2, bool SPLIT = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_tile_kernel(GemmArgs g) {
    constexpr int NT = 64 * WM * WN;                                         // threads per block
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64, LS = BK + 8;  // LS: padded row
    constexpr int NB = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;                  // 16-byte chunks per thread
    constexpr int D = (NB == 2 && B_CH > 2) ? 2 : 4;                         // prefetch distance (even)
    constexpr int NA = SPLIT ? 2 : 1;
    __shared__ __attribute__((aligned(16))) f16 sA[2][NA][BM * LS];
    __shared__ __attribute__((aligned(16))) f16 sB[2][NB][BN * LS];
    __shared__ float s_inv[BM];

    const f16* __restrict__ A = (const f16*)g.A;
    const bf16* __restrict__ W = (const bf16*)g.W;
    const bf16* __restrict__ W2 = (const bf16*)g.W2;
    const int M = g.M, N = g.N, K = g.K;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lg = lane >> 5;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kspan = g.ksplit > 1 ? K / g.ksplit : K, kbase = blockIdx.z * kspan;   // this block's K slice

    f32x16 acc[NB][TM][TN];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[b][i][j][r] = 0.f;

    // Software pipeline: global loads run D k-steps ahead in a register ring (slot = step % D),
    // LDS is double buffered, one barrier per k-step.  At step s: issue the loads of s + D,
    // multiply out of LDS buffer s % 2, move the registers of s + 1 into the other buffer.
    f16x8 ra[D][NA][A_CH];
    u32x4 rb[D][NB][B_CH];          // weights as packed (fp16, MFMA operand order)
    long long a_off[A_CH], b_off[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int c = tid + NT * i, row = c >> 3, cc = c & 7;
        const int gm = min(m0 + row, M - 1);
        a_off[i] = (long long)(g.a_rows ? g.a_rows[gm] : gm) * K + kbase + cc * 8;
    }
    // weights (packed layout): a 64-wide k-step of one 16-row panel is 2 KB of contiguous memory,
    // 128 units of 16 bytes: unit = chunk (k / 32) * 64 + k-group * 16 + row
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        const int c = tid + NT * i, panel = min((n0 >> 4) + (c >> 7), (N >> 4) - 1);
        b_off[i] = (long long)panel * 16 * K + (long long)kbase * 16 + (c & 127) * 8;
    }
    auto load_global = [&](int slot, int k0) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            ra[slot][0][i] = *(const f16x8*)(A + a_off[i] + k0);
            if (SPLIT) ra[slot][NA - 1][i] = *(const f16x8*)(A + a_off[i] + k0 + g.a_lo_off);
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            rb[slot][0][i] = __builtin_nontemporal_load((const u32x4*)(W + b_off[i] + (long long)k0 * 16));
            if (NB == 2) rb[slot][NB - 1][i] = __builtin_nontemporal_load((const u32x4*)(W2 + b_off[i] + (long long)k0 * 16));
        }
    };
    auto store_lds = [&](int slot, int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int c = tid + NT * i, row = c >> 3, cc = c & 7;
#pragma unroll
            for (int p = 0; p < NA; ++p) *(f16x8*)(sA[buf][p] + row * LS + cc * 8) = ra[slot][p][i];
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            const int c = tid + NT * i, u = c & 127;
            const int row = (c >> 7) * 16 + (u & 15), col = (u >> 6) * 32 + ((u >> 4) & 3) * 8;
#pragma unroll
            for (int b = 0; b < NB; ++b) *(f16x8*)(sB[buf][b] + row * LS + col) = __builtin_bit_cast(f16x8, rb[slot][b][i]);
        }
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            f16x8 fa[NA][TM], fb[NB][TN];
#pragma unroll
            for (int p = 0; p < NA; ++p)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[p][i] = *(const f16x8*)(sA[buf][p] + ((wm * TM + i) * 32 + lrow) * LS + kk * 16 + lg * 8);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[b][j] = *(const f16x8*)(sB[buf][b] + ((wn * TN + j) * 32 + lrow) * LS + kk * 16 + lg * 8);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int p = 0; p < NA; ++p)
                            acc[b][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[p][i], fb[b][j], acc[b][i][j], 0, 0, 0);
        }
    };

    const int nsteps = kspan / BK;
#pragma unroll
    for (int s = 0; s < D; ++s)
        if (s < nsteps) load_global(s, s * BK);
    // deferred RMSNorm: 1/rms of this block's rows, 64 rows per batch (more loads in flight would cost the 64-row
    // blocks the registers for their second block per CU)
    if (g.ssq) {
        if (g.nparts <= 4) block_inv_rms_few(g, m0, BM, s_inv);
        else block_inv_rms<BM >= 128 ? 4 : 2>(g, m0, BM, s_inv);
    }
    store_lds(0, 0);
    __syncthreads();
    // steady state: groups of D steps with every load and store unconditional (branch-free, so
    // the loads of the next D steps stay in flight across the barriers)
    int step0 = 0;
    for (; step0 + 2 * D <= nsteps; step0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {                    // D is even: buffer = u % 2, slot = u
            load_global(u, (step0 + u + D) * BK);
            multiply(u & 1);
            store_lds((u + 1) % D, (u + 1) & 1);
            __syncthreads();
        }
    }
    // drain: at most 2 D - 1 steps, loads only while there is something left to load
    for (; step0 < nsteps; step0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int step = step0 + u;
            if (step < nsteps) {
                if (step + D < nsteps) load_global(u, (step + D) * BK);
                multiply(u & 1);
                if (step + 1 < nsteps) store_lds((u + 1) % D, (u + 1) & 1);
                __syncthreads();
            }
        }
    }

    // Epilogues.  Each one first requests everything it needs from memory for all of the
    // thread's 16 * TM * TN outputs and only then computes and stores: stores and loads through
    // the same pointers would otherwise be kept in program order, one round trip per element.
    auto row_of = [&](int i, int r) { return (wm * TM + i) * 32 + (r >> 2) * 8 + lg * 4 + (r & 3); };
    auto col_of = [&](int j) { return n0 + (wn * TN + j) * 32 + lrow; };
    float inv[TM][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) inv[i][r] = g.ssq ? s_inv[row_of(i, r)] : 1.0f;

    if constexpr (EPI == EPI_STORE_F32) {
        float* __restrict__ C = g.Cf + (g.ksplit > 1 ? (long long)blockIdx.z * M * N : 0);   // K slice: its own slab
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int m = m0 + row_of(i, r), n = col_of(j);
                    if (m < M && n < N) C[(long long)m * N + n] = acc[0][i][j][r] * inv[i][r];
                }
    } else if constexpr (EPI == EPI_SWIGLU) {
        f16* __restrict__ out = (f16*)g.C16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int m = m0 + row_of(i, r), n = col_of(j);
                    if (m < M && n < N)
                        store_split(out + (long long)m * N + n, g.c_lo_off,
                                    silu_f(acc[0][i][j][r] * inv[i][r]) * (acc[NB - 1][i][j][r] * inv[i][r]));
                }
    } else if constexpr (EPI == EPI_RESIDUAL) {
        if (g.ksplit > 1) {          // K slice: raw partial products, finished by residual_reduce_kernel
            float* part = g.split_ws + (long long)blockIdx.z * M * N;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int m = m0 + row_of(i, r), n = col_of(j);
                        if (m < M && n < N) part[(long long)m * N + n] = acc[0][i][j][r];
                    }
            return;
        }
        float gain[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) gain[j] = g.gain_next ? (float)((const bf16*)g.gain_next)[min(col_of(j), N - 1)] : 0.f;
        float xv[TM][TN][16];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = min(m0 + row_of(i, r), M - 1), n = min(col_of(j), N - 1);
                    xv[i][j][r] = g.Cf[(long long)m * N + n];
                }
        f16* __restrict__ a16 = (f16*)g.C16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + row_of(i, r);
                float ss = 0.f;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = col_of(j);
                    if (m < M && n < N) {
                        const long long o = (long long)m * N + n;
                        const float xn = xv[i][j][r] + acc[0][i][j][r];
                        g.Cf[o] = xn;
                        if (g.gain_next) {
                            store_split(a16 + o, g.c_lo_off, xn * gain[j]);
                            ss += xn * xn;
                        }
                    }
                }
                if (g.gain_next) {   // partial sum of squares over this wavefront's TN*32 columns
#pragma unroll
                    for (int o = 16; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
                    const int part = n0 / (TN * 32) + wn;                 // this wavefront's block of columns
                    if (lrow == 0 && m < M && part < N / (TN * 32)) g.ssq_out[(long long)m * (N / (TN * 32)) + part] = ss;
                }
            }
    }
}

// Second half of a K-split residual GEMM: x += sum of the K-slice partials (in slice order),
// a = fp16(x * gain_next), and the sum of x^2 over the block's columns.  Block = 1024 columns of
// one row (four per thread, every operand requested before anything is added), so a row leaves
// only ceil(N / 1024) partial sums behind - the GEMM that consumes the pending norm reads 2-4
// values per row instead of N / 32.  grid (ceil(N / 1024), M); N % 4 == 0.
constexpr int REDUCE_COLS = 1024;
__global__ __launch_bounds__(256) void residual_reduce_kernel(GemmArgs g) {
    __shared__ float s_ss[4];
    const int m = blockIdx.y, n = (blockIdx.x * 256 + threadIdx.x) * 4;
    const bool live = n < g.N;
    const int nc = min(n, g.N - 4);
    const long long o = (long long)m * g.N + nc, slab = (long long)g.M * g.N;
    f32x4 part[SPLITK_MAX];
#pragma unroll
    for (int ks = 0; ks < SPLITK_MAX; ++ks)
        part[ks] = ks < g.ksplit ? *(const f32x4*)(g.split_ws + ks * slab + o) : (f32x4){0.f, 0.f, 0.f, 0.f};
    f32x4 xn = *(const f32x4*)(g.Cf + o);
    float gain[4] = {0.f, 0.f, 0.f, 0.f};
    if (g.gain_next) {
#pragma unroll
        for (int r = 0; r < 4; ++r) gain[r] = (float)((const bf16*)g.gain_next)[nc + r];
    }
#pragma unroll
    for (int ks = 0; ks < SPLITK_MAX; ++ks) xn += part[ks];
    if (live) *(f32x4*)(g.Cf + o) = xn;
    if (g.gain_next) {
        float ss = 0.f;
        if (live) {
            float h[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                h[r] = xn[r] * gain[r];
                ss += xn[r] * xn[r];
            }
            store_split4((f16*)g.C16 + o, g.c_lo_off, h);
        }
#pragma unroll
        for (int w = 32; w > 0; w >>= 1) ss += __shfl_xor(ss, w, 64);
        if ((threadIdx.x & 63) == 0) s_ss[threadIdx.x >> 6] = ss;
        __syncthreads();
        if (threadIdx.x == 0) g.ssq_out[(long long)m * gridDim.x + blockIdx.x] = (s_ss[0] + s_ss[1]) + (s_ss[2] + s_ss[3]);
    }
}
// launches it; returns the partial sums per row it leaves
static int launch_residual_reduce(const GemmArgs& g, hipStream_t s) {
    const int parts = (g.N + REDUCE_COLS - 1) / REDUCE_COLS;
    residual_reduce_kernel<<<dim3((unsigned)parts, (unsigned)g.M), 256, 0, s>>>(g);
    return parts;
}

// Second half of a K-split QKV GEMM: sums the K-slice partials, applies 1 / rms of the row,
// rotates q and k heads by the row's position and writes q to the activation buffer, k and v
// into the row's KV slot.  grid (rows, ceil(items / 256)): a thread owns one (head, channel pair)
// item of its row, so all its operands are requested in one go while wavefront 0 works out the
// row's 1 / rms.
__global__ __launch_bounds__(256) void qkv_reduce_rope_kernel(GemmArgs g) {
    __shared__ float s_inv;
    const int m = blockIdx.x, N = g.N;
    const RopeArgs& ro = g.rope;
    const int Hq = ro.n_q_heads, Hkv = ro.kv.n_kv_heads, hd = ro.kv.head_dim, half = hd >> 1;
    const int n_items = (Hq + 2 * Hkv) * half;
    const int it = min((int)(blockIdx.y * 256 + threadIdx.x), n_items - 1);
    const bool live = blockIdx.y * 256 + threadIdx.x < n_items;
    const int head = it / half, j = it - head * half;
    const int pos = ro.row_pos[m], slot = ro.row_slot[m];
    const long long slab = (long long)g.M * N;
    const float* p = g.split_ws + (long long)m * N + head * hd + j;
    float pa[SPLITK_MAX], pb[SPLITK_MAX];
#pragma unroll
    for (int ks = 0; ks < SPLITK_MAX; ++ks) {
        pa[ks] = ks < g.ksplit ? p[ks * slab] : 0.f;
        pb[ks] = ks < g.ksplit ? p[ks * slab + half] : 0.f;
    }
    const float c = ro.cos[(long long)pos * half + j], sg = ro.sin[(long long)pos * half + j];
    if (threadIdx.x < 64) {
        const float inv = g.ssq ? wave_inv_rms(g.ssq, m, g.nparts, g.d_norm, g.eps, threadIdx.x) : 1.0f;
        if (threadIdx.x == 0) s_inv = inv;
    }
    __syncthreads();
    if (!live) return;
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int ks = 0; ks < SPLITK_MAX; ++ks) { a += pa[ks]; b += pb[ks]; }
    a *= s_inv;
    b *= s_inv;
    f16* pool = (f16*)ro.kv.base;
    if (head < Hq + Hkv) {
        f16* dst = head < Hq ? (f16*)ro.q_out + ((long long)m * Hq + head) * hd
                             : pool + ro.kv.plane(ro.layer, 0, head - Hq) + (long long)slot * hd;
        const long long lo_off = head < Hq ? g.c_lo_off : 0;      // q may be split; the cache holds one fp16 per entry
        store_split(dst + j, lo_off, a * c - b * sg);
        store_split(dst + j + half, lo_off, b * c + a * sg);
    } else {
        f16* dst = pool + ro.kv.plane(ro.layer, 1, head - Hq - Hkv) + (long long)(slot >> 4) * 16 * hd + (slot & 15);
        dst[(long long)j * 16] = (f16)a;
        dst[(long long)(j + half) * 16] = (f16)b;
    }
}

// Second half of a K-sliced SwiGLU GEMM: out[m, n] = fp16(silu(gate * inv) * (up * inv)) with gate
// and up the sums of the slices' raw products (slabs [ksplit][M][2 N]: gate | up) and inv the row's
// 1 / rms.  grid (rows, ceil(N / 256)).
__global__ __launch_bounds__(256) void swiglu_reduce_kernel(GemmArgs g) {
    __shared__ float s_inv;
    const int m = blockIdx.x, N = g.N, n = blockIdx.y * 256 + threadIdx.x;
    const long long slab = (long long)g.M * 2 * N;
    const float* p = g.split_ws + (long long)m * 2 * N + min(n, N - 1);
    float pa[SPLITK_MAX], pb[SPLITK_MAX];
#pragma unroll
    for (int ks = 0; ks < SPLITK_MAX; ++ks) {
        pa[ks] = ks < g.ksplit ? p[ks * slab] : 0.f;
        pb[ks] = ks < g.ksplit ? p[ks * slab + N] : 0.f;
    }
    if (threadIdx.x < 64) {
        const float inv = g.ssq ? wave_inv_rms(g.ssq, g.a_rows ? g.a_rows[m] : m, g.nparts, g.d_norm, g.eps, threadIdx.x) : 1.0f;
        if (threadIdx.x == 0) s_inv = inv;
    }
    __syncthreads();
    if (n >= N) return;
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int ks = 0; ks < SPLITK_MAX; ++ks) { a += pa[ks]; b += pb[ks]; }
    store_split((f16*)g.C16 + (long long)m * N + n, g.c_lo_off, silu_f(a * s_inv) * (b * s_inv));
}

// ------------------------------------------------------------------------------ stream SwiGLU kernel
// First written for the SwiGLU gate/up GEMM of a few hundred rows.  The LDS-staged kernel above moves both operands through
// LDS and spends more cycles there than on the matrix cores (a 32 x 64 wavefront tile reads
// 1.5 KB of LDS per MFMA).  Here only the activation tile goes through LDS; every wavefront
// streams its own weight rows HBM/L2 -> registers -> MFMA, as the skinny kernel does.  Block = 4
// wavefronts side by side along N, all working on the same BM = TM*32 rows; a wavefront owns 32
// output columns, i.e. one 32-row tile each of W (gate) and W2 (up).  The weight loads run D
// k-steps ahead in a register ring, the activation tile is double buffered in LDS, one barrier
// per k-step of 64.  Measured against the LDS-staged kernel at M = 512 / 1024: 79 / 147 us
// instead of 110 / 184 us (N = 8192, K = 3072), 174 / 332 instead of 246 / 410 us (N = 14336,
// K = 4096); at M = 256 it has too few blocks per CU and loses, so it is not used there.
//
// Blocks are renumbered so that the gy row tiles that share a weight tile have consecutive ids
// on one XCD (workgroups are dealt to the 8 XCDs round robin), i.e. share that XCD's L2.
//
// The same kernel serves the other GEMMs of calls with thousands of rows (EPI_STORE_F32: the QKV
// products, EPI_RESIDUAL): there a wavefront's two weight streams are two 32-row tiles of the ONE
// matrix, 32 columns apart, and a block covers 256 output columns.
//
// NS = 1: one weight stream per wavefront (block = 128 columns), and K may be cut into g.ksplit
// slices over extra blocks whose raw fp32 partial products go to slabs that qkv_reduce_rope_kernel /
// residual_reduce_kernel add up: calls of 129-192 rows (16 sessions verified together), where one
// 160- or 192-row block reads each weight once and the slices give the chip its ~200 blocks.
//
// SPLIT: split activations - the hi and lo parts of the A tile are both staged in LDS and multiplied against the
// same weight registers.
template <int EPI, int TM, int D, int NS = 2, bool SLICED = false, bool SPLIT = false>
__global__ __launch_bounds__(256) void gemm_bf16_stream_kernel(GemmArgs g, int gx, int gy) {
    static_assert(EPI != EPI_SWIGLU || NS == 2, "SwiGLU streams gate and up");
    constexpr int BM = TM * 32, BN = EPI == EPI_SWIGLU ? 128 : NS * 128, BK = 64, LS = BK + 8;
    constexpr int A_CH = BM * 8 / 256;                       // 16-byte chunks of the A tile per thread
    constexpr int NA = SPLIT ? 2 : 1;
    __shared__ __attribute__((aligned(16))) f16 sA[2][NA][BM * LS];
    __shared__ float s_inv[BM];

    const f16* __restrict__ A = (const f16*)g.A;
    const int M = g.M, N = g.N, K = g.K;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int lrow = lane & 31, lg = lane >> 5;
    const int nblk = gx * gy;
    const int kz = blockIdx.x / nblk;                        // K slice (0 unless g.ksplit > 1)
    int bid = blockIdx.x - kz * nblk;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int bx = bid / gy, by = bid - bx * gy;
    const int m0 = by * BM, n0 = bx * BN;
    const int kspan = SLICED ? K / g.ksplit : K, kbase = kz * kspan;      // SLICED: g.ksplit > 1 slices, a slab each

    // this lane's output columns = weight rows of its two streams: row n of W and of W2 (SwiGLU),
    // or rows n and n + 32 of W
    int ncol[NS];
    const bf16* wp[NS];
    // packed layout: MFMA step c of a k-step covers k = 16 c + 8 lg .. + 7, i.e. chunk c / 2, k-group 2 (c % 2) + lg
#pragma unroll
    for (int t = 0; t < NS; ++t) {
        ncol[t] = n0 + wave * (BN / 4) + lrow + (EPI == EPI_SWIGLU ? 0 : 32 * t);
        wp[t] = (const bf16*)(EPI == EPI_SWIGLU && t == 1 ? g.W2 : g.W) + packed_row(min(ncol[t], N - 1), K) +
                (long long)kbase * 16 + lg * PK_KG;
    }
    long long a_off[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int c = tid + 256 * i, row = c >> 3, cc = c & 7;
        const int gm = min(m0 + row, M - 1);
        a_off[i] = (long long)(g.a_rows ? g.a_rows[gm] : gm) * K + kbase + cc * 8;
    }

    f32x16 acc[NS][TM];
#pragma unroll
    for (int t = 0; t < NS; ++t)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][i][r] = 0.f;

    u32x4 rw[D][NS][4];             // weights: 4 chunks of 8 k per stream and k-step
    f16x8 ra[D][NA][A_CH];
    auto load_global = [&](int slot, int k0) {
#pragma unroll
        for (int t = 0; t < NS; ++t)
#pragma unroll
            for (int c = 0; c < 4; ++c) rw[slot][t][c] = __builtin_nontemporal_load((const u32x4*)(wp[t] + (long long)k0 * 16 + (c >> 1) * PK_CHUNK + (c & 1) * 2 * PK_KG));
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            ra[slot][0][i] = *(const f16x8*)(A + a_off[i] + k0);
            if (SPLIT) ra[slot][NA - 1][i] = *(const f16x8*)(A + a_off[i] + k0 + g.a_lo_off);
        }
    };
    auto store_lds = [&](int slot, int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int c = tid + 256 * i, row = c >> 3, cc = c & 7;
#pragma unroll
            for (int p = 0; p < NA; ++p) *(f16x8*)(sA[buf][p] + row * LS + cc * 8) = ra[slot][p][i];
        }
    };
    auto multiply = [&](int slot, int buf) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f16x8 fa[NA][TM], fw[NS];
#pragma unroll
            for (int p = 0; p < NA; ++p)
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[p][i] = *(const f16x8*)(sA[buf][p] + (i * 32 + lrow) * LS + c * 16 + lg * 8);
#pragma unroll
            for (int t = 0; t < NS; ++t) fw[t] = __builtin_bit_cast(f16x8, rw[slot][t][c]);
#pragma unroll
            for (int t = 0; t < NS; ++t)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int p = 0; p < NA; ++p)
                        acc[t][i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[p][i], fw[t], acc[t][i], 0, 0, 0);
        }
    };

    const int nsteps = kspan / BK;
    // deferred RMSNorm: 1/rms of this block's rows, before the operand rings take the registers (16
    // rows x 4 loads per thread in flight: one or two round trips; behind the ring loads the same
    // table cost four to six, 10-15 % of the launch at 512-1024 rows).  Sliced SwiGLU: the reduce kernel scales.
    // Few partials per row (K-split producer): behind the ring loads, their cold misses overlap.
    const bool inv_here = g.ssq && !(EPI == EPI_SWIGLU && SLICED);
    if (inv_here && g.nparts > 4) block_inv_rms<16>(g, m0, BM, s_inv);
#pragma unroll
    for (int s = 0; s < D; ++s)
        if (s < nsteps) load_global(s, s * BK);
    if (inv_here && g.nparts <= 4) block_inv_rms_few(g, m0, BM, s_inv);
    store_lds(0, 0);
    __syncthreads();
    // steady state, branch free: multiply step s out of ring slot s % D and LDS buffer s % 2,
    // refill the slot with step s + D, move the activations of step s + 1 into the other buffer
    int step0 = 0;
    for (; step0 + 2 * D <= nsteps; step0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int buf = (step0 + u) & 1;
            multiply(u, buf);
            store_lds((u + 1) % D, buf ^ 1);
            load_global(u, (step0 + u + D) * BK);
            __syncthreads();
        }
    }
    for (; step0 < nsteps; step0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int step = step0 + u;
            if (step < nsteps) {
                const int buf = step & 1;
                multiply(u, buf);
                if (step + 1 < nsteps) store_lds((u + 1) % D, buf ^ 1);
                if (step + D < nsteps) load_global(u, (step + D) * BK);
                __syncthreads();
            }
        }
    }

    auto row_of = [&](int i, int r) { return i * 32 + (r >> 2) * 8 + lg * 4 + (r & 3); };
    if constexpr (EPI == EPI_SWIGLU && SLICED) {             // raw gate | up products of this K slice: slab [M][2 N]
        float* __restrict__ C = g.split_ws + (long long)kz * M * 2 * N;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + row_of(i, r);
                    if (m < M && ncol[0] < N) C[(long long)m * 2 * N + t * N + ncol[0]] = acc[t][i][r];
                }
    } else if constexpr (EPI == EPI_SWIGLU) {
        f16* __restrict__ out = (f16*)g.C16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row_of(i, r), m = m0 + row;
                const float inv = g.ssq ? s_inv[row] : 1.0f;
                if (m < M && ncol[0] < N)
                    store_split(out + (long long)m * N + ncol[0], g.c_lo_off, silu_f(acc[0][i][r] * inv) * (acc[1][i][r] * inv));
            }
    } else if constexpr (EPI == EPI_STORE_F32 || SLICED) {  // K slice: its own slab of raw products
        float* __restrict__ C = SLICED ? (EPI == EPI_STORE_F32 ? g.Cf : g.split_ws) + (long long)kz * M * N : g.Cf;
#pragma unroll
        for (int t = 0; t < NS; ++t)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = row_of(i, r), m = m0 + row;
                    const float inv = g.ssq ? s_inv[row] : 1.0f;
                    if (m < M && ncol[t] < N) C[(long long)m * N + ncol[t]] = acc[t][i][r] * inv;
                }
    } else {                                                  // EPI_RESIDUAL; N % 32 == 0 (checked by the launcher)
        static_assert(TM % 2 == 0, "the residual epilogue works on pairs of row tiles");
        f16* __restrict__ a16 = (f16*)g.C16;
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            const int n = min(ncol[t], N - 1);
            const float gain = g.gain_next ? (float)((const bf16*)g.gain_next)[n] : 0.f;
#pragma unroll
            for (int i0 = 0; i0 < TM; i0 += 2) {
            float xv[2][16];                                  // the loads of two row tiles first, then their stores
#pragma unroll
            for (int i = i0; i < i0 + 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) xv[i - i0][r] = g.Cf[(long long)min(m0 + row_of(i, r), M - 1) * N + n];
#pragma unroll
            for (int i = i0; i < i0 + 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + row_of(i, r);
                    const bool live = m < M && ncol[t] < N;
                    const float xn = xv[i - i0][r] + acc[t][i][r];
                    float ss = live ? xn * xn : 0.f;
                    if (live) {
                        const long long o = (long long)m * N + n;
                        g.Cf[o] = xn;
                        if (g.gain_next) store_split(a16 + o, g.c_lo_off, xn * gain);
                    }
                    if (g.gain_next) {                        // partial sum of squares over this tile's 32 columns
#pragma unroll
                        for (int o = 16; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
                        if (lrow == 0 && live) g.ssq_out[(long long)m * (N / 32) + (ncol[t] >> 5)] = ss;
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------ skinny kernel
// MFMA 16x16x32 operand layout: lane l supplies row/col (l % 16) and the 8 k values
// 8*(l/16) .. +7; result register r of lane l is D[4*(l/16) + r][l % 16].  Here D = W_tile * x^T:
// D rows are output columns n, D columns are activation rows m, so a lane ends up with four
// consecutive n of one row m (one 16-byte store).
//
// COLS < 16 (residual GEMMs): a block owns fewer columns so that every CU gets a block; the
// unused MFMA rows are zero and their lanes issue no loads.
//
// For EPI_QKV the 16 columns of a block are 8 + 8 rotary partners of one head: local columns
// 0..7 are channels j0..j0+7, local columns 8..15 are channels hd/2 + j0 .. +7, so the partner
// of a lane's value lives in lane ^ 32.
//
// SPLIT: split activations - each weight fragment meets the hi and the lo part of the activation rows (two MFMAs);
// weight traffic is unchanged, the activation slice a wavefront reads doubles.
template <int EPI, int MT, int NW, int COLS = 16, bool SPLIT = false>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, NW >= 8 ? 4 : 8)))
void gemm_bf16_skinny_kernel(GemmArgs g) {
    constexpr int NB = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr int NA = SPLIT ? 2 : 1;
    __shared__ __attribute__((aligned(16))) f32x4 red[NW][NB][MT][64];
    __shared__ float s_inv[MT * 16];

    const f16* __restrict__ X = (const f16*)g.A;
    const bf16* __restrict__ W = (const bf16*)g.W;
    const bf16* __restrict__ W2 = (const bf16*)g.W2;
    const int M = g.M, N = g.N, K = g.K;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int lr = lane & 15, lg = lane >> 4;
    const int n0 = blockIdx.x * COLS;
    const int kslice = K / NW, kbeg = wave * kslice, kend = kbeg + kslice;

    int wrow;                            // weight row this lane streams
    int q_head = 0, q_j0 = 0;            // EPI_QKV: head and first channel of the block
    if (EPI == EPI_QKV) {
        const int hd = g.rope.kv.head_dim, per = hd / 16;
        q_head = blockIdx.x / per;
        q_j0 = (blockIdx.x % per) * 8;
        wrow = q_head * hd + (lr < 8 ? q_j0 + lr : hd / 2 + q_j0 + lr - 8);
    } else {
        wrow = min(n0 + min(lr, COLS - 1), N - 1);
    }
    const bool wlane = lr < COLS;      // COLS < 16: the other MFMA rows are zero, their lanes request nothing
    const bf16* wp = W + packed_row(wrow, K) + lg * PK_KG;          // packed layout: k advances by 32 -> + 512 elements
    const bf16* wp2 = NB == 2 ? W2 + packed_row(wrow, K) + lg * PK_KG : nullptr;
    // 8-column blocks: a load instruction costs the memory pipeline the same with half of its lanes
    // idle (the 8 MFMA rows that are not there), and these launches are bound by exactly that - a CU
    // pulled 16 GB/s of weights against 26 GB/s from 16-column blocks.  So the upper half of each
    // 16-lane row fetches the block's 8 rows at the NEXT k-step (one chunk further), and for that
    // step the operand is shifted down 8 lanes; MFMA rows 8-15 then hold products nobody reads.
    constexpr bool DUAL = COLS == 8 && MT <= 2 && NB == 1;
    const bf16* wpd = W + packed_row(min(n0 + (lr & 7), N - 1), K) + lg * PK_KG + (lr >> 3) * PK_CHUNK;
    const f16* xp[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = min(t * 16 + lr, M - 1);
        xp[t] = X + (long long)(g.a_rows ? g.a_rows[m] : m) * K + lg * 8;
    }

    f32x4 acc[NB][MT];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[b][t] = (f32x4){0.f, 0.f, 0.f, 0.f};


    // Epilogue operands that do not depend on the product are requested now, by the wavefront
    // that will run the epilogue: at these sizes a kernel is a chain of memory latencies, and
    // anything loaded after the K loop would add a full round trip to it.
    f32x4 pre_x[MT], pre_cs[MT], pre_sn[MT];
    float pre_g[4] = {0.f, 0.f, 0.f, 0.f};
    int pre_pos[MT], pre_slot[MT];
    if (wave == 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int m = min(t * 16 + lr, M - 1);
            if (EPI == EPI_RESIDUAL) {
                pre_x[t] = *(const f32x4*)(g.Cf + (long long)m * N + min(n0 + lg * 4, N - 4));
            } else if (EPI == EPI_QKV) {
                const int hd = g.rope.kv.head_dim;
                pre_pos[t] = g.rope.row_pos[m];
                pre_slot[t] = g.rope.row_slot[m];
                const long long ao = (long long)pre_pos[t] * (hd / 2) + q_j0 + (lg & 1) * 4;
                pre_cs[t] = *(const f32x4*)(g.rope.cos + ao);
                pre_sn[t] = *(const f32x4*)(g.rope.sin + ao);
            }
        }
        if (EPI == EPI_RESIDUAL && g.gain_next) {
#pragma unroll
            for (int r = 0; r < 4; ++r) pre_g[r] = (float)((const bf16*)g.gain_next)[min(n0 + lg * 4 + r, N - 1)];
        }
    }

    // The same for the partial sums of x^2 behind the deferred RMSNorm: wavefront w turns those of
    // rows w, w + NW, .. into 1 / rms after the K loop, from registers filled here (up to 16 rows, 256
    // partials per row and 4 rows per wavefront; anything larger is fetched after the loop).
    constexpr int RPW = (MT * 16 + NW - 1) / NW;
    constexpr bool PRE_SSQ = MT == 1 && RPW <= 4;          // 17-32 rows: only small test shapes arrive here with a norm pending
    float pre_ss[PRE_SSQ ? RPW : 1][4];
    const bool pre_ssq = PRE_SSQ && g.ssq && g.nparts <= 256;
    if (pre_ssq) {
#pragma unroll
        for (int j = 0; j < (PRE_SSQ ? RPW : 1); ++j) {
            const int m = min(wave + j * NW, M - 1);
            const float* src = g.ssq + (long long)(g.a_rows ? g.a_rows[m] : m) * g.nparts;
#pragma unroll
            for (int u = 0; u < 4; ++u) pre_ss[j][u] = src[min(u * 64 + lane, g.nparts - 1)];
        }
    }

    // ... and turned into 1 / rms while the first trip's operands are on their way (the partial sums were
    // requested before them, so waiting for these does not wait for those): nothing of it is left after the K loop,
    // and its registers are free during the loop.
    auto finish_pre_ssq = [&]() {
#pragma unroll
        for (int j = 0; j < (PRE_SSQ ? RPW : 1); ++j) {
            float v = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) v += u * 64 + lane < g.nparts ? pre_ss[j][u] : 0.f;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            const int r = wave + j * NW;
            if (lane == 0 && r < MT * 16) s_inv[r] = 1.0f / sqrtf(v / (float)g.d_norm + g.eps);
        }
    };

    // One trip = U MFMA k-steps (32 each).  All weight and activation loads of trip i + 1 are issued
    // before trip i is multiplied (two register sets), so a wavefront always has a trip's worth
    // of loads (U KB of weights) in flight while its matrix pipe is busy.
    int k = kbeg;
    if constexpr (MT <= 2) {
        constexpr int U = 4, S = 32 * U;
        u32x4 rw[2][NB][DUAL ? U / 2 : U];
        f16x8 fx[2][NA][MT][U];
#pragma unroll
        for (int set = 0; set < 2; ++set)
#pragma unroll
            for (int p = 0; p < NA; ++p)
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int u = 0; u < U; ++u) fx[set][p][t][u] = (f16x8){0, 0, 0, 0, 0, 0, 0, 0};   // rows past M stay zero
        auto loads = [&](int set, int kk) {
            if constexpr (DUAL) {
#pragma unroll
                for (int v = 0; v < U / 2; ++v) rw[set][0][v] = __builtin_nontemporal_load((const u32x4*)(wpd + (long long)(kk + 64 * v) * 16));
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    rw[set][0][u] = (COLS == 16 || wlane) ? __builtin_nontemporal_load((const u32x4*)(wp + (long long)(kk + 32 * u) * 16)) : (u32x4){0u, 0u, 0u, 0u};
                    if (NB == 2) rw[set][NB - 1][u] = __builtin_nontemporal_load((const u32x4*)(wp2 + (long long)(kk + 32 * u) * 16));
                }
            }
            // activation rows past M: no load (a block re-reads its wavefronts' whole activation slice, and at
            // 9 rows of 16 that is most of what the CU's load pipeline carries)
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                if (t * 16 + lr < M) {
#pragma unroll
                    for (int u = 0; u < U; ++u) fx[set][0][t][u] = *(const f16x8*)(xp[t] + kk + 32 * u);
                    if (SPLIT) {
#pragma unroll
                        for (int u = 0; u < U; ++u) fx[set][NA - 1][t][u] = *(const f16x8*)(xp[t] + g.a_lo_off + kk + 32 * u);
                    }
                }
            }
        };
        auto compute = [&](int set) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    u32x4 raw = rw[set][b][DUAL ? u >> 1 : u];
                    if (DUAL && (u & 1)) {                 // odd k-step: lanes 8-15 of each row hold it; row_shl:8 brings it to lanes 0-7
#pragma unroll
                        for (int i = 0; i < 4; ++i) raw[i] = (unsigned)__builtin_amdgcn_update_dpp(0, (int)raw[i], 0x108, 0xf, 0xf, true);
                    }
                    const f16x8 fw = __builtin_bit_cast(f16x8, raw);
#pragma unroll
                    for (int t = 0; t < MT; ++t)
#pragma unroll
                        for (int p = 0; p < NA; ++p)
                            acc[b][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw, fx[set][p][t][u], acc[b][t], 0, 0, 0);
                }
        };
        const int ntr = kslice / S;
        if (ntr > 0) loads(0, kbeg);
        if (pre_ssq) finish_pre_ssq();
        int t = 0;
        for (; t + 2 < ntr; t += 2) {                                // both loads unconditional
            loads(1, kbeg + (t + 1) * S);
            compute(0);
            loads(0, kbeg + (t + 2) * S);
            compute(1);
        }
        if (t + 1 < ntr) {
            loads(1, kbeg + (t + 1) * S);
            compute(0);
            compute(1);
        } else if (t < ntr) {
            compute(0);
        }
        k = kbeg + ntr * S;
    } else {
        for (; k + 128 <= kend; k += 128) {
            static_assert(!SPLIT, "more than two row tiles: not instantiated with split activations");
            u32x4 rw[NB][4];
            f16x8 fx[MT][4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                rw[0][u] = (COLS == 16 || wlane) ? __builtin_nontemporal_load((const u32x4*)(wp + (long long)(k + 32 * u) * 16)) : (u32x4){0u, 0u, 0u, 0u};
                if (NB == 2) rw[NB - 1][u] = __builtin_nontemporal_load((const u32x4*)(wp2 + (long long)(k + 32 * u) * 16));
            }
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int u = 0; u < 4; ++u) fx[t][u] = *(const f16x8*)(xp[t] + k + 32 * u);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const f16x8 fw = __builtin_bit_cast(f16x8, rw[b][u]);
#pragma unroll
                    for (int t = 0; t < MT; ++t)
                        acc[b][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw, fx[t][u], acc[b][t], 0, 0, 0);
                }
        }
    }
    for (; k < kend; k += 32) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const f16x8 fw = load_w((b == 0 ? wp : wp2) + (long long)k * 16);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const f16x8 fx = *(const f16x8*)(xp[t] + k);
                acc[b][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw, fx, acc[b][t], 0, 0, 0);
                if (SPLIT) {
                    const f16x8 fl = *(const f16x8*)(xp[t] + g.a_lo_off + k);
                    acc[b][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw, fl, acc[b][t], 0, 0, 0);
                }
            }
        }
    }

#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int t = 0; t < MT; ++t) red[wave][b][t][lane] = acc[b][t];
    if (pre_ssq) {                       // deferred RMSNorm: the wavefronts share the rows
        if (MT > 2) finish_pre_ssq();    // (the MT <= 2 loop did it behind its first loads)
    } else if (g.ssq) {
        for (int r = wave; r < min(MT * 16, M); r += NW) {
            const float inv = wave_inv_rms(g.ssq, g.a_rows ? g.a_rows[r] : r, g.nparts, g.d_norm, g.eps, lane);
            if (lane == 0) s_inv[r] = inv;
        }
    }
    __syncthreads();
    if (wave != 0) return;

#pragma unroll
    for (int t = 0; t < MT; ++t) {
        f32x4 sum[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            sum[b] = red[0][b][t][lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) sum[b] += red[w][b][t][lane];
        }
        const int m = t * 16 + lr, n = n0 + lg * 4;
        const bool mok = m < M && lg * 4 < COLS;
        const float inv = g.ssq ? s_inv[t * 16 + lr] : 1.0f;
        const long long o = (long long)m * N + n;
        if (EPI == EPI_STORE_F32) {
            if (mok && n < N) *(f32x4*)(g.Cf + o) = sum[0] * inv;
        } else if (EPI == EPI_SWIGLU) {
            if (mok && n < N) {
                float h[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) h[r] = silu_f(sum[0][r] * inv) * (sum[NB - 1][r] * inv);
                store_split4((f16*)g.C16 + o, g.c_lo_off, h);
            }
        } else if (EPI == EPI_RESIDUAL) {
            float ss = 0.f;
            if (mok && n < N) {
                const f32x4 xn = pre_x[t] + sum[0];
                *(f32x4*)(g.Cf + o) = xn;
                if (g.gain_next) {
                    float h[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        h[r] = xn[r] * pre_g[r];
                        ss += xn[r] * xn[r];
                    }
                    store_split4((f16*)g.C16 + o, g.c_lo_off, h);
                }
            }
            if (g.gain_next) {           // sum of squares over the block's COLS columns, per row
                ss += __shfl_xor(ss, 16, 64);
                ss += __shfl_xor(ss, 32, 64);
                if (lg == 0 && mok) g.ssq_out[(long long)m * (N / COLS) + blockIdx.x] = ss;
            }
        } else {                         // EPI_QKV
            const RopeArgs& ro = g.rope;
            const int Hq = ro.n_q_heads, Hkv = ro.kv.n_kv_heads, hd = ro.kv.head_dim;
            const int mm = min(m, M - 1);
            f16* pool = (f16*)ro.kv.base;
            const int chan = (lg < 2 ? q_j0 + lg * 4 : hd / 2 + q_j0 + (lg - 2) * 4);   // first of 4 channels
            f32x4 own = sum[0] * inv, other;
#pragma unroll
            for (int r = 0; r < 4; ++r) other[r] = __shfl_xor(own[r], 32, 64);
            if (q_head < Hq + Hkv) {
                const f32x4 cs = pre_cs[t], sn = pre_sn[t];      // angles q_j0 + (lg & 1) * 4 + r at the row's position
                float h[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    h[r] = lg < 2 ? own[r] * cs[r] - other[r] * sn[r]                   // first half: a c - b s
                                  : own[r] * cs[r] + other[r] * sn[r];                  // second half: b c + a s
                f16* dst;
                long long lo_off = 0;                                                    // the cache holds one fp16 per entry
                if (q_head < Hq) {
                    dst = (f16*)ro.q_out + ((long long)mm * Hq + q_head) * hd;
                    lo_off = g.c_lo_off;
                } else {
                    dst = pool + ro.kv.plane(ro.layer, 0, q_head - Hq) + (long long)pre_slot[t] * hd;
                }
                if (mok) store_split4(dst + chan, lo_off, h);
            } else if (mok) {
                f16* dst = pool + ro.kv.plane(ro.layer, 1, q_head - Hq - Hkv) + (long long)(pre_slot[t] >> 4) * 16 * hd + (pre_slot[t] & 15);
#pragma unroll
                for (int r = 0; r < 4; ++r) dst[(long long)(chan + r) * 16] = (f16)own[r];
            }
        }
    }
}

// Launch KERNEL<TARGS..., SPLIT>: the split-activation instantiation when the GEMM's A operand comes in two parts.
#define AX_UNPAREN(...) __VA_ARGS__
#define AX_SPLIT_LAUNCH(split_, KERNEL, TARGS, GRID, BLOCK, ...)                                        \
    do {                                                                                                \
        if (split_) KERNEL<AX_UNPAREN TARGS, true><<<GRID, BLOCK, 0, s>>>(__VA_ARGS__);                  \
        else KERNEL<AX_UNPAREN TARGS, false><<<GRID, BLOCK, 0, s>>>(__VA_ARGS__);                        \
    } while (0)

// Columns per block of the skinny kernel.  A CU pulls only ~26 GB/s of weights however many
// wavefronts it runs (measured), so a launch streams at the chip's rate only if every CU has a
// block: residual GEMMs (N = d_model, too few blocks of 16 columns) use 12 or 8 columns per
// block when that shortens rounds-of-256-blocks x columns.
static int skinny_cols(int epi, int N) {
    if (epi != EPI_RESIDUAL) return 16;
    int best = 16, best_cost = ((N / 16 + 255) / 256) * 16;
    for (int c : {12, 8}) {
        if (N % c) continue;
        const int cost = ((N / c + 255) / 256) * c;
        if (cost < best_cost) { best = c; best_cost = cost; }
    }
    return best;
}

template <int EPI, int MT, int COLS>
static void launch_skinny_cols(const GemmArgs& g, int nw, hipStream_t s) {
    const int grid = (g.N + COLS - 1) / COLS;
    if (nw == 16) AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_skinny_kernel, (EPI, MT, 16, COLS), grid, 1024, g);
    else if (nw == 1) AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_skinny_kernel, (EPI, MT, 1, COLS), grid, 64, g);
    else if (nw == 2) AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_skinny_kernel, (EPI, MT, 2, COLS), grid, 128, g);
    else if (nw == 8) AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_skinny_kernel, (EPI, MT, 8, COLS), grid, 512, g);
    else AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_skinny_kernel, (EPI, MT, 4, COLS), grid, 256, g);
}

template <int EPI, int MT>
static void launch_skinny_nw(const GemmArgs& g, int nw, hipStream_t s) {
    if constexpr (EPI == EPI_RESIDUAL) {
        const int c = skinny_cols(EPI, g.N);
        if (c == 8) { launch_skinny_cols<EPI, MT, 8>(g, nw, s); return; }
        if (c == 12) { launch_skinny_cols<EPI, MT, 12>(g, nw, s); return; }
    }
    launch_skinny_cols<EPI, MT, 16>(g, nw, s);
}

// Dispatch thresholds.  Each is a measured crossover (figures at its use); the product build compiles them in
// as constants.  Only a build with -DAX_TUNING_KNOBS (kernel tuning sessions) lets the environment override them.
#ifdef AX_TUNING_KNOBS
static int env_int(const char* name, int dflt) {
    const char* v = std::getenv(name);
    return v && *v ? std::atoi(v) : dflt;
}
#else
static constexpr int env_int(const char*, int dflt) { return dflt; }
#endif
static const int kSwigluStreamMinNK = env_int("AX_SWIGLU_STREAM_MIN_NK", 0);   // measurement switch: gate/up weights (2^20) per matrix from which verify-size calls stream (0 = never)
static const int kStreamTm = env_int("AX_STREAM_TM", 1);   // experiment knob: 0 = always 128-row blocks
static const int kSwigluWaves = env_int("AX_SWIGLU_WAVES", 4096);   // wavefronts in flight the SwiGLU launch aims for (two weight streams per wavefront)
static const int kLmStream = env_int("AX_LM_STREAM", 1);   // experiment knob
static const int kSkinnyMaxM = std::min(32, env_int("AX_SKINNY_MAX_M", 32));   // experiment knob: rows up to which the skinny kernel may run
static const int kForceNW = env_int("AX_SKINNY_NW", 0);   // experiment knob: wavefronts per block, 0 = automatic

// More rows: LDS-staged tiles.
static const int kStreamMinBlocks = env_int("AX_STREAM_MIN_BLOCKS", 128);
static const int kStreamMinM = env_int("AX_STREAM_MIN_M", 512);   // rows from which QKV / residual GEMMs stream their weights (0 = never)
static const int kSliceMinM = env_int("AX_SLICE_MIN_M", 257);   // rows from which the down projection may stream over K slices
static const int kSliceStream = env_int("AX_SLICE_STREAM", 1);   // experiment knob
static const int kMidStream = env_int("AX_MID_STREAM", 1);   // experiment knob: 0 = tile kernels for 129-192 rows
static const int kQkvTile = env_int("AX_QKV_TILE", -1);   // experiment knobs: force 64-row (0) or 128-row (1) blocks
static const int kResTile = env_int("AX_RES_TILE", -1);
static const int kResBig = env_int("AX_RES_BIG", 256);
static const int kQkvKs = env_int("AX_QKV_KS", 0);   // experiment knob: K slices of the QKV GEMM (1 = never split)
template <int EPI>
static int launch_lds_tile(const GemmArgs& g, hipStream_t s) {
    const int M = g.M, N = g.N, K = g.K;
    // Two block shapes, both of 8 wavefronts: 64 x 128 (2 x 4 wavefronts of 32 x 32) and 128 x 128
    // (wavefront tile 64 x 32).  The larger one pulls a third fewer operand bytes per output and
    // wins wherever it still gives the chip enough blocks (measured per GEMM class below).
    const long long tiles64 = (long long)((N + 127) / 128) * ((M + 63) / 64);
    const long long tiles128 = (long long)((N + 127) / 128) * ((M + 127) / 128);
    // 128-row blocks only when their row padding costs at most ~15 % more rows than 64-row blocks' (M = 144 does not qualify)
    const bool pad_ok = (long long)((M + 127) / 128) * 128 * 100 <= (long long)((M + 63) / 64) * 64 * 115;
    // Calls with several hundred rows or more: the streaming kernel (weights straight to the MFMA
    // operands, 128 x 256 blocks, one block per CU at a time) where its blocks fill the 256 CUs
    // evenly - a single round of 128 or more blocks (160 for the down projection, which otherwise
    // goes over K slices), or rounds that are at least 3/4 full - and,
    // for the residual GEMMs, only with the long K of the down projection.  Measured against the
    // tile kernel: ~8B QKV 94-101 -> 81 us at M = 704-768, 106 -> 88 at 1024, 326 -> 278 at 3584;
    // ~8B down 293 -> 259 at 2048 and 558 -> 493 at 3584, ~3B down 168 -> 153 at 2048; O projections
    // and half-empty last rounds (336 blocks) lose 5-40 % and stay with the tile kernel.
    const long long sblocks = (long long)((N + 255) / 256) * ((M + 127) / 128), rounds = (sblocks + 255) / 256;
    const bool stream = kStreamMinM > 0 && M >= kStreamMinM && N % 32 == 0 && sblocks >= (EPI == EPI_RESIDUAL ? 160 : kStreamMinBlocks) &&
                        (rounds == 1 || sblocks * 4 >= rounds * 256 * 3) && (EPI != EPI_RESIDUAL || K >= 8192);
    // 129-192 rows (16 sessions verified together), residual GEMM with a long K (down projection):
    // one 160- or 192-row streaming block per 128 columns reads every weight once (64-row tiles
    // pull it three times out of L2) and K slices give the chip its ~200 blocks: ~3B down
    // projection at M = 144 36 -> 27 us.  With the shorter K of the QKV and O projections the
    // slices are too short for a kernel with one wavefront per SIMD (QKV 24 -> 29 us): tile kernels.
    const int mid_cb = (N + 127) / 128;
    int mid_ks = 1;
    const bool split = g.a_lo_off != 0;   // split activations: streaming blocks of at most 128 rows (a second A ring does not fit the registers of larger ones)
    if (EPI == EPI_RESIDUAL && kMidStream && !split && M > 128 && M <= 192 && K >= 8192 && N % 64 == 0 && g.split_ws)
        for (int ks : {8, 6, 4, 3, 2})
            if (mid_ks == 1 && mid_cb * ks <= 288 && K % (ks * 64) == 0 && K / (ks * 64) >= 4 &&
                (size_t)ks * 2 * M * N * sizeof(float) <= g.split_ws_bytes)
                mid_ks = ks;
    if constexpr (EPI == EPI_QKV) {
        if (stream && (size_t)M * N * sizeof(float) <= g.split_ws_bytes) {
            GemmArgs gs = g;
            gs.ksplit = 1;
            GemmArgs gp = gs;
            gp.ssq = nullptr;
            gp.Cf = g.split_ws;
            const int gx = (N + 255) / 256, gy = (M + 127) / 128;
            AX_SPLIT_LAUNCH(gp.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_STORE_F32, 4, 3, 2, false), gx * gy, 256, gp, gx, gy);
            qkv_reduce_rope_kernel<<<dim3((unsigned)M, (unsigned)((N / 2 + 255) / 256)), 256, 0, s>>>(gs);
            return 0;
        }
        // A plain store GEMM writes fp32 products, a second kernel does the rms scaling, rotary
        // embedding and KV append: measured faster than a fused epilogue (one head per wavefront)
        // at every size tried (M = 256 / 512, all three model shapes).  With few tiles K is cut in
        // two slices that the second kernel adds up.
        // (The workspace holds at least one [M, N] fp32 slab - a model's layout reserves max_tokens x N of it
        // whatever the ratio of N to d_model; a caller that brings less gets nothing launched.)
        // 128-row blocks from 80 tiles up (~3B / ~8B at M = 256: 36 -> 29 / 43 -> 34 us; M = 3584:
        // 275 -> 221 / 443 -> 329 us); the ~1B shape at M = 256 has 48 such tiles and stays with 64 rows
        const bool big = kQkvTile >= 0 ? kQkvTile > 0 : (pad_ok && tiles128 >= 80);
        // 64-row blocks: two slices only while both fit one round of 256 blocks (more blocks than CUs run two to a
        // CU and gain nothing from the cut: ~1B at 384 rows 26.8 -> 24.7 us, ~3B / ~8B at 320 rows 35.2 -> 32.3 / 43.0 -> 39.1 us)
        int ks = big ? (tiles128 < 128 ? 2 : 1) : (tiles64 * 2 <= 256 ? 2 : 1);
        // three slices where they fill the chip better than two and K divides (~3B at 193-256 rows: 80 tiles,
        // 240 blocks instead of 160: 30.6 -> 28.8 us; four slices, 320 blocks in two rounds: 37.5 us)
        if (big && ks == 2 && tiles128 * 3 <= 256 && K % (3 * 64) == 0 && K / (3 * 64) >= 8 &&
            (size_t)3 * M * N * sizeof(float) <= g.split_ws_bytes)
            ks = 3;
        if (kQkvKs > 0) ks = kQkvKs;
        while (ks > 1 && (K % (ks * 64) != 0 || (size_t)ks * M * N * sizeof(float) > g.split_ws_bytes)) ks >>= 1;
        if (!g.split_ws || (size_t)M * N * sizeof(float) > g.split_ws_bytes) return -1;
        GemmArgs gs = g;
        gs.ksplit = ks;
        GemmArgs gp = gs;                                 // the products: no scaling, no epilogue work
        gp.ssq = nullptr;
        gp.Cf = g.split_ws;
        if (big) {
            dim3 grid((N + 127) / 128, (M + 127) / 128, ks);
            AX_SPLIT_LAUNCH(gp.a_lo_off != 0, gemm_bf16_tile_kernel, (EPI_STORE_F32, 2, 1, 2, 4), grid, 512, gp);
        } else {
            dim3 grid((N + 127) / 128, (M + 63) / 64, ks);
            AX_SPLIT_LAUNCH(gp.a_lo_off != 0, gemm_bf16_tile_kernel, (EPI_STORE_F32, 1, 1, 2, 4), grid, 512, gp);
        }
        qkv_reduce_rope_kernel<<<dim3((unsigned)M, (unsigned)((N / 2 + 255) / 256)), 256, 0, s>>>(gs);
        return 0;
    } else if constexpr (EPI == EPI_RESIDUAL) {
        if (mid_ks > 1 && mid_cb * mid_ks >= 160) {            // (~1B width: 128 blocks, slower than the tile kernels)
            GemmArgs gs = g;
            gs.ksplit = mid_ks;
            if (M <= 160) gemm_bf16_stream_kernel<EPI_RESIDUAL, 5, 3, 1, true, false><<<mid_cb * mid_ks, 256, 0, s>>>(gs, mid_cb, 1);
            else gemm_bf16_stream_kernel<EPI_RESIDUAL, 6, 3, 1, true, false><<<mid_cb * mid_ks, 256, 0, s>>>(gs, mid_cb, 1);
            return launch_residual_reduce(gs, s);
        }
        if (stream) {
            const int gx = (N + 255) / 256, gy = (M + 127) / 128;
            AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_RESIDUAL, 4, 3, 2, false), gx * gy, 256, g, gx, gy);
            return N / 32;
        }
        // a few hundred rows against the long K of the down projection: too few 128 x 256 blocks for
        // the streaming kernel as it is, enough once K is cut into 2-4 slices (160-256 blocks).
        // Against the tile kernel: ~8B 107 -> 70 us at M = 288-320, 85 -> 71 at 384, 145 -> 118 at 768, 145 -> 131 at 1024;
        // ~3B 58 -> 50 at 512, 93 -> 78 at 1024; ~1B 57 -> 49 at 768.
        if (kSliceStream && M >= kSliceMinM && K >= 8192 && N % 64 == 0 && g.split_ws) {
            int ks = 1;
            for (int c : {4, 3, 2})                        // one block per CU at a time: at most 256 blocks
                if (ks == 1 && sblocks * c <= 256 && K % (c * 64) == 0 && K / (c * 64) >= 16 &&
                    (size_t)c * 2 * M * N * sizeof(float) <= g.split_ws_bytes)
                    ks = c;
            if (ks > 1 && sblocks * ks >= (ks == 2 ? 128 : 160)) {       // two slices pay from half the CUs up (~3B at 704-768 rows: 88 -> 74 us)
                GemmArgs gs = g;
                gs.ksplit = ks;
                const int gx = (N + 255) / 256, gy = (M + 127) / 128;
                AX_SPLIT_LAUNCH(gs.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_RESIDUAL, 4, 3, 2, true), gx * gy * ks, 256, gs, gx, gy);
                return launch_residual_reduce(gs, s);
            }
        }
        // Few output tiles (M = 256 against N = 2048 is 64 tiles of 64 x 128 for 256 CUs): cut K
        // until there are ~256 blocks, each still with 8 or more k-steps; fp32 partial slabs go to
        // the workspace and residual_reduce_kernel finishes.
        auto slices = [&](long long tiles) {
            int ks = 1;
            if (!g.split_ws || N % 64 != 0) return ks;
            // (a cut that would overshoot one round of 256 blocks is not taken once 144 or more CUs have a block:
            // ~3B at 193-256 rows, 96 tiles: 192 blocks instead of 384, O projection 20.6 -> 18.7 us, down projection -
            // then on 128-row blocks, 4 slices, 192 blocks - 39.1 -> 30.7 us; ~1B at 384 rows 37.5 -> 30.2 us,
            // ~8B O projection at 384 rows 39.3 -> 31.0 us, ~3B at 144 rows 18.5 -> 16.8 us)
            static const int fill = env_int("AX_SLICE_FILL", 144);   // measurement switch: 256 = always cut up to a full round
            while (ks < SPLITK_MAX && tiles * ks < 256 && !(tiles * ks >= fill && tiles * ks * 2 > 256) &&
                   K % (ks * 2 * 64) == 0 && K / (ks * 2 * 64) >= 8 && (size_t)ks * 2 * M * N * sizeof(float) <= g.split_ws_bytes)
                ks *= 2;
            return ks;
        };
        // 128-row blocks: when there are plenty of tiles without any cut (or more 64-row tiles than one
        // round of two per CU: ~3B O projection at 704-768 rows 52 -> 45-48 us), or when K is long (down
        // projection) and at most 4 slices give ~200 blocks or more.  Measured against 64-row
        // blocks: ~8B down projection 57 -> 49 us at M = 256, 98 -> 81 at 512, 907 -> 564 at 3584;
        // ~1B at M = 256 would need 8 slices and is no faster, so it keeps 64-row blocks.
        const int ks128 = slices(tiles128);
        const bool big = kResTile >= 0 ? kResTile > 0 : (M > 128 && pad_ok && (tiles128 >= kResBig || tiles64 > 256 || (K >= 4096 && ks128 <= 4 && tiles128 * ks128 >= 192)));
        const int ks = big ? ks128 : slices(tiles64);
        GemmArgs gs = g;
        gs.ksplit = ks;
        if (big) {
            dim3 grid((N + 127) / 128, (M + 127) / 128, ks);
            AX_SPLIT_LAUNCH(gs.a_lo_off != 0, gemm_bf16_tile_kernel, (EPI_RESIDUAL, 2, 1, 2, 4), grid, 512, gs);
        } else {
            dim3 grid((N + 127) / 128, (M + 63) / 64, ks);
            AX_SPLIT_LAUNCH(gs.a_lo_off != 0, gemm_bf16_tile_kernel, (EPI_RESIDUAL, 1, 1, 2, 4), grid, 512, gs);
        }
        return ks > 1 ? launch_residual_reduce(gs, s) : N / 32;
    } else if constexpr (EPI == EPI_SWIGLU) {
        // 17-192 rows: one streaming block of all the rows (32 to 192) per 128 columns, over K slices
        // (raw gate | up products in slabs, swiglu_reduce_kernel finishes): every weight is read
        // once and the slices give the chip ~256 blocks, where the tile kernels have 64 blocks (up
        // to 64 rows: no K slices for two products) or pull every weight twice out of L2, and the
        // skinny kernel re-reads its activations per 16 columns.  ~3B shape: 33 -> 26 us at 32 rows,
        // 48 -> 28 us at 64 rows, 49 -> 42 us at 144 rows; ~8B: 72 -> 48 us at 32-48 rows.
        // (above 128 rows only for matrices of the ~3B size or larger: at the ~1B size the 128 x 64 tiles are as fast or faster)
        if (kMidStream && M <= (split ? 128 : 192) && (M <= 128 || (long long)N * K >= (20LL << 20)) && g.split_ws) {
            const int cb = (N + 127) / 128;
            int ks = 1;
            for (int c : {8, 6, 4, 3, 2})
                if (ks == 1 && cb * c <= 288 && K % (c * 64) == 0 && K / (c * 64) >= 6 &&
                    (size_t)c * 2 * M * N * sizeof(float) <= g.split_ws_bytes)
                    ks = c;
            if (ks > 1 && cb * ks >= 128) {
                GemmArgs gs = g;
                gs.ksplit = ks;
                const unsigned nb = (unsigned)(cb * ks);
                switch ((M + 31) / 32) {
                    case 1: AX_SPLIT_LAUNCH(gs.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_SWIGLU, 1, 3, 2, true), nb, 256, gs, cb, 1); break;
                    case 2: AX_SPLIT_LAUNCH(gs.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_SWIGLU, 2, 3, 2, true), nb, 256, gs, cb, 1); break;
                    case 3: AX_SPLIT_LAUNCH(gs.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_SWIGLU, 3, 3, 2, true), nb, 256, gs, cb, 1); break;
                    case 4: AX_SPLIT_LAUNCH(gs.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_SWIGLU, 4, 3, 2, true), nb, 256, gs, cb, 1); break;
                    case 5: gemm_bf16_stream_kernel<EPI_SWIGLU, 5, 3, 2, true, false><<<nb, 256, 0, s>>>(gs, cb, 1); break;
                    default: gemm_bf16_stream_kernel<EPI_SWIGLU, 6, 3, 2, true, false><<<nb, 256, 0, s>>>(gs, cb, 1); break;
                }
                swiglu_reduce_kernel<<<dim3((unsigned)M, (unsigned)((N + 255) / 256)), 256, 0, s>>>(gs);
                return 0;
            }
        }
        // gate/up with two or more 128-row tiles: 128 x 64 tiles make a CU pull (128 + 2 * 64) rows of
        // operands per k instead of (64 + 2 * 128) for the same number of blocks (2-3 % faster)
        if (M > 128) {
            dim3 tgrid((N + 63) / 64, (M + 127) / 128);
            AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_tile_kernel, (EPI_SWIGLU, 1, 1, 4, 2), tgrid, 512, g);
            return 0;
        }
    }
    if constexpr (EPI == EPI_STORE_F32 || EPI == EPI_SWIGLU) {
        // logits (N >= 64 K columns) of 17 rows or more: streaming blocks of up to 192 rows per 256 columns
        // read the LM head once per block row at 5-6 TB/s; the skinny kernel re-reads its activations
        // per 16 columns (17 rows of the ~3B shape: 182 -> 128 us) and 64-row tiles read the weights
        // once per tile (96-128 rows: 282-294 -> 149-157 us; 144 rows: 436 -> 202 us).  Rows per
        // block by the same rounds x block cost as the SwiGLU kernel.
        if (EPI == EPI_STORE_F32 && M > 16 && N >= 256 * 256 && N % 32 == 0 && kLmStream) {
            const int gx = (N + 255) / 256;
            int tm = (M + 31) / 32;
            if (M > 512) {
                tm = 4;                                    // compute-bound there: 128-row blocks (1024 rows: 669 us against 804 with 192-row blocks)
            } else if (tm > (split ? 4 : 6)) {
                long long best = -1;
                for (int t : {4, 3, 5, 6}) {
                    if (split && t > 4) continue;
                    const long long blocks = (long long)gx * ((M + 32 * t - 1) / (32 * t));
                    const long long cost = ((blocks + 255) / 256) * (32 * t + 512) * (t >= 5 ? 115 : 100);
                    if (best < 0 || cost < best) { best = cost; tm = t; }
                }
            }
            const int gy = (M + 32 * tm - 1) / (32 * tm);
            switch (tm) {
                case 1: AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_STORE_F32, 1, 3, 2, false), gx * gy, 256, g, gx, gy); break;
                case 2: AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_STORE_F32, 2, 3, 2, false), gx * gy, 256, g, gx, gy); break;
                case 3: AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_STORE_F32, 3, 3, 2, false), gx * gy, 256, g, gx, gy); break;
                case 4: AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_STORE_F32, 4, 3, 2, false), gx * gy, 256, g, gx, gy); break;
                case 5: gemm_bf16_stream_kernel<EPI_STORE_F32, 5, 3, 2, false, false><<<gx * gy, 256, 0, s>>>(g, gx, gy); break;
                default: gemm_bf16_stream_kernel<EPI_STORE_F32, 6, 3, 2, false, false><<<gx * gy, 256, 0, s>>>(g, gx, gy); break;
            }
            return 0;
        }
        if (EPI == EPI_STORE_F32 && stream) {              // logits of thousands of rows
            const int gx = (N + 255) / 256, gy = (M + 127) / 128;
            AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_STORE_F32, 4, 3, 2, false), gx * gy, 256, g, gx, gy);
            return 0;
        }
        dim3 grid((N + 127) / 128, (M + 63) / 64);
        AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_tile_kernel, (EPI, 1, 1, 2, 4), grid, 512, g);
    }
    return 0;
}

// Which rows go to the skinny kernel: a block of it re-reads the whole activation slice of its
// wavefronts (M x K / NW fp16) per 8-16 columns, so its time grows with M while one 64-row tile
// costs the same for any M <= 64.  Measured crossovers (all three model shapes): every GEMM is
// faster on the other kernels from 33 rows up (64 rows of the ~3B shape: 172 -> 114 us per layer);
// from 17 rows up the QKV GEMM and the residual GEMM with the long K (down projection) are too
// (~3B at 17-32 rows: 18-22 -> 17-19 us and 18-23 -> 15-16 us) and so is the SwiGLU GEMM on its
// K-sliced streaming blocks (see launch_lds_tile); the O projection is not.
static bool use_skinny(int epi, int M, int N, int K) {
    // (the largest gate/up matrices - ~8B shape, 2 x 59 M weights - once streamed faster through the K-sliced
    // streaming blocks even at verify sizes, 51 -> 44 us at 9 rows; since this kernel skips activation rows
    // past M and finishes 1 / rms behind its first loads it is ahead again: 37.8 / 38.3 / 41.0 us at 1 / 9 / 16
    // rows against 41.9 / 42.1 / 42.2.  The switch stays for measurements: weights (2^20) per matrix from which to stream.)
    if (epi == EPI_SWIGLU && kSwigluStreamMinNK > 0 && (long long)N * K >= (long long)kSwigluStreamMinNK << 20) return false;
    if (M <= 16) return true;
    if (M > kSkinnyMaxM) return false;
    if (epi == EPI_STORE_F32 && N >= 256 * 256 && kLmStream) return false;    // logits: streaming blocks (see launch_lds_tile)
    // (re-measured on whole verify steps of 17 rows, ~3B shape, 2.50 ms per step: keeping the QKV / SwiGLU / down
    // GEMM on this kernel there - no reduce kernel behind them - gives 2.50 / 2.52 / 2.58 ms, all three 2.59 ms)
    return !(epi == EPI_QKV || epi == EPI_SWIGLU || (epi == EPI_RESIDUAL && K >= 2 * N));
}

template <int EPI>
static int launch_bf16(const GemmArgs& g, hipStream_t s) {
    const int M = g.M, N = g.N, K = g.K;
    if (use_skinny(EPI, M, N, K)) {
        // wavefronts per block (= K slices): enough to keep ~2k wavefronts in flight (~4k for the SwiGLU
        // GEMM: 8 instead of 4 wavefronts per block took the ~1B verify kernel from 16.6 to 14.7 us), each with
        // at least 128 of K; K / nw must stay a multiple of the MFMA k (32)
        const int cols = skinny_cols(EPI, N);
        const long long tiles = (N + cols - 1) / cols;
        int nw = 1;
        const int wave_target = EPI == EPI_SWIGLU ? kSwigluWaves : 2048;
        while (nw < 16 && tiles * nw < wave_target && K % (nw * 2 * 32) == 0 && K / (nw * 2) >= 128) nw *= 2;
        if (kForceNW > 0 && K % (std::max(kForceNW, 1) * 32) == 0) nw = kForceNW;
        if (EPI == EPI_SWIGLU && nw == 16) nw = 8;        // LDS reduction buffer stays <= 64 KB
        if (M <= 16) launch_skinny_nw<EPI, 1>(g, nw, s);
        else launch_skinny_nw<EPI, 2>(g, nw, s);
        return EPI == EPI_RESIDUAL ? N / cols : 0;
    }
    // streaming SwiGLU kernel: from three 128-row blocks up, and with two when the matrix is wide
    // enough for ~200 blocks (~8B shape at 193-256 rows: 118 -> 97 us; ~1B / ~3B have 128 blocks
    // there and lose: 32 -> 52, 45 -> 68 us)
    if (EPI == EPI_SWIGLU && (M > 256 || (M > 192 && (long long)((N + 127) / 128) * ((M + 127) / 128) >= 192))) {
        // rows per block: 96, 128, 160 or 192.  One block runs per CU at a time, so a launch takes
        // (rounds of 256 blocks) x (time of a block), and a block's time grows with the operand rows
        // it pulls (its activation rows + 2 x 128 weight rows): pick the shape with the smallest
        // product.  257 rows of the ~1B shape: 3 x 96 rows (192 blocks) instead of 3 x 128, 56 -> 45 us;
        // 640 rows: 4 x 160 (256 blocks, one round) instead of 5 x 128 (320 blocks, two), 99 -> 65 us.
        int tm = 4;
        if (kStreamTm) {
            long long best = -1;
            for (int t : {4, 3, 5, 6}) {
                if (g.a_lo_off != 0 && t > 4) continue;      // split activations: at most 128-row blocks
                const long long blocks = (long long)((N + 127) / 128) * ((M + 32 * t - 1) / (32 * t));
                const long long cost = ((blocks + 255) / 256) * (32 * t + 256) * (t >= 5 ? 115 : 100);   // the two large shapes run ~15 % below the model
                if (best < 0 || cost < best) { best = cost; tm = t; }
            }
        }
        const int gx = (N + 127) / 128, gy = (M + 32 * tm - 1) / (32 * tm);
        switch (tm) {
            case 3: AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_SWIGLU, 3, 3, 2, false), gx * gy, 256, g, gx, gy); break;
            case 5: gemm_bf16_stream_kernel<EPI_SWIGLU, 5, 3, 2, false, false><<<gx * gy, 256, 0, s>>>(g, gx, gy); break;
            case 6: gemm_bf16_stream_kernel<EPI_SWIGLU, 6, 3, 2, false, false><<<gx * gy, 256, 0, s>>>(g, gx, gy); break;
            default: AX_SPLIT_LAUNCH(g.a_lo_off != 0, gemm_bf16_stream_kernel, (EPI_SWIGLU, 4, 3, 2, false), gx * gy, 256, g, gx, gy); break;
        }
        return 0;
    }
    return launch_lds_tile<EPI>(g, s);
}

int launch_gemm_bf16(Epilogue epi, const GemmArgs& g, hipStream_t s) {
    if (epi == EPI_STORE_F32) return launch_bf16<EPI_STORE_F32>(g, s);
    if (epi == EPI_RESIDUAL) return launch_bf16<EPI_RESIDUAL>(g, s);
    if (epi == EPI_SWIGLU) return launch_bf16<EPI_SWIGLU>(g, s);
    return launch_bf16<EPI_QKV>(g, s);
}

void launch_gemm(DType dt, Epilogue epi, const void* A, const void* W, const void* W2, void* C,
                 int M, int N, int K, hipStream_t s) {
    if (dt == F32) {
        launch_gemm_f32(epi, (const float*)A, (const float*)W, (const float*)W2, (float*)C, M, N, K, s);
        return;
    }
    GemmArgs g{};
    g.A = A; g.W = W; g.W2 = W2; g.M = M; g.N = N; g.K = K;
    g.Cf = (float*)C;
    g.C16 = C;
    launch_gemm_bf16(epi, g, s);
}

}  // namespace ax
