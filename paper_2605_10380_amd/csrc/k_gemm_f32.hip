// fp32 GEMM for fp32-weight models: C = A[M,K] * W[N,K]^T, plain vector FMAs with fp32
// accumulation, any M, N, K.  The fp32 configuration is the exactness configuration (1e-4
// against the float64 oracle), so no reduced-precision matrix instruction is used here.
// 64x64 output tile per 256-thread block, 4x4 outputs per thread, K staged through LDS in
// slices of 16 (stored k-major so the inner loop reads float4 rows without bank conflicts).
#include "kernels.h"

namespace ax {

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A,
                                                       const float* __restrict__ W,
                                                       const float* __restrict__ W2,
                                                       float* __restrict__ C, int M, int N, int K) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float sA[BK][BM + 4];
    __shared__ float sB[BK][BN + 4];
    __shared__ float sB2[EPI == EPI_SWIGLU ? BK : 1][BN + 4];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;          // thread's 4 columns / 4 rows
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    // loader: 64 rows x 16 k = 1024 elements per operand, 4 per thread: row = tid/4, k = (tid%4)*4..+3
    const int lr = tid >> 2, lk = (tid & 3) * 4;

    float acc[4][4] = {};
    float acc2[4][4] = {};

    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = k0 + lk + i;
            const int am = m0 + lr, bn = n0 + lr;
            sA[lk + i][lr] = (am < M && k < K) ? A[(long long)am * K + k] : 0.f;
            sB[lk + i][lr] = (bn < N && k < K) ? W[(long long)bn * K + k] : 0.f;
            if (EPI == EPI_SWIGLU) sB2[lk + i][lr] = (bn < N && k < K) ? W2[(long long)bn * K + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], b[4], b2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = sB[kk][tx * 4 + j];
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int j = 0; j < 4; ++j) b2[j] = sB2[kk][tx * 4 + j];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
                    if (EPI == EPI_SWIGLU) acc2[i][j] = fmaf(a[i], b2[j], acc2[i][j]);
                }
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float* c = C + (long long)m * N + n;
            if (EPI == EPI_STORE_F32) {
                *c = acc[i][j];
            } else if (EPI == EPI_RESIDUAL) {
                *c += acc[i][j];
            } else {
                const float g = acc[i][j];
                *c = g / (1.0f + expf(-g)) * acc2[i][j];
            }
        }
    }
}

void launch_gemm_f32(Epilogue epi, const float* A, const float* W, const float* W2, float* C,
                     int M, int N, int K, hipStream_t s) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    if (epi == EPI_STORE_F32)
        gemm_f32_kernel<EPI_STORE_F32><<<grid, 256, 0, s>>>(A, W, W2, C, M, N, K);
    else if (epi == EPI_RESIDUAL)
        gemm_f32_kernel<EPI_RESIDUAL><<<grid, 256, 0, s>>>(A, W, W2, C, M, N, K);
    else
        gemm_f32_kernel<EPI_SWIGLU><<<grid, 256, 0, s>>>(A, W, W2, C, M, N, K);
}

}  // namespace ax
