// k_peaks.hip - what this machine delivers, measured beside the nominal peaks: a read-only
// stream over a caller's buffer (HBM read rate) and a register-resident MFMA loop (fp16 matrix
// rate).  Test / bench support only; nothing on the serving path calls these.
#include <hip/hip_runtime.h>
#include "kernels.h"

namespace ax {

typedef _Float16 pk_f16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned pk_u32x4 __attribute__((ext_vector_type(4)));

// Every thread reads 16-byte words at a grid stride, four loads in flight per trip; the xor of
// what it read is stored only if it equals `never` (it does not), so nothing is written.
__global__ void __launch_bounds__(256) read_stream_kernel(const pk_u32x4* __restrict__ src, size_t n16,
                                                          unsigned never, unsigned* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const pk_u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        const pk_u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const pk_u32x4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == never) sink[0] = acc;
}

// Four independent 32x32x16 fp16 MFMA chains per wavefront, operands and accumulators in
// registers throughout: 4 * iters MFMAs of 32768 flops each per wavefront.
__global__ void __launch_bounds__(512) mfma_loop_kernel(int iters, float never, float* __restrict__ sink) {
    pk_f16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(0.001f * (float)((threadIdx.x + i) & 7));
        b[i] = (_Float16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
    }
    pk_f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == never) sink[0] = s;
}

void launch_read_stream(const void* src, size_t n16, void* sink, hipStream_t s) {
    read_stream_kernel<<<4096, 256, 0, s>>>((const pk_u32x4*)src, n16, 0x9e3779b9u, (unsigned*)sink);
}

// 2 blocks of 8 wavefronts per compute unit: 4 wavefronts per SIMD.
double launch_mfma_loop(int iters, void* sink, hipStream_t s) {
    const int blocks = 512, waves = 8;
    mfma_loop_kernel<<<blocks, waves * 64, 0, s>>>(iters, -1.0f, (float*)sink);
    return (double)blocks * waves * 4.0 * iters * 32768.0;
}

}  // namespace ax
