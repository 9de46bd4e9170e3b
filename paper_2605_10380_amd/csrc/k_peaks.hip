// k_peaks.hip - what this machine delivers, measured beside the nominal peaks: a read-only
// stream over a caller's buffer (HBM read rate), a register-resident MFMA loop (fp16 matrix
// rate), and the two ways to order dependent phases of a step (a kernel boundary on one stream
// against a barrier across the workgroups of one resident kernel).  Test / bench support only;
// nothing on the serving path calls these.
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

// A barrier across all workgroups of a launch whose workgroups are all resident, `rounds` times.
// Two levels, so that no counter takes more than gridDim.x / 8 arrivals: workgroups are dealt to the
// 8 XCDs round robin, group g = blockIdx.x % 8 counts its arrivals on its own 128-byte line, the last
// arrival of a group counts on the master line, the last group stores the round number into the 8
// group flags, and every workgroup polls its group's flag (device-scope relaxed accesses between a
// release and an acquire fence).  Every wait is bounded: a workgroup that polls `spin_limit` times
// without success sets *err and leaves, and so do all others.
// ctr: 24 lines of 32 words, zero at launch (line 0 master, 1-8 group counters, 9-16 group flags).
__global__ void __launch_bounds__(512) grid_barrier_kernel(unsigned* __restrict__ ctr, int* __restrict__ err, int rounds, int spin_limit) {
    const unsigned grp = blockIdx.x & 7u, per = gridDim.x >> 3;
    unsigned* gc = ctr + 32 * (1 + grp);
    unsigned* gf = ctr + 32 * (9 + grp);
    for (unsigned r = 1; r <= (unsigned)rounds; ++r) {
        __syncthreads();
        bool ok = true;
        if (threadIdx.x == 0) {
            __threadfence();
            if (__hip_atomic_fetch_add(gc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == r * per &&
                __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == r * 8) {
                for (int g = 0; g < 8; ++g) __hip_atomic_store(ctr + 32 * (9 + g), r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            int spins = 0;
            while (__hip_atomic_load(gf, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < r) {
                if (++spins > spin_limit) { ok = false; *err = 1; break; }
                __builtin_amdgcn_s_sleep(2);
            }
            __threadfence();
        }
        if (!__syncthreads_and(ok)) return;
    }
}

__global__ void __launch_bounds__(512) boundary_kernel(unsigned* __restrict__ sink, unsigned never) {
    if (threadIdx.x == never) sink[0] = never;      // never: a kernel of the step's launch shape with nothing in it
}

void launch_grid_barrier(void* ctr, int* err, int blocks, int rounds, hipStream_t s) {
    grid_barrier_kernel<<<blocks, 512, 0, s>>>((unsigned*)ctr, err, rounds, 1 << 16);
}

void launch_boundary(void* sink, int blocks, hipStream_t s) {
    boundary_kernel<<<blocks, 512, 0, s>>>((unsigned*)sink, 0xffffffffu);
}

// What ONE compute unit can pull: every block (one per CU) reads its own region of `words` 16-byte words `passes`
// times, 8 wavefronts with four 16-byte loads in flight per lane (far more than the memory pipeline keeps outstanding).
// A 64 KB region is served by the XCD's L2 from the second pass on (it does not fit the CU's own cache and the loads are
// non-temporal); a region of several MB read once comes from HBM.
__global__ void __launch_bounds__(512) cu_fill_kernel(const pk_u32x4* __restrict__ src, size_t words, int passes, unsigned never,
                                                      unsigned* __restrict__ sink) {
    const pk_u32x4* base = src + (size_t)blockIdx.x * words;
    unsigned acc = 0;
    for (int p = 0; p < passes; ++p) {
        size_t i = threadIdx.x;
        for (; i + 3 * 512 < words; i += 4 * 512) {
            const pk_u32x4 a = __builtin_nontemporal_load(base + i), b = __builtin_nontemporal_load(base + i + 512);
            const pk_u32x4 c = __builtin_nontemporal_load(base + i + 1024), d = __builtin_nontemporal_load(base + i + 1536);
            acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
        }
        for (; i < words; i += 512) {
            const pk_u32x4 a = __builtin_nontemporal_load(base + i);
            acc ^= a.x ^ a.y ^ a.z ^ a.w;
        }
        acc = acc * 2654435761u + (unsigned)p;          // keeps the passes from being folded into one
    }
    if (acc == never) sink[0] = acc;
}

void launch_cu_fill(const void* src, size_t words_per_block, int blocks, int passes, void* sink, hipStream_t s) {
    cu_fill_kernel<<<blocks, 512, 0, s>>>((const pk_u32x4*)src, words_per_block, passes, 0x9e3779b9u, (unsigned*)sink);
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
