// Geometry of the paged KV pool, shared by the host bookkeeping (plain C++) and the kernels.
#pragma once

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define AX_HOST_DEVICE __host__ __device__
#else
#define AX_HOST_DEVICE
#endif

namespace ax {

// Element offsets (not bytes):
//   K(l, hk, blk, slot, c) = (((l*2 + 0)*Hkv + hk)*n_blocks + blk)*B*hd + slot*hd + c
//   V(l, hk, blk, c, slot) = (((l*2 + 1)*Hkv + hk)*n_blocks + blk)*B*hd + c*B + slot
struct KVGeom {
    void* base;
    long long n_blocks;
    int n_kv_heads, head_dim, block_tokens;
    AX_HOST_DEVICE long long plane(int layer, int kv, int hk) const {
        return ((long long)(layer * 2 + kv) * n_kv_heads + hk) * n_blocks * block_tokens * head_dim;
    }
};

}  // namespace ax
