// Handle types of the C ABI and the registry of live handles.  Plain C++ (no HIP): the host-only
// half of the library (ax_host.cpp) builds with any C++17 compiler, e.g. under AddressSanitizer.
//
// A handle is valid iff the registry holds its address with the right kind.  Validation never
// reads the object itself, so a stale handle (freed, or never a handle at all) is rejected without
// touching freed memory.  (An address the allocator hands out again for a new object of the same
// kind is that new object's handle; stale copies of the old one then alias it, as with any
// pointer-valued handle.)
#pragma once

#include <cstdint>

#include "../../include/agentx.h"
#include "block_manager.h"
#include "kv_geom.h"
#include "ngram_lut.h"
#include "prefix_index.h"

struct ax_pool {
    uint64_t uid;                     // never reused: captured graphs are keyed by it
    ax_model_config cfg;              // geometry fields only are compared with the model's
    ax::KVGeom geom;
    ax::BlockPool blocks;
};

struct ax_kv {
    ax_pool* pool;
    ax::Sequence seq;
};

struct ax_lut {
    ax::NgramLut lut;
};

struct ax_index {
    ax_pool* pool;
    ax::PrefixIndex idx;
};

namespace ax {

enum HandleKind { H_MODEL = 1, H_POOL = 2, H_KV = 3, H_LUT = 4, H_INDEX = 5 };

void handle_register(const void* h, HandleKind kind);
void handle_unregister(const void* h);
bool handle_live(const void* h, HandleKind kind);      // thread safe; never dereferences h

// A live sequence keeps its pool alive (ax_pool_destroy refuses while sequences exist), so k->pool
// may be read once k itself is known to be live; an index may outlive a pool it holds nothing of.
inline bool ok(const ax_pool* p) { return handle_live(p, H_POOL); }
inline bool ok(const ax_kv* k) { return handle_live(k, H_KV) && handle_live(k->pool, H_POOL); }
inline bool ok(const ax_lut* l) { return handle_live(l, H_LUT); }
inline bool ok(const ax_index* x) { return handle_live(x, H_INDEX) && handle_live(x->pool, H_POOL); }

// Records the message ax_last_error returns on this thread; returns st.
ax_status fail(ax_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// INVALID for nonsense, UNSUPPORTED for shapes the kernels do not cover.
bool config_ok(const ax_model_config* c, ax_status* why);

inline int itemsize(int dtype) { return dtype == AX_F32 ? 4 : 2; }

// Whether a model keeps its activations as hi + lo fp16 pairs (ax_model_config.act_split; see agentx.h).
inline bool act_split_on(const ax_model_config& c) {
    if (c.dtype != AX_BF16 || c.act_split < 0) return false;
    return c.act_split > 0 || (long long)c.n_layers * c.d_model >= 131072;
}

}  // namespace ax
