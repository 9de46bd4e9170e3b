"""ctypes binding over the C ABI of libagentx.so (see include/agentx.h).

Argument marshalling only: every step of the extend / verify path runs inside the library's
HIP kernels.  PyTorch supplies device memory (weights, KV pool, workspace, outputs) and the
stream.  There is no CPU fallback: a missing library raises at import of this module.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libagentx.so")

AX_OK, AX_ERR_INVALID, AX_ERR_OOM, AX_ERR_DEVICE, AX_ERR_UNSUPPORTED, AX_ERR_STATE = 0, -1, -2, -3, -4, -5
AX_F32, AX_BF16 = 0, 1
AX_OUT_NONE, AX_OUT_LAST_LOGITS, AX_OUT_ALL_LOGITS, AX_OUT_LAST_ARGMAX, AX_OUT_ALL_ARGMAX = range(5)


class ax_model_config(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ff", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int), ("max_pos", C.c_int),
        ("max_tokens", C.c_int), ("max_seqs", C.c_int), ("act_split", C.c_int)]


class ax_exspec_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("rounds", "fallbacks", "drafted", "accepted")]


class ax_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + [
        (n, C.POINTER(C.c_void_p)) for n in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_mlp")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_10380_amd.build` "
                          "(there is no fallback path)")
    # PyTorch ships its own HIP runtime (same soname as the system one the library is linked
    # against).  Whichever is loaded first serves the whole process, and PyTorch only works with
    # its own: load it before the library so that both use that copy.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32p, i64 = C.c_void_p, C.POINTER(C.c_int32), C.c_int64
    sig = {
        "ax_last_error": (C.c_char_p, []),
        "ax_workspace_bytes": (C.c_size_t, [C.POINTER(ax_model_config)]),
        "ax_model_create": (C.c_int, [C.POINTER(ax_model_config), C.POINTER(ax_weights), vp, C.c_size_t, C.POINTER(vp)]),
        "ax_model_destroy": (None, [vp]),
        "ax_pool_block_bytes": (C.c_size_t, [C.POINTER(ax_model_config), C.c_int]),
        "ax_pool_create": (C.c_int, [C.POINTER(ax_model_config), vp, C.c_size_t, C.c_int, C.POINTER(vp)]),
        "ax_pool_destroy": (C.c_int, [vp]),
        "ax_pool_stats": (C.c_int, [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]),
        "ax_kv_alloc": (C.c_int, [vp, C.POINTER(vp)]),
        "ax_kv_fork": (C.c_int, [vp, i64, C.POINTER(vp)]),
        "ax_kv_truncate": (C.c_int, [vp, i64]),
        "ax_kv_len": (i64, [vp]),
        "ax_kv_free": (C.c_int, [vp]),
        "ax_kv_blocks": (i64, [vp, i32p, i64]),
        "ax_pool_refcount": (C.c_int, [vp, i64]),
        "ax_kv_reserve_host": (C.c_int, [vp, i64, i32p, i32p]),
        "ax_extend": (C.c_int, [vp, vp, i32p, C.c_int, C.c_int, vp, vp]),
        "ax_extend_batch": (C.c_int, [vp, C.c_int, C.POINTER(vp), i32p, C.POINTER(C.c_int), C.c_int, vp, vp]),
        "ax_kv_image_bytes": (i64, [vp, i64]),
        "ax_kv_export": (C.c_int, [vp, vp, i64, vp, i64, vp]),
        "ax_kv_import": (C.c_int, [vp, vp, vp, i64, C.POINTER(vp), vp]),
        "ax_kv_export_static": (C.c_int, [vp, i64, vp, i64, vp]),
        "ax_index_create": (C.c_int, [vp, C.POINTER(vp)]),
        "ax_index_destroy": (None, [vp]),
        "ax_index_entries": (i64, [vp]),
        "ax_index_insert": (C.c_int, [vp, vp, i32p, i64]),
        "ax_index_match": (C.c_int, [vp, i32p, i64, i64, C.POINTER(vp), C.POINTER(i64)]),
        "ax_select_combinations": (C.c_int, [i32p, i32p, i64, C.c_int, i32p, i64, i32p, C.POINTER(i64), C.POINTER(C.c_int)]),
        "ax_coverage": (i64, [i32p, i32p, i64, i32p, i32p, i64]),
        "ax_lut_build": (C.c_int, [i32p, i64, C.c_int, C.c_int, C.POINTER(vp)]),
        "ax_lut_free": (None, [vp]),
        "ax_lut_size": (i64, [vp]),
        "ax_lut_draft": (C.c_int, [vp, i32p, i64, C.c_int, C.c_int, C.c_uint64, i64, i32p, C.POINTER(C.c_int)]),
        "ax_exspec_generate": (C.c_int, [vp, vp, vp, i32p, i64, C.c_int32, C.c_int, C.c_int, C.c_int, C.c_uint64, i32p,
                                         C.POINTER(ax_exspec_stats), vp]),
        "ax_dbg_gemm": (C.c_int, [C.c_int, C.c_int, vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, vp]),
        "ax_dbg_gemm_time": (C.c_int, [C.c_int, C.c_int, vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_size_t,
                                       C.c_int, C.POINTER(C.c_float), vp]),
        "ax_dbg_gemm_residual": (C.c_int, [vp, vp, vp, vp, vp, vp, C.POINTER(C.c_int), C.c_int, C.c_int, C.c_int, vp,
                                           C.c_size_t, vp]),
        "ax_dbg_copy": (C.c_int, [vp, vp, C.c_size_t, vp]),
        "ax_dbg_cu_fill": (C.c_int, [vp, C.c_size_t, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]),
        "ax_dbg_check_guards": (C.c_int, [vp, C.POINTER(C.c_int)]),
        "ax_dbg_phase_order": (C.c_int, [vp, C.c_size_t, C.c_int, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]),
        "ax_dbg_peaks": (C.c_int, [vp, C.c_size_t, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float),
                                   C.POINTER(C.c_float), vp]),
        "ax_dbg_read": (C.c_int, [vp, C.c_int, vp, C.c_size_t]),
        "ax_dbg_profile": (C.c_int, [vp, C.c_int]),
        "ax_dbg_use_graphs": (C.c_int, [vp, C.c_int]),
        "ax_dbg_profile_read": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(i64)]),
        "ax_verify": (C.c_int, [vp, vp, C.c_int32, i32p, C.c_int, C.POINTER(C.c_int), i32p, vp]),
        "ax_verify_batch": (C.c_int, [vp, C.c_int, C.POINTER(vp), i32p, i32p, C.POINTER(C.c_int), C.POINTER(C.c_int), i32p, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


class AxError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"ax status {status}: {lib.ax_last_error().decode()}")


def _check(status: int):
    if status != AX_OK:
        raise AxError(status)


def make_config(shape, max_pos: int, max_tokens: int, max_seqs: int = 1, act_split: int = 0) -> ax_model_config:
    """act_split: 0 = the library decides (hi + lo fp16 activations for deep, wide bf16 models), 1 = on, -1 = off."""
    return ax_model_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                           shape.d_ff, shape.vocab, shape.rms_eps, shape.rope_base,
                           AX_F32 if shape.dtype == "f32" else AX_BF16, max_pos, max_tokens, max_seqs, act_split)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


# ------------------------------------------------------------------ paged KV (host only)

def ax_pool_block_bytes(cfg: ax_model_config, block_tokens: int = 16) -> int:
    return lib.ax_pool_block_bytes(C.byref(cfg), block_tokens)


def ax_pool_create(cfg: ax_model_config, dev_ptr: int, nbytes: int, block_tokens: int = 16) -> int:
    out = C.c_void_p()
    _check(lib.ax_pool_create(C.byref(cfg), C.c_void_p(dev_ptr), nbytes, block_tokens, C.byref(out)))
    return out.value


def ax_pool_destroy(pool: int):
    _check(lib.ax_pool_destroy(pool))


def ax_pool_stats(pool: int):
    f, t, s = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib.ax_pool_stats(pool, C.byref(f), C.byref(t), C.byref(s)))
    return f.value, t.value, s.value


def ax_kv_alloc(pool: int) -> int:
    out = C.c_void_p()
    _check(lib.ax_kv_alloc(pool, C.byref(out)))
    return out.value


def ax_kv_fork(src: int, n_tokens: int = -1) -> int:
    out = C.c_void_p()
    _check(lib.ax_kv_fork(src, n_tokens, C.byref(out)))
    return out.value


def ax_kv_truncate(kv: int, new_len: int):
    _check(lib.ax_kv_truncate(kv, new_len))


def ax_kv_len(kv: int) -> int:
    return lib.ax_kv_len(kv)


def ax_kv_free(kv: int):
    _check(lib.ax_kv_free(kv))


def ax_kv_blocks(kv: int):
    n = lib.ax_kv_blocks(kv, None, 0)
    if n < 0:
        raise AxError(AX_ERR_INVALID)
    ids = np.zeros(max(n, 1), dtype=np.int32)
    lib.ax_kv_blocks(kv, ids.ctypes.data_as(C.POINTER(C.c_int32)), n)
    return ids[:n]


def ax_pool_refcount(pool: int, block: int) -> int:
    return lib.ax_pool_refcount(pool, block)


def ax_kv_reserve_host(kv: int, n: int):
    s, d = C.c_int32(), C.c_int32()
    _check(lib.ax_kv_reserve_host(kv, n, C.byref(s), C.byref(d)))
    return s.value, d.value


# ------------------------------------------------------------------ model and forward (GPU)

def ax_workspace_bytes(cfg: ax_model_config) -> int:
    return lib.ax_workspace_bytes(C.byref(cfg))


def ax_model_create(cfg: ax_model_config, ptrs: dict, ws_ptr: int, ws_bytes: int) -> int:
    """ptrs: {"tok_emb": int, ..., "wqkv": [int per layer], ...} of device addresses."""
    w = ax_weights()
    keep = []
    for name in ("tok_emb", "lm_head", "final_norm"):
        setattr(w, name, ptrs[name])
    for name in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_mlp"):
        arr = (C.c_void_p * cfg.n_layers)(*ptrs[name])
        keep.append(arr)
        setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
    out = C.c_void_p()
    _check(lib.ax_model_create(C.byref(cfg), C.byref(w), C.c_void_p(ws_ptr), ws_bytes, C.byref(out)))
    return out.value


def ax_model_destroy(model: int):
    lib.ax_model_destroy(model)


def ax_extend(model: int, kv: int, tokens, out_mode: int = AX_OUT_NONE, out_ptr: int = 0, stream: int = 0):
    t, tp = _i32(tokens)
    _check(lib.ax_extend(model, kv, tp, len(t), out_mode, C.c_void_p(out_ptr), C.c_void_p(stream)))


def ax_extend_batch(model: int, kvs, tokens_concat, T_each, out_mode: int = AX_OUT_NONE, out_ptr: int = 0,
                    stream: int = 0):
    t, tp = _i32(tokens_concat)
    te = (C.c_int * len(T_each))(*[int(v) for v in T_each])
    ka = (C.c_void_p * len(kvs))(*kvs)
    _check(lib.ax_extend_batch(model, len(kvs), ka, tp, te, out_mode, C.c_void_p(out_ptr), C.c_void_p(stream)))


def ax_verify(model: int, kv: int, pending: int, drafts, stream: int = 0):
    d, dp = _i32(drafts)
    a, nxt = C.c_int(), C.c_int32()
    _check(lib.ax_verify(model, kv, int(pending), dp if len(d) else None, len(d), C.byref(a), C.byref(nxt),
                         C.c_void_p(stream)))
    return a.value, nxt.value


def ax_kv_image_bytes(pool: int, n_tokens: int) -> int:
    return lib.ax_kv_image_bytes(pool, n_tokens)


def ax_kv_export(model: int, kv: int, n_tokens: int, image_ptr: int, image_bytes: int, stream: int = 0):
    _check(lib.ax_kv_export(model, kv, n_tokens, C.c_void_p(image_ptr), image_bytes, C.c_void_p(stream)))


def ax_kv_export_static(kv: int, n_tokens: int, image_ptr: int, image_bytes: int, stream: int = 0):
    """Enqueues only: synchronise the stream before reading the image."""
    _check(lib.ax_kv_export_static(kv, n_tokens, C.c_void_p(image_ptr), image_bytes, C.c_void_p(stream)))


def ax_kv_import(model: int, pool: int, image_ptr: int, image_bytes: int, stream: int = 0) -> int:
    out = C.c_void_p()
    _check(lib.ax_kv_import(model, pool, C.c_void_p(image_ptr), image_bytes, C.byref(out), C.c_void_p(stream)))
    return out.value


def ax_verify_batch(model: int, kvs, pending, drafts_each, stream: int = 0):
    """drafts_each: one list of drafts per sequence.  Returns ([accepted], [next token])."""
    n = len(kvs)
    p, pp = _i32(pending)
    flat = [int(t) for d in drafts_each for t in d]
    d, dp = _i32(flat)
    ke = (C.c_int * n)(*[len(d_) for d_ in drafts_each])
    ka = (C.c_void_p * n)(*kvs)
    acc = (C.c_int * n)()
    nxt = np.zeros(n, dtype=np.int32)
    _check(lib.ax_verify_batch(model, n, ka, pp, dp if len(d) else None, ke, acc, nxt.ctypes.data_as(C.POINTER(C.c_int32)),
                               C.c_void_p(stream)))
    return list(acc), nxt.tolist()


# ------------------------------------------------------------------ prefix index and offline selection (host)

def ax_index_create(pool: int) -> int:
    out = C.c_void_p()
    _check(lib.ax_index_create(pool, C.byref(out)))
    return out.value


def ax_index_destroy(index: int):
    lib.ax_index_destroy(index)


def ax_index_entries(index: int) -> int:
    return lib.ax_index_entries(index)


def ax_index_insert(index: int, kv: int, tokens):
    t, tp = _i32(tokens)
    _check(lib.ax_index_insert(index, kv, tp, len(t)))


def ax_index_match(index: int, prompt, max_reuse: int = -1):
    """(new sequence handle, reused tokens)."""
    t, tp = _i32(prompt)
    out, m = C.c_void_p(), C.c_int64()
    _check(lib.ax_index_match(index, tp if len(t) else None, len(t), max_reuse, C.byref(out), C.byref(m)))
    return out.value, m.value


def _pack_seqs(seqs):
    flat = np.asarray([int(c) for s in seqs for c in s], dtype=np.int32)
    lens = np.asarray([len(s) for s in seqs], dtype=np.int32)
    p32 = C.POINTER(C.c_int32)
    return flat, lens, (flat.ctypes.data_as(p32) if len(flat) else None), (lens.ctypes.data_as(p32) if len(lens) else None)


def ax_select_combinations(samples, budget: int):
    """([chosen prefixes as tuples, in the order chosen], [coverage after each])."""
    flat, lens, fp, lp = _pack_seqs(samples)
    cap = max(1, budget * (int(lens.max()) if len(lens) else 1))
    out = np.zeros(cap, dtype=np.int32)
    out_len = np.zeros(max(budget, 1), dtype=np.int32)
    cov = np.zeros(max(budget, 1), dtype=np.int64)
    n = C.c_int()
    p32 = C.POINTER(C.c_int32)
    _check(lib.ax_select_combinations(fp, lp, len(lens), budget, out.ctypes.data_as(p32), cap, out_len.ctypes.data_as(p32),
                                      cov.ctypes.data_as(C.POINTER(C.c_int64)), C.byref(n)))
    chosen, at = [], 0
    for i in range(n.value):
        chosen.append(tuple(int(c) for c in out[at:at + out_len[i]]))
        at += out_len[i]
    return chosen, cov[:n.value].tolist()


def ax_coverage(samples, cached) -> int:
    _f, sl, fp, lp = _pack_seqs(samples)
    _g, cl, cp, clp = _pack_seqs(cached)
    return lib.ax_coverage(fp, lp, len(sl), cp, clp, len(cl))


# ------------------------------------------------------------------ example-based drafter (host) and decode loop

def ax_lut_build(stream, n: int, vocab: int) -> int:
    t, tp = _i32(stream)
    out = C.c_void_p()
    _check(lib.ax_lut_build(tp if len(t) else None, len(t), n, vocab, C.byref(out)))
    return out.value


def ax_lut_free(lut: int):
    lib.ax_lut_free(lut)


def ax_lut_size(lut: int) -> int:
    return lib.ax_lut_size(lut)


def ax_lut_draft(lut: int, context, k: int, selective: bool = True, seed: int = 0, stream_pos: int = 0):
    c, cp = _i32(context)
    d = np.zeros(max(k, 1), dtype=np.int32)
    hits = C.c_int()
    n = lib.ax_lut_draft(lut, cp if len(c) else None, len(c), k, int(selective), seed, stream_pos,
                         d.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(hits))
    if n < 0:
        raise AxError(AX_ERR_INVALID)
    return d[:n].tolist(), hits.value


def ax_exspec_generate(model: int, kv: int, lut: int, history, pending: int, max_new: int, k: int,
                       selective: bool = True, seed: int = 0, stream: int = 0):
    h, hp = _i32(history)
    out = np.zeros(max(max_new, 1), dtype=np.int32)
    st = ax_exspec_stats()
    _check(lib.ax_exspec_generate(model, kv, lut, hp if len(h) else None, len(h), int(pending), max_new, k, int(selective),
                                  seed, out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(st), C.c_void_p(stream)))
    return out[:max_new].tolist(), dict(rounds=st.rounds, fallbacks=st.fallbacks, drafted=st.drafted, accepted=st.accepted)


# ------------------------------------------------------------------ test-only entry points

def ax_dbg_gemm(dtype: int, epilogue: int, A: int, W: int, W2: int, Cptr: int, M: int, N: int, K: int, stream: int = 0):
    _check(lib.ax_dbg_gemm(dtype, epilogue, C.c_void_p(A), C.c_void_p(W), C.c_void_p(W2), C.c_void_p(Cptr), M, N, K,
                           C.c_void_p(stream)))


def ax_dbg_gemm_time(dtype: int, epilogue: int, A: int, W: int, W2: int, Cptr: int, M: int, N: int, K: int, iters: int,
                     w_stride_bytes: int = 0, w_count: int = 1, stream: int = 0) -> float:
    us = C.c_float()
    _check(lib.ax_dbg_gemm_time(dtype, epilogue, C.c_void_p(A), C.c_void_p(W), C.c_void_p(W2), C.c_void_p(Cptr), M, N, K,
                                iters, w_stride_bytes, w_count, C.byref(us), C.c_void_p(stream)))
    return us.value


def ax_dbg_gemm_residual(A: int, W: int, gain: int, x: int, a16: int, ssq: int, M: int, N: int, K: int,
                         split_ws: int = 0, split_ws_bytes: int = 0, stream: int = 0) -> int:
    """Returns the number of sum-of-squares partials per row the call wrote."""
    parts = C.c_int()
    _check(lib.ax_dbg_gemm_residual(C.c_void_p(A), C.c_void_p(W), C.c_void_p(gain), C.c_void_p(x), C.c_void_p(a16),
                                    C.c_void_p(ssq), C.byref(parts), M, N, K, C.c_void_p(split_ws), split_ws_bytes,
                                    C.c_void_p(stream)))
    return parts.value


def ax_dbg_copy(dst: int, src: int, nbytes: int, stream: int = 0):
    _check(lib.ax_dbg_copy(C.c_void_p(dst), C.c_void_p(src), nbytes, C.c_void_p(stream)))


def ax_dbg_peaks(buf: int, nbytes: int, reps: int = 5, stream: int = 0):
    """(GB/s of a read-only stream, GB/s of a plain copy counting both directions, fp16 MFMA TFLOP/s)."""
    r, c, m = C.c_float(), C.c_float(), C.c_float()
    _check(lib.ax_dbg_peaks(C.c_void_p(buf), nbytes, reps, C.byref(r), C.byref(c), C.byref(m), C.c_void_p(stream)))
    return r.value, c.value, m.value


def ax_dbg_cu_fill(buf: int, nbytes: int, stream: int = 0):
    """(GB/s one compute unit pulls out of its XCD's L2, GB/s per compute unit out of HBM with all of them pulling)."""
    a, b = C.c_float(), C.c_float()
    _check(lib.ax_dbg_cu_fill(C.c_void_p(buf), nbytes, C.byref(a), C.byref(b), C.c_void_p(stream)))
    return a.value, b.value


def ax_dbg_phase_order(buf: int, nbytes: int, blocks: int = 256, rounds: int = 200, stream: int = 0):
    """(microseconds per kernel boundary, microseconds per barrier across the workgroups of one resident kernel)."""
    a, b = C.c_float(), C.c_float()
    _check(lib.ax_dbg_phase_order(C.c_void_p(buf), nbytes, blocks, rounds, C.byref(a), C.byref(b), C.c_void_p(stream)))
    return a.value, b.value


def ax_dbg_read(model: int, which: int, dst: np.ndarray):
    assert dst.flags["C_CONTIGUOUS"]
    _check(lib.ax_dbg_read(model, which, dst.ctypes.data_as(C.c_void_p), dst.nbytes))
    return dst


PROFILE_CLASSES = ("qkv_proj", "attention", "o_proj", "swiglu_gate_up", "down_proj", "lm_head", "empty_bracket")


WORKSPACE_REGIONS = ("rotary cos", "rotary sin", "descriptor slots", "residual stream", "normed activations", "norm partial sums",
                     "fp32 qkv", "q", "attention output", "SwiGLU activations", "attention slice records", "GEMM slabs",
                     "logits chunk", "argmax scratch", "argmax output", "result words", "packed weights")


def ax_dbg_check_guards(model: int) -> int:
    """Index of the first workspace region whose guard bytes were overwritten, or -1."""
    bad = C.c_int(-1)
    _check(lib.ax_dbg_check_guards(model, C.byref(bad)))
    return bad.value


def ax_dbg_use_graphs(model: int, enable: bool):
    _check(lib.ax_dbg_use_graphs(model, int(enable)))


def ax_dbg_profile(model: int, enable: bool):
    _check(lib.ax_dbg_profile(model, int(enable)))


def ax_dbg_profile_read(model: int) -> dict:
    ms = (C.c_double * len(PROFILE_CLASSES))()
    n = (C.c_int64 * len(PROFILE_CLASSES))()
    _check(lib.ax_dbg_profile_read(model, ms, n))
    return {name: (ms[i], n[i]) for i, name in enumerate(PROFILE_CLASSES)}


# ------------------------------------------------------------------ device memory through PyTorch

class DeviceModel:
    """Owns the torch tensors a model borrows (weights, workspace, KV pool) and the handles.

    weights: the dict produced by inputs.make_weights (numpy, storage format) or a dict of
    torch device tensors of the right dtype.  PyTorch is used for allocation and the stream only.
    """

    def __init__(self, shape, weights: dict, max_pos: int, max_tokens: int, pool_tokens: int,
                 max_seqs: int = 1, device: str = "cuda:0", pool_fill=None, act_split: int = 0):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the extend / verify path has no CPU fallback")
        self.torch, self.shape, self.device = torch, shape, torch.device(device)
        tdt = torch.float32 if shape.dtype == "f32" else torch.bfloat16

        def up(a):
            if isinstance(a, torch.Tensor):
                assert a.dtype == tdt and a.is_cuda and a.is_contiguous()
                return a
            t = torch.from_numpy(np.ascontiguousarray(a))
            if a.dtype == np.uint16:
                t = t.view(torch.bfloat16)
            return t.to(self.device)

        self.w = {k: ([up(a) for a in v] if isinstance(v, list) else up(v)) for k, v in weights.items()}
        self.cfg = make_config(shape, max_pos, max_tokens, max_seqs, act_split)
        ws_bytes = ax_workspace_bytes(self.cfg)
        if ws_bytes == 0:
            raise AxError(AX_ERR_UNSUPPORTED)
        self.ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=self.device)
        ptrs = {k: ([t.data_ptr() for t in v] if isinstance(v, list) else v.data_ptr()) for k, v in self.w.items()}
        self.model = ax_model_create(self.cfg, ptrs, self.ws.data_ptr(), ws_bytes)
        bb = ax_pool_block_bytes(self.cfg)
        n_blocks = -(-pool_tokens // 16)
        # pool_fill: byte the pool memory starts out with (tests use 0xFF: every slot a NaN)
        self.pool_mem = torch.full((n_blocks * bb,), pool_fill or 0, dtype=torch.uint8, device=self.device)
        self.pool = ax_pool_create(self.cfg, self.pool_mem.data_ptr(), n_blocks * bb)

    @property
    def stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def new_kv(self) -> int:
        return ax_kv_alloc(self.pool)

    def extend(self, kv: int, tokens, out_mode: int = AX_OUT_NONE):
        """Runs ax_extend on the current stream; returns a device tensor (or None)."""
        torch = self.torch
        n = len(tokens)
        out = None
        if out_mode == AX_OUT_LAST_LOGITS:
            out = torch.empty((1, self.shape.vocab), dtype=torch.float32, device=self.device)
        elif out_mode == AX_OUT_ALL_LOGITS:
            out = torch.empty((n, self.shape.vocab), dtype=torch.float32, device=self.device)
        elif out_mode == AX_OUT_LAST_ARGMAX:
            out = torch.empty(1, dtype=torch.int32, device=self.device)
        elif out_mode == AX_OUT_ALL_ARGMAX:
            out = torch.empty(n, dtype=torch.int32, device=self.device)
        ax_extend(self.model, kv, tokens, out_mode, out.data_ptr() if out is not None else 0, self.stream)
        return out

    def extend_batch(self, kvs, token_lists, out_mode: int = AX_OUT_NONE):
        torch = self.torch
        T_each = [len(t) for t in token_lists]
        rows = {AX_OUT_NONE: 0, AX_OUT_LAST_LOGITS: len(kvs), AX_OUT_LAST_ARGMAX: len(kvs)}.get(out_mode, sum(T_each))
        out = None
        if out_mode in (AX_OUT_LAST_LOGITS, AX_OUT_ALL_LOGITS):
            out = torch.empty((rows, self.shape.vocab), dtype=torch.float32, device=self.device)
        elif out_mode != AX_OUT_NONE:
            out = torch.empty(rows, dtype=torch.int32, device=self.device)
        ax_extend_batch(self.model, list(kvs), np.concatenate([np.asarray(t, dtype=np.int32) for t in token_lists]),
                        T_each, out_mode, out.data_ptr() if out is not None else 0, self.stream)
        return out

    def verify(self, kv: int, pending: int, drafts):
        return ax_verify(self.model, kv, pending, drafts, self.stream)

    def export_kv(self, kv: int, n_tokens: int = -1, device: bool = False):
        """Image of the first n_tokens of kv as a uint8 tensor (pinned host memory, or device)."""
        import torch
        n = ax_kv_len(kv) if n_tokens < 0 else n_tokens
        nbytes = ax_kv_image_bytes(self.pool, n)
        img = (torch.empty(nbytes, dtype=torch.uint8, device="cuda") if device
               else torch.empty(nbytes, dtype=torch.uint8, pin_memory=True))
        ax_kv_export(self.model, kv, n_tokens, img.data_ptr(), nbytes, self.stream)
        return img

    def import_kv(self, image) -> int:
        return ax_kv_import(self.model, self.pool, image.data_ptr(), image.numel(), self.stream)

    def verify_batch(self, kvs, pending, drafts_each):
        return ax_verify_batch(self.model, list(kvs), pending, drafts_each, self.stream)

    def close(self):
        if self.model:
            self.torch.cuda.synchronize(self.device)
            bad = ax_dbg_check_guards(self.model)         # no kernel of this model's calls wrote past a workspace region
            ax_model_destroy(self.model)
            self.model = 0
            if bad >= 0:
                raise AssertionError(f"workspace region {bad} ({WORKSPACE_REGIONS[bad]}) was overrun")
