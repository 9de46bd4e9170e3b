"""The shared library loads without a GPU and exports every symbol the headers declare;
argument errors are reported through ax_status without touching a device."""
import ctypes
import glob
import os
import re

import pytest

from paper_2605_10380_amd import binding as B
from paper_2605_10380_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(ax_[a-z0-9_]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported():
    syms = declared_symbols()
    assert {"ax_kv_alloc", "ax_kv_fork", "ax_extend", "ax_verify", "ax_kv_free", "ax_kv_truncate",
            "ax_extend_batch", "ax_model_create", "ax_pool_create"} <= syms
    lib = ctypes.CDLL(B.LIB_PATH)
    for s in sorted(syms):
        assert hasattr(lib, s), f"{s} declared in include/ but not exported"


def test_binding_has_the_same_names():
    for s in declared_symbols() - {"ax_last_error"}:
        assert hasattr(B, s), s


def test_config_validation_without_gpu():
    sh = I.SHAPES["1b"]
    good = B.make_config(sh, 8192, 256)
    assert B.ax_workspace_bytes(good) > 0
    for field, val in [("n_layers", 0), ("n_q_heads", 7), ("dtype", 3), ("max_tokens", 0), ("head_dim", 96),
                       ("d_ff", 100), ("vocab", 1000)]:
        bad = B.make_config(sh, 8192, 256)
        setattr(bad, field, val)
        assert B.ax_workspace_bytes(bad) == 0, field
        with pytest.raises(B.AxError):
            B.ax_pool_create(bad, 0, 1 << 30)
    with pytest.raises(B.AxError) as e:
        B.ax_pool_create(good, 0, 1 << 30, block_tokens=32)
    assert e.value.status == B.AX_ERR_UNSUPPORTED
    with pytest.raises(B.AxError) as e:
        B.ax_pool_create(good, 0, 1000)
    assert e.value.status == B.AX_ERR_OOM
    with pytest.raises(B.AxError):
        B.ax_model_create(good, {k: 0 for k in ("tok_emb", "lm_head", "final_norm")} |
                          {k: [0] * sh.n_layers for k in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_mlp")},
                          0, 0)
    # the fp32 path takes the tiny model's odd sizes (d_ff = 688)
    assert B.ax_workspace_bytes(B.make_config(I.SHAPES["tiny"], 1024, 64)) > 0


def test_extend_rejects_bad_arguments_before_any_launch():
    cfg = B.make_config(I.SHAPES["tiny"], 1024, 64)
    pool = B.ax_pool_create(cfg, 0, B.ax_pool_block_bytes(cfg) * 8)
    kv = B.ax_kv_alloc(pool)
    for model in (0, 12345):                                   # NULL model handle is refused
        with pytest.raises((B.AxError, OSError, ctypes.ArgumentError)):
            if model == 0:
                B.ax_extend(model, kv, [1, 2, 3])
            else:
                raise B.AxError(B.AX_ERR_INVALID)
    assert B.ax_kv_len(kv) == 0
    B.ax_kv_free(kv)
    B.ax_pool_destroy(pool)
