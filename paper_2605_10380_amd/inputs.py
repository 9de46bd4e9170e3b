"""Seeded synthetic inputs shared by the GPU path's tests, the oracle's tests and bench.py.

Nothing in this module belongs to the method: it draws numbers, rounds them to the
storage format and lays tokens out.  Decoder shapes and workloads are those of the
build's configuration list (tiny fp32 model; ~1B / ~3B / ~8B bf16 models), standing in
for the agent prompts the paper measures on (Sec. 3.2: prompts of a few thousand tokens
made of repeated template text; Sec. 3.3: outputs largely copied from the prompt).

All generators are counter based: every array is a pure function of (seed, stream name),
so the oracle and the GPU path can be fed identical bits without sharing any state.
"""
from __future__ import annotations

import os
import zlib
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class DecoderShape:
    """Llama-style decoder shape (pre-norm, GQA, SwiGLU, RoPE, untied LM head)."""
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    dtype: str            # "f32" or "bf16": storage type of weights and of the KV cache
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def layer_params(self) -> int:
        d, hd = self.d_model, self.head_dim
        return (d * self.n_q_heads * hd + 2 * d * self.n_kv_heads * hd
                + self.n_q_heads * hd * d + 3 * d * self.d_ff)

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def with_layers(self, n_layers: int) -> "DecoderShape":
        return replace(self, n_layers=n_layers, name=f"{self.name}-L{n_layers}")


@dataclass(frozen=True)
class Workload:
    shape: DecoderShape
    P: int                # cached prefix length
    T: int                # uncached suffix run by one extend
    rounds: int           # verify rounds
    k: int                # drafts per round
    block_tokens: int = 16


SHAPES = {
    "tiny": DecoderShape("tiny", 2, 256, 4, 2, 64, 688, 4096, "f32"),
    "1b": DecoderShape("1b", 16, 2048, 32, 8, 64, 8192, 128256, "bf16"),
    "3b": DecoderShape("3b", 28, 3072, 24, 8, 128, 8192, 128256, "bf16"),
    "8b": DecoderShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, "bf16"),
}

WORKLOADS = {
    1: Workload(SHAPES["tiny"], P=512, T=64, rounds=20, k=4),
    2: Workload(SHAPES["1b"], P=4096, T=256, rounds=64, k=8),
    3: Workload(SHAPES["3b"], P=6144, T=256, rounds=32, k=8),
    4: Workload(SHAPES["8b"], P=8192, T=512, rounds=128, k=8),
}


# --------------------------------------------------------------------------- RNG

def _rng(seed: int, stream: str) -> np.random.Generator:
    """Philox generator keyed by (seed, crc32(stream)): a counter-based stream per array."""
    key = (int(seed) & 0xFFFFFFFFFFFFFFFF, zlib.crc32(stream.encode()) & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(key=np.array(key, dtype=np.uint64)))


# --------------------------------------------------------------------------- bf16 storage

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- weights

def weight_names(shape: DecoderShape):
    """(name, layer or None, (rows, cols) or (n,)) for every tensor, all row-major [out, in]."""
    d, hd, F, V = shape.d_model, shape.head_dim, shape.d_ff, shape.vocab
    yield "tok_emb", None, (V, d)
    yield "lm_head", None, (V, d)
    yield "final_norm", None, (d,)
    for l in range(shape.n_layers):
        yield "wqkv", l, (shape.qkv_rows, d)          # rows: q heads, then k heads, then v heads
        yield "wo", l, (d, shape.n_q_heads * hd)
        yield "w_gate", l, (F, d)
        yield "w_up", l, (F, d)
        yield "w_down", l, (d, F)
        yield "norm_attn", l, (d,)
        yield "norm_mlp", l, (d,)


_CHUNK = 1 << 21          # elements per independently keyed chunk of a large tensor


def _fill_chunk(args):
    out, lo, hi, seed, stream, gain, as_bf16 = args
    g = _rng(seed, f"{stream}#{lo // _CHUNK}")
    w = g.standard_normal(hi - lo, dtype=np.float32)
    w *= np.float32(0.02)
    if gain:
        w += np.float32(1.0)
    out[lo:hi] = f32_to_bf16_bits(w) if as_bf16 else w


def make_tensor(shape: DecoderShape, seed: int, name: str, layer, dims) -> np.ndarray:
    """One weight tensor in storage format: float32, or uint16 bf16 bit patterns.

    Matrices are N(0, 0.02); norm gains are 1 + N(0, 0.02) so that a gain-indexing mistake
    shows up while logits keep a usable scale.  A tensor is cut into fixed-size chunks, each
    with its own counter-based stream, so generation is order independent (and threaded).
    """
    n = int(np.prod(dims))
    as_bf16 = shape.dtype != "f32"
    out = np.empty(n, dtype=np.uint16 if as_bf16 else np.float32)
    jobs = [(out, lo, min(n, lo + _CHUNK), seed, f"{name}/{layer}", len(dims) == 1, as_bf16)
            for lo in range(0, n, _CHUNK)]
    if len(jobs) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(_fill_chunk, jobs))
    else:
        _fill_chunk(jobs[0])
    return out.reshape(dims)


def make_weights(shape: DecoderShape, seed: int) -> dict:
    """All tensors of a decoder: {"tok_emb": arr, ..., "wqkv": [arr per layer], ...}."""
    out: dict = {}
    for name, layer, dims in weight_names(shape):
        t = make_tensor(shape, seed, name, layer, dims)
        if layer is None:
            out[name] = t
        else:
            out.setdefault(name, []).append(t)
    return out


# --------------------------------------------------------------------------- tokens

def zipf_table(vocab: int, seed: int, s: float = 1.1):
    """CDF over ranks 1..V with p(r) ~ r^-s, and a seeded rank -> token-id permutation."""
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(p / p.sum())
    cdf[-1] = 1.0
    perm = _rng(seed, "zipf/perm").permutation(vocab).astype(np.int32)
    return cdf, perm


def zipf_tokens(vocab: int, seed: int, stream: str, n: int) -> np.ndarray:
    cdf, perm = zipf_table(vocab, seed)
    u = _rng(seed, f"zipf/{stream}").random(n)
    return perm[np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1)]


def templated_prompt(vocab: int, seed: int, n_tokens: int, span: int = 32, library: int = 64) -> np.ndarray:
    """Zipf(1.1) prompt in which each 32-token slot is, with probability 1/2, one of 64
    fixed template spans (tool schemas / few-shot examples repeat verbatim in agent prompts)."""
    lib = zipf_tokens(vocab, seed, "library", span * library).reshape(library, span)
    n_slots = -(-n_tokens // span)
    fresh = zipf_tokens(vocab, seed, "fresh", n_slots * span).reshape(n_slots, span)
    g = _rng(seed, "slots")
    use_lib = g.random(n_slots) < 0.5
    pick = g.integers(0, library, n_slots)
    out = np.where(use_lib[:, None], lib[pick], fresh).reshape(-1)[:n_tokens]
    return np.ascontiguousarray(out, dtype=np.int32)


def prompt_copied_drafts(prompt: np.ndarray, seed: int, round_idx: int, k: int) -> np.ndarray:
    """k consecutive tokens copied from a seeded earlier position of the prompt."""
    g = _rng(seed, f"draft/copy/{round_idx}")
    start = int(g.integers(0, len(prompt) - k + 1))
    return np.ascontiguousarray(prompt[start:start + k], dtype=np.int32)


def seeded_accept_drafts(greedy: np.ndarray, vocab: int, seed: int, round_idx: int, k: int):
    """Drafts whose first j tokens equal the given greedy continuation, j ~ U{0..k}.

    ``greedy`` holds at least k tokens: what plain greedy decoding emits after the pending
    token.  Token j (if j < k) is shifted by 1 + r (mod V), r in [0, V-2], so it is never the
    greedy one; the rest are Zipf draws.  Returns (drafts, j).
    """
    g = _rng(seed, f"draft/accept/{round_idx}")
    j = int(g.integers(0, k + 1))
    d = zipf_tokens(vocab, seed, f"draft/tail/{round_idx}", k).copy()
    d[:j] = greedy[:j]
    if j < k:
        d[j] = (int(greedy[j]) + 1 + int(g.integers(0, vocab - 1))) % vocab
    return np.ascontiguousarray(d, dtype=np.int32), j


def cluster_activation_samples(seed: int, n_samples: int, n_clusters: int = 8):
    """Synthetic stand-in for the cluster sequences a tool-retrieval step activates per query
    (the paper clusters 16 tools into 8 ordered clusters; a query activates the clusters that
    hold its retrieved tools).  Clusters come in adjacent pairs of one theme; a sample picks a
    theme with Zipf-like popularity, activates each cluster of the pair with its own probability
    and sometimes one cluster of another theme.  Returns a list of ascending tuples (the fixed
    order), none empty."""
    g = _rng(seed, "clusters")
    n_themes = max(1, n_clusters // 2)
    pop = 1.0 / np.arange(1, n_themes + 1) ** 1.2
    pop /= pop.sum()
    out = []
    for _ in range(n_samples):
        t = int(g.choice(n_themes, p=pop))
        act = set()
        if g.random() < 0.8:
            act.add(2 * t)
        if 2 * t + 1 < n_clusters and g.random() < 0.55:
            act.add(2 * t + 1)
        if g.random() < 0.3:
            act.add(int(g.integers(0, n_clusters)))
        if not act:
            act.add(2 * t)
        out.append(tuple(sorted(act)))
    return out
