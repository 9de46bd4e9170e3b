"""Plain float64 CPU oracle: decoder forward over a contiguous KV cache, greedy decoding and
greedy draft verification.  TEST INFRASTRUCTURE ONLY - never imported by the product path.

What it follows
---------------
* Prefix caching (paper Sec. 2.3, "Prefix caching"): every token attends only to earlier
  tokens, so the K/V rows of a shared prefix can be reused and only the new tokens are run.
  Here that is simply `forward` called with a cache that already holds the prefix.
* Speculative decoding, verification phase (Sec. 2.3, "Speculative decoding"; Fig. 4): the
  target model is given the most recent token followed by the N drafts; the first mismatching
  draft and everything after it are dropped; the target's own token at that point starts the
  next round.  Here: `verify`.  With a lookup-table drafter (Sec. 4.3) there are no draft
  logits, so acceptance is exact match against the target's greedy token.
* Tail cut (Sec. 4.2, cluster ordering: a stored "1-3-2" cache serves "1-3" once the
  mismatched tail is removed): `KVCache.truncate`.

The paper names its models (Sec. 5.1) but never writes the decoder out; the block below is
the usual pre-norm decoder with grouped-query attention, rotary positions (half-split pairing,
base 10000), SwiGLU MLP and RMSNorm, without biases.  Everything is float64: weights are
widened exactly from their storage format and no step is blocked, fused or reordered.

Weight layout: every matrix is row-major [out_features, in_features] and is applied as
y = x @ W.T; `wqkv` stacks the query heads, then the key heads, then the value heads.
"""
from __future__ import annotations

import numpy as np


_WIDE = {}                      # id(array) -> (array, float64 copy); see widen()
_WIDE_BYTES = [0]
WIDE_CACHE_LIMIT = 24 << 30     # bytes of float64 copies kept; beyond it tensors are widened per use


def _to_f64(t: np.ndarray) -> np.ndarray:
    if t.dtype == np.uint16:
        return (t.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return t.astype(np.float64)


def widen(t: np.ndarray) -> np.ndarray:
    """Storage format -> float64, exactly.  uint16 arrays are bfloat16 bit patterns.

    Whole weight tensors (base arrays) are memoised so that repeated forwards do not convert
    gigabytes again; the cache holds the source array too, so an id is never reused.
    """
    hit = _WIDE.get(id(t))
    if hit is not None and hit[0] is t:
        return hit[1]
    out = _to_f64(t)
    if t.ndim == 2 and _WIDE_BYTES[0] + out.nbytes <= WIDE_CACHE_LIMIT:
        _WIDE[id(t)] = (t, out)
        _WIDE_BYTES[0] += out.nbytes
    return out


def clear_widen_cache() -> None:
    _WIDE.clear()
    _WIDE_BYTES[0] = 0


class KVCache:
    """Contiguous per-layer K and V, float64, [position, kv_head, head_dim]; grows on append."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int):
        self.K = [np.zeros((0, n_kv_heads, head_dim)) for _ in range(n_layers)]
        self.V = [np.zeros((0, n_kv_heads, head_dim)) for _ in range(n_layers)]

    def __len__(self) -> int:
        return self.K[0].shape[0]

    def append(self, layer: int, k: np.ndarray, v: np.ndarray) -> None:
        self.K[layer] = np.concatenate([self.K[layer], k], axis=0)
        self.V[layer] = np.concatenate([self.V[layer], v], axis=0)

    def truncate(self, new_len: int) -> None:
        """Drop every position >= new_len (rejected drafts, or a mismatched cached tail)."""
        assert 0 <= new_len <= len(self)
        self.K = [a[:new_len] for a in self.K]
        self.V = [a[:new_len] for a in self.V]

    def fork(self, n_tokens: int = -1) -> "KVCache":
        """Independent copy of the first n_tokens positions (a shared prefix, by value)."""
        n = len(self) if n_tokens < 0 else n_tokens
        assert n <= len(self)
        out = KVCache(len(self.K), self.K[0].shape[1], self.K[0].shape[2])
        out.K = [a[:n].copy() for a in self.K]
        out.V = [a[:n].copy() for a in self.V]
        return out


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x_i / sqrt(mean_j x_j^2 + eps) * g_i along the last axis."""
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding of x[t, head, hd] at absolute positions pos[t].

    Pair (j, j + hd/2) is rotated by the angle pos * base^(-2j/hd).
    """
    hd = x.shape[-1]
    half = hd // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = pos.astype(np.float64)[:, None, None] * theta[None, None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, pos: np.ndarray) -> np.ndarray:
    """Causal grouped-query attention.

    q[t, Hq, hd] are the new rows at absolute positions pos[t]; K, V[n, Hkv, hd] hold every
    position 0..n-1 (the new rows included).  Row t sees key j iff j <= pos[t].  Query head h
    reads KV head h // (Hq / Hkv).  Returns [t, Hq, hd].
    """
    T, Hq, hd = q.shape
    n, Hkv, _ = K.shape
    group = Hq // Hkv
    visible = np.arange(n)[None, :] <= pos[:, None]
    out = np.empty_like(q)
    for h in range(Hq):
        hk = h // group
        s = q[:, h, :] @ K[:, hk, :].T / np.sqrt(hd)
        s = np.where(visible, s, -np.inf)
        out[:, h, :] = softmax_rows(s) @ V[:, hk, :]
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def forward(shape, weights: dict, tokens, kv: KVCache, trace: dict = None, rows=None) -> np.ndarray:
    """Run `tokens` on top of the cache (length P before, P + T after); logits [T, vocab].

    `shape` needs n_layers, n_q_heads, n_kv_heads, head_dim, rms_eps, rope_base; `weights`
    is {"tok_emb", "lm_head", "final_norm", and per-layer lists "wqkv", "wo", "w_gate",
    "w_up", "w_down", "norm_attn", "norm_mlp"} in storage format.  If `trace` is a dict it
    receives the last layer's intermediates (for tests that localise a mismatch).  `rows`
    (indices into the T new rows) limits the LM head to those rows, e.g. [-1] for a prefill
    that only needs the first output token.
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    T = tokens.shape[0]
    Hq, Hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    pos = len(kv) + np.arange(T)

    x = _to_f64(weights["tok_emb"][tokens])
    for l in range(shape.n_layers):
        h = rmsnorm(x, widen(weights["norm_attn"][l]), shape.rms_eps)
        qkv = h @ widen(weights["wqkv"][l]).T
        q = qkv[:, :Hq * hd].reshape(T, Hq, hd)
        k = qkv[:, Hq * hd:(Hq + Hkv) * hd].reshape(T, Hkv, hd)
        v = qkv[:, (Hq + Hkv) * hd:].reshape(T, Hkv, hd)
        q = rope(q, pos, shape.rope_base)
        k = rope(k, pos, shape.rope_base)
        kv.append(l, k, v)
        o = attention(q, kv.K[l], kv.V[l], pos)
        x = x + o.reshape(T, Hq * hd) @ widen(weights["wo"][l]).T
        h2 = rmsnorm(x, widen(weights["norm_mlp"][l]), shape.rms_eps)
        act = silu(h2 @ widen(weights["w_gate"][l]).T) * (h2 @ widen(weights["w_up"][l]).T)
        x = x + act @ widen(weights["w_down"][l]).T
        if trace is not None:
            trace.update(qkv=qkv, q=q, attn=o, ffn=act)
    h_out = rmsnorm(x, widen(weights["final_norm"]), shape.rms_eps)
    if trace is not None:
        trace.update(x=x, h_out=h_out)
    if rows is not None:
        h_out = h_out[np.asarray(rows)]
    return h_out @ widen(weights["lm_head"]).T


def argmax_lowest(row: np.ndarray) -> int:
    """Index of the maximum; the lowest index among exact ties."""
    return int(np.argmax(row))


def greedy_decode(shape, weights, kv: KVCache, pending: int, n: int) -> list:
    """Plain autoregressive greedy decoding: n tokens, one forward per token."""
    out = []
    for _ in range(n):
        pending = argmax_lowest(forward(shape, weights, [pending], kv)[0])
        out.append(pending)
    return out


def accept_length(greedy_tokens, drafts) -> int:
    """Largest a such that drafts[i] == greedy_tokens[i] for every i < a.

    greedy_tokens[i] is the target's greedy token after row i of the verify input, i.e.
    its prediction for the slot that drafts[i] occupies.
    """
    a = 0
    while a < len(drafts) and int(drafts[a]) == int(greedy_tokens[a]):
        a += 1
    return a


def verify_from_logits(logits: np.ndarray, drafts):
    """Greedy verification given the [1 + k, vocab] logits of [pending, drafts]."""
    g = [argmax_lowest(r) for r in logits]
    a = accept_length(g, drafts)
    return a, g[a], g


def verify(shape, weights, kv: KVCache, pending: int, drafts):
    """One speculative round.

    The cache holds everything before `pending` (length P).  The rows [pending, d_1..d_k]
    are run in one forward; a drafts are accepted; the cache is cut back to P + 1 + a
    (prefix, pending, accepted drafts).  Returns (a, next_pending, logits); the round emits
    d_1..d_a followed by next_pending, which is not yet in the cache.
    """
    P = len(kv)
    drafts = [int(d) for d in drafts]
    logits = forward(shape, weights, [int(pending)] + drafts, kv)
    a, nxt, _ = verify_from_logits(logits, drafts)
    kv.truncate(P + 1 + a)
    return a, nxt, logits


def top2_margin(row: np.ndarray) -> float:
    """Gap between the largest and second-largest logit of a row."""
    part = np.partition(row, -2)
    return float(part[-1] - part[-2])


def kv_bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int, itemsize: int) -> int:
    """K and V, every layer, one position."""
    return 2 * n_layers * n_kv_heads * head_dim * itemsize
