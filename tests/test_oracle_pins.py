"""Pins for the CPU oracle: brute force, closed forms, invariants the paper states, the paper's
worked example and an independent library implementation.  None of these touch the GPU path."""
import cmath
import math
import os

import numpy as np
import pytest

from oracle import decoder as O
from paper_2605_10380_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_shape(**kw):
    base = dict(name="pin", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16,
                d_ff=96, vocab=97, dtype="f32")
    base.update(kw)
    return I.DecoderShape(**base)


def new_kv(sh):
    return O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)


# ------------------------------------------------------------------ attention: brute force

def brute_attention(q, K, V, pos):
    """Definition, scalar by scalar: o = sum_j softmax_j(q.k_j / sqrt(hd)) v_j over j <= pos."""
    T, Hq, hd = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.zeros_like(q)
    for t in range(T):
        for h in range(Hq):
            hk = h // G
            scores = []
            for j in range(int(pos[t]) + 1):
                scores.append(sum(q[t, h, c] * K[j, hk, c] for c in range(hd)) / math.sqrt(hd))
            m = max(scores)
            e = [math.exp(s - m) for s in scores]
            z = sum(e)
            for c in range(hd):
                out[t, h, c] = sum(e[j] / z * V[j, hk, c] for j in range(len(e)))
    return out


@pytest.mark.parametrize("P", [0, 1, 17, 33])
@pytest.mark.parametrize("T", [1, 5])
@pytest.mark.parametrize("G", [1, 2, 3, 4])
def test_attention_matches_brute_force(P, T, G):
    rng = np.random.default_rng(100 * P + 10 * T + G)
    Hkv, hd = 2, 8
    q = rng.standard_normal((T, Hkv * G, hd))
    K = rng.standard_normal((P + T, Hkv, hd))
    V = rng.standard_normal((P + T, Hkv, hd))
    pos = P + np.arange(T)
    np.testing.assert_allclose(O.attention(q, K, V, pos), brute_attention(q, K, V, pos),
                               rtol=0, atol=1e-13)


def test_attention_special_cases():
    rng = np.random.default_rng(7)
    q = rng.standard_normal((1, 4, 8))
    V = rng.standard_normal((6, 2, 8))
    K = rng.standard_normal((6, 2, 8))
    # one visible key: the output is that key's value row, whatever the score is
    o = O.attention(q, K[:1], V[:1], np.array([0]))
    for h in range(4):
        np.testing.assert_allclose(o[0, h], V[0, h // 2], atol=1e-15)
    # all keys equal: uniform weights, output is the mean of the visible values
    Ke = np.repeat(K[:1], 6, axis=0)
    o = O.attention(q, Ke, V, np.array([5]))
    np.testing.assert_allclose(o[0, 3], V[:, 1].mean(axis=0), atol=1e-14)
    o = O.attention(q, Ke, V, np.array([2]))          # causal: only positions 0..2
    np.testing.assert_allclose(o[0, 0], V[:3, 0].mean(axis=0), atol=1e-14)
    # softmax is shift invariant: adding c*q-direction to every key adds a constant score
    shift = 3.0 * q[0, 1] / np.dot(q[0, 1], q[0, 1])
    K2 = K.copy()
    K2[:, 0, :] += shift
    o1 = O.attention(q, K, V, np.array([5]))
    o2 = O.attention(q, K2, V, np.array([5]))
    np.testing.assert_allclose(o1[0, 1], o2[0, 1], atol=1e-13)
    # rows are independent of which other rows are in the call
    q3 = rng.standard_normal((3, 4, 8))
    pos = np.array([3, 4, 5])
    full = O.attention(q3, K, V, pos)
    one = O.attention(q3[1:2], K, V, pos[1:2])
    np.testing.assert_allclose(full[1], one[0], atol=1e-15)


# ------------------------------------------------------------------ RoPE

def test_rope_position_zero_is_identity_and_norms_kept():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 3, 16))
    np.testing.assert_array_equal(O.rope(x[:1], np.array([0]), 10000.0), x[:1])
    y = O.rope(x, np.array([5, 77, 1234, 8191]), 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-14)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((1, 1, 32))
    k = rng.standard_normal((1, 1, 32))
    def score(m, n):
        return float(np.sum(O.rope(q, np.array([m]), 10000.0) * O.rope(k, np.array([n]), 10000.0)))
    assert abs(score(9, 4) - score(1009, 1004)) < 1e-10
    assert abs(score(9, 4) - score(5, 0)) < 1e-12
    assert abs(score(9, 4) - score(4, 9)) > 1e-3      # direction matters


def test_rope_equals_complex_rotation():
    """Pair (j, j+hd/2) read as the complex number x_j + i x_{j+hd/2} is multiplied by
    exp(i * pos * base^(-2j/hd))."""
    rng = np.random.default_rng(5)
    hd, base = 16, 10000.0
    x = rng.standard_normal((3, 2, hd))
    pos = np.array([1, 50, 4097])
    y = O.rope(x, pos, base)
    for t in range(3):
        for h in range(2):
            for j in range(hd // 2):
                z = complex(x[t, h, j], x[t, h, j + hd // 2]) * cmath.exp(1j * pos[t] * base ** (-2.0 * j / hd))
                assert abs(y[t, h, j] - z.real) < 1e-12 and abs(y[t, h, j + hd // 2] - z.imag) < 1e-12


# ------------------------------------------------------------------ RMSNorm, SiLU

def test_rmsnorm_unit_rms_and_scale_invariance():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 64)) * 3.0
    y = O.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, rtol=1e-14)
    np.testing.assert_allclose(O.rmsnorm(7.5 * x, np.ones(64), 0.0), y, rtol=1e-13)
    g = rng.standard_normal(64)
    np.testing.assert_allclose(O.rmsnorm(x, g, 0.0), y * g, rtol=1e-14)
    # eps enters under the root: a zero row stays zero, a constant row c gives c/sqrt(c^2+eps)
    assert np.all(O.rmsnorm(np.zeros((1, 8)), np.ones(8), 1e-5) == 0.0)
    np.testing.assert_allclose(O.rmsnorm(np.full((1, 8), 2.0), np.ones(8), 0.5), 2.0 / math.sqrt(4.5))


def test_silu_values():
    np.testing.assert_allclose(O.silu(np.array([0.0, 1.0, -1.0, 20.0])),
                               [0.0, 1.0 / (1.0 + math.exp(-1.0)), -1.0 / (1.0 + math.e), 20.0 / (1 + math.exp(-20.0))],
                               rtol=1e-15)


# ------------------------------------------------------------------ whole forward

def test_closed_form_when_output_projections_are_zero():
    """With Wo = 0 and W_down = 0 every block is the identity, so logits depend on the token
    alone: rmsnorm(E[tok]) @ W_lm^T."""
    sh = small_shape()
    w = I.make_weights(sh, 11)
    w["wo"] = [np.zeros_like(a) for a in w["wo"]]
    w["w_down"] = [np.zeros_like(a) for a in w["w_down"]]
    toks = I.zipf_tokens(sh.vocab, 11, "t", 9)
    lg = O.forward(sh, w, toks, new_kv(sh))
    e = w["tok_emb"][toks].astype(np.float64)
    h = e / np.sqrt((e * e).mean(-1, keepdims=True) + sh.rms_eps) * w["final_norm"].astype(np.float64)
    np.testing.assert_allclose(lg, h @ w["lm_head"].astype(np.float64).T, atol=1e-14)


def torch_forward(sh, w, tokens):
    """Independent float64 implementation from a tensor library's stock primitives: no cache
    (full recomputation), explicit causal mask, rotary via complex multiplication."""
    import torch
    import torch.nn.functional as F
    f = lambda a: torch.from_numpy(O.widen(a))
    T = len(tokens)
    Hq, Hkv, hd = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    x = F.embedding(torch.from_numpy(np.asarray(tokens, dtype=np.int64)), f(w["tok_emb"]))
    pos = torch.arange(T, dtype=torch.float64)
    inv = sh.rope_base ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])
    def rotary(t):                                     # t [T, H, hd]
        z = torch.complex(t[..., :hd // 2], t[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)
    mask = torch.ones(T, T, dtype=torch.bool).tril()
    for l in range(sh.n_layers):
        h = F.rms_norm(x, (sh.d_model,), f(w["norm_attn"][l]), sh.rms_eps)
        qkv = F.linear(h, f(w["wqkv"][l]))
        q, k, v = torch.split(qkv, [Hq * hd, Hkv * hd, Hkv * hd], dim=-1)
        q = rotary(q.reshape(T, Hq, hd)).transpose(0, 1)
        k = rotary(k.reshape(T, Hkv, hd)).transpose(0, 1).repeat_interleave(Hq // Hkv, dim=0)
        v = v.reshape(T, Hkv, hd).transpose(0, 1).repeat_interleave(Hq // Hkv, dim=0)
        o = F.scaled_dot_product_attention(q, k, v, attn_mask=mask)
        x = x + F.linear(o.transpose(0, 1).reshape(T, Hq * hd), f(w["wo"][l]))
        h = F.rms_norm(x, (sh.d_model,), f(w["norm_mlp"][l]), sh.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, f(w["w_gate"][l]))) * F.linear(h, f(w["w_up"][l])), f(w["w_down"][l]))
    return F.linear(F.rms_norm(x, (sh.d_model,), f(w["final_norm"]), sh.rms_eps), f(w["lm_head"])).numpy()


@pytest.mark.parametrize("which", ["pin-f32", "pin-bf16-g3", "tiny"])
def test_forward_matches_tensor_library(which):
    if which == "tiny":
        sh, n = I.SHAPES["tiny"], 96
    elif which == "pin-f32":
        sh, n = small_shape(), 37
    else:
        sh, n = small_shape(n_q_heads=6, n_kv_heads=2, dtype="bf16", d_model=96), 37
    w = I.make_weights(sh, 21)
    toks = I.templated_prompt(sh.vocab, 21, n)
    kv = new_kv(sh)
    a = O.forward(sh, w, toks[:n // 2], kv)
    b = O.forward(sh, w, toks[n // 2:], kv)           # second half as an extend over the cache
    ref = torch_forward(sh, w, toks)
    np.testing.assert_allclose(np.concatenate([a, b]), ref, rtol=0, atol=1e-11)


# ------------------------------------------------------------------ prefix reuse (Sec. 2.3)

def test_extend_over_cached_prefix_equals_full_recompute():
    sh = I.SHAPES["tiny"]
    w = I.make_weights(sh, 31)
    toks = I.templated_prompt(sh.vocab, 31, 200)
    full = O.forward(sh, w, toks, new_kv(sh))
    for chunks in ([150, 50], [1, 64, 17, 118], [16] * 12 + [8]):
        kv, outs, at = new_kv(sh), [], 0
        for c in chunks:
            outs.append(O.forward(sh, w, toks[at:at + c], kv))
            at += c
        assert len(kv) == 200
        np.testing.assert_allclose(np.concatenate(outs), full, rtol=0, atol=1e-12)


def test_reuse_stops_at_first_mismatch_and_order_matters():
    """One changed token changes the K/V of every later position even where the later tokens
    are identical, and swapping two spans ("A-B" vs "B-A") changes their cached values."""
    sh = small_shape()
    w = I.make_weights(sh, 32)
    toks = I.zipf_tokens(sh.vocab, 32, "p", 40)
    kv_a, kv_b = new_kv(sh), new_kv(sh)
    O.forward(sh, w, toks, kv_a)
    changed = toks.copy()
    changed[10] = (changed[10] + 1) % sh.vocab
    O.forward(sh, w, changed, kv_b)
    last = sh.n_layers - 1
    np.testing.assert_array_equal(kv_a.K[last][:10], kv_b.K[last][:10])
    assert np.abs(kv_a.K[last][11:] - kv_b.K[last][11:]).min(axis=(1, 2)).min() > 0
    swapped = np.concatenate([toks[20:], toks[:20]])
    kv_c = new_kv(sh)
    O.forward(sh, w, swapped, kv_c)
    assert np.abs(kv_c.V[last][:20] - kv_a.V[last][20:]).max() > 1e-6


def test_tail_cut_and_fork():
    """Cutting the tail of a longer cached sequence, or forking its first n positions, then
    extending equals never having had the tail (Sec. 4.2)."""
    sh = small_shape()
    w = I.make_weights(sh, 33)
    toks = I.zipf_tokens(sh.vocab, 33, "p", 60)
    kv = new_kv(sh)
    O.forward(sh, w, toks[:50], kv)
    fk = kv.fork(30)
    kv.truncate(30)
    other = I.zipf_tokens(sh.vocab, 33, "q", 12)
    a = O.forward(sh, w, other, kv)
    b = O.forward(sh, w, other, fk)
    fresh = new_kv(sh)
    O.forward(sh, w, toks[:30], fresh)
    c = O.forward(sh, w, other, fresh)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_allclose(a, c, rtol=0, atol=1e-12)


# ------------------------------------------------------------------ verification (Sec. 2.3)

def _parse_example():
    kv = {}
    for line in open(os.path.join(GOLDEN, "specdec_worked_example.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        key, val = line.split(":", 1)
        kv[key.strip()] = val.split()
    ids = {t.split("=")[0]: int(t.split("=")[1]) for t in kv["vocab"]}
    return kv, ids


def test_worked_example_from_the_paper():
    ex, ids = _parse_example()
    drafts = [ids[t] for t in ex["drafts"]]
    target = [ids[t] for t in ex["target_after"]]
    logits = np.full((1 + len(drafts), len(ids)), -1.0)
    for r, t in enumerate(target):
        logits[r, t] = 2.0
    a, nxt, g = O.verify_from_logits(logits, drafts)
    assert a == int(ex["accepted"][0]) and nxt == ids[ex["next"][0]]
    assert drafts[:a] + [nxt] == [ids[t] for t in ex["emitted"]]
    assert 1 + a == int(ex["kv_growth"][0])


def test_accept_length_cases():
    assert O.accept_length([5, 6, 7, 8, 9], [5, 6, 7, 8]) == 4      # all right: bonus is g[4]
    assert O.accept_length([5, 6, 7, 8, 9], [4, 6, 7, 8]) == 0      # first wrong
    assert O.accept_length([5, 6, 7, 8, 9], [5, 6, 0, 8]) == 2      # later matches do not count
    assert O.accept_length([5], []) == 0                            # k = 0: plain decode
    assert O.argmax_lowest(np.array([1.0, 3.0, 3.0, 2.0])) == 1     # ties: lowest id


def _spec_stream(sh, w, prompt, n_out, k, make_drafts):
    kv = new_kv(sh)
    lg = O.forward(sh, w, prompt, kv)
    pending = O.argmax_lowest(lg[-1])
    out, rounds, hist = [pending], 0, []
    while len(out) < n_out:
        P = len(kv)
        drafts = make_drafts(rounds, kv, pending)
        a, nxt, _ = O.verify(sh, w, kv, pending, drafts)
        assert len(kv) == P + 1 + a
        out += [int(d) for d in drafts[:a]] + [nxt]
        pending = nxt
        hist.append(a)
        rounds += 1
    return out[:n_out], hist


@pytest.mark.parametrize("mode", ["all_right", "all_wrong", "seeded", "prompt_copy", "k0"])
def test_speculative_stream_equals_greedy_stream(mode):
    """Accuracy preservation (Sec. 1, Sec. 2.3): whatever the drafts are, the emitted tokens are
    exactly those of one-token-at-a-time greedy decoding."""
    sh = small_shape(vocab=53)
    w = I.make_weights(sh, 41)
    prompt = I.templated_prompt(sh.vocab, 41, 48)
    n_out, k = 40, 4
    kv = new_kv(sh)
    first = O.argmax_lowest(O.forward(sh, w, prompt, kv)[-1])
    greedy = [first] + O.greedy_decode(sh, w, kv, first, n_out + k)

    def drafts_for(r, kv_now, pending):
        at = len(kv_now) - len(prompt) + 1              # index in `greedy` of the next token
        nxt = np.array(greedy[at:at + k])
        if mode == "all_right":
            return nxt
        if mode == "all_wrong":
            return (nxt + 1) % sh.vocab
        if mode == "seeded":
            return I.seeded_accept_drafts(nxt, sh.vocab, 41, r, k)[0]
        if mode == "k0":
            return np.zeros(0, dtype=np.int32)
        return I.prompt_copied_drafts(prompt, 41, r, k)

    out, hist = _spec_stream(sh, w, prompt, n_out, k, drafts_for)
    assert out == greedy[:n_out]
    if mode == "all_right":
        assert all(a == k for a in hist)
    if mode in ("all_wrong", "k0"):
        assert all(a == 0 for a in hist)
    if mode == "seeded":
        assert 0 < sum(hist) < k * len(hist)


def test_rollback_equals_never_appending():
    sh = small_shape()
    w = I.make_weights(sh, 42)
    prompt = I.zipf_tokens(sh.vocab, 42, "p", 20)
    kv = new_kv(sh)
    pending = O.argmax_lowest(O.forward(sh, w, prompt, kv)[-1])
    ref = kv.fork()
    a, nxt, _ = O.verify(sh, w, kv, pending, [(pending + 1) % sh.vocab] * 4)
    g = O.argmax_lowest(O.forward(sh, w, [pending], ref)[0])
    assert nxt == g and len(kv) == len(ref)
    for l in range(sh.n_layers):
        # equal up to the library matmul's grouping of rows (1 row here, 5 rows there)
        np.testing.assert_allclose(kv.K[l], ref.K[l], rtol=0, atol=1e-13)
        np.testing.assert_allclose(kv.V[l], ref.V[l], rtol=0, atol=1e-13)


# ------------------------------------------------------------------ numbers the paper prints

def test_kv_footprint_matches_the_papers_figures():
    vals = {}
    for line in open(os.path.join(GOLDEN, "kv_footprint.txt")):
        if not line.startswith("#") and ":" in line:
            k, v = line.split(":")
            vals[k.strip()] = float(v)
    bpt = O.kv_bytes_per_token(int(vals["layers"]), int(vals["kv_heads"]), int(vals["head_dim"]), int(vals["itemsize"]))
    assert bpt == int(vals["bytes_per_token"])
    assert round(vals["tokens_a"] * bpt / 2 ** 20) == vals["size_a_MB"]
    assert abs(vals["tokens_b"] * bpt / 2 ** 30 - vals["size_b_GB"]) < 0.1
    sh = I.SHAPES["8b"]
    assert O.kv_bytes_per_token(sh.n_layers, sh.n_kv_heads, sh.head_dim, sh.itemsize) == bpt


def test_draft_accuracy_matches_table3():
    """accuracy = accepted / generated drafts: the oracle's bookkeeping reproduces the paper's column."""
    from oracle import exspec as X
    rows = 0
    for line in open(os.path.join(GOLDEN, "draft_accuracy.txt")):
        if line.startswith("#"):
            continue
        *_, gen, acc, ratio = line.split()
        assert round(X.draft_accuracy(dict(drafted=int(gen), accepted=int(acc))), 2) == float(ratio)
        rows += 1
    assert rows == 4
    assert X.draft_accuracy(dict(drafted=0, accepted=0)) == 0.0


def test_top2_margin_hand_written_rows():
    """The function that decides which GPU / oracle disagreements are exempt: gap between the two
    largest entries, 0 on an exact tie for first place."""
    assert O.top2_margin(np.array([1.0, 3.0, 2.0])) == 1.0
    assert O.top2_margin(np.array([5.0, 5.0, 1.0])) == 0.0              # tie for first place
    assert O.top2_margin(np.array([-3.0, -1.0, -2.0])) == 1.0            # all negative
    assert O.top2_margin(np.array([9.0, 0.0, 0.0, 1.0])) == 8.0          # maximum first
    assert O.top2_margin(np.array([0.0, 1.0, 0.0, 9.0])) == 8.0          # maximum last
    assert O.top2_margin(np.array([2.0, 2.5])) == 0.5                    # two entries
    assert O.top2_margin(np.array([7.0, -7.0, 7.0, 7.0])) == 0.0
    assert abs(O.top2_margin(np.array([0.125, 0.120, -4.0])) - 0.005) < 1e-15
    # not the range, not the gap to the mean, not the signed gap in storage order
    row = np.array([4.0, 1.0, 3.5, -10.0])
    assert O.top2_margin(row) == 0.5 and O.top2_margin(row[::-1].copy()) == 0.5
    # brute force over random rows
    rng = np.random.default_rng(5)
    for _ in range(50):
        r = rng.standard_normal(int(rng.integers(2, 40)))
        s_ = sorted(r.tolist())
        assert O.top2_margin(r) == s_[-1] - s_[-2]


# ------------------------------------------------------------------ planted mistakes are caught

@pytest.mark.parametrize("mistake", ["gqa_map", "rope_sign", "scale", "causal_off_by_one", "transpose_wo"])
def test_pins_catch_planted_mistakes(mistake, monkeypatch):
    """Each planted mistake in the oracle must make the library-comparison pin fail."""
    sh = small_shape(n_q_heads=4, n_kv_heads=2)
    w = I.make_weights(sh, 51)
    if mistake == "transpose_wo":
        w2 = dict(w)
        w2["wo"] = [np.ascontiguousarray(a.T) for a in w["wo"]]       # square here: a silent transpose
        bad = O.forward(sh, w2, I.zipf_tokens(sh.vocab, 51, "p", 12), new_kv(sh))
    else:
        if mistake == "gqa_map":
            orig = O.attention
            def att(q, K, V, pos):
                return orig(q, K[:, ::-1], V[:, ::-1], pos)
            monkeypatch.setattr(O, "attention", att)
        elif mistake == "rope_sign":
            orig_r = O.rope
            monkeypatch.setattr(O, "rope", lambda x, pos, base: orig_r(x, -pos, base))
        elif mistake == "scale":
            orig = O.attention
            monkeypatch.setattr(O, "attention", lambda q, K, V, pos: orig(q * 2.0, K, V, pos))
        elif mistake == "causal_off_by_one":
            orig = O.attention
            monkeypatch.setattr(O, "attention", lambda q, K, V, pos: orig(q, K, V, np.maximum(pos - 1, 0)))
        bad = O.forward(sh, w, I.zipf_tokens(sh.vocab, 51, "p", 12), new_kv(sh))
    ref = torch_forward(sh, w, I.zipf_tokens(sh.vocab, 51, "p", 12))
    assert np.abs(bad - ref).max() > 1e-8


# ------------------------------------------------------------------ n-gram drafter (Sec. 4.3)

def _lut_example():
    ex = {"entry": []}
    for line in open(os.path.join(GOLDEN, "ngram_lut_example.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":")
        vals = [int(t) for t in v.split()]
        if k == "entry":
            ex["entry"].append(vals)
        else:
            ex[k] = vals
    return ex


def test_ngram_lut_matches_hand_worked_example():
    from oracle import exspec as X
    ex = _lut_example()
    lut = X.build_lut(ex["stream"], ex["n"][0])
    assert lut == {tuple(e[:-1]): e[-1] for e in ex["entry"]}
    d, hits = X.draft(lut, 3, ex["context"], 4, True, 100, 0, 0)
    assert d == ex["drafts"] and hits == 4
    assert X.draft(lut, 3, ex["miss_context"], 4, True, 100, 0, 0) == ([], 0)
    # non-selective: a miss still produces k (random) drafts; a later hit is used again
    d2, hits2 = X.draft(lut, 3, ex["miss_context"], 4, False, 100, 5, 0)
    assert len(d2) == 4 and hits2 <= 3 and d2[0] == X.splitmix64(5) % 100
    # too little context is a miss, n = 1 proposes the most frequent token of the stream
    assert X.draft(lut, 3, [7], 2, True, 100, 0, 0) == ([], 0)
    uni = X.build_lut(ex["stream"], 1)
    assert uni == {(): 3}
    assert X.splitmix64(0) == 0xE220A8397B1DCDAF          # published first output for seed 0


def _loop_example():
    ex = {}
    for line in open(os.path.join(GOLDEN, "exspec_loop_example.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":")
        ex[k.strip()] = [float(t) if "." in t else int(t) for t in v.split()]
    return ex


def successor_model(vocab=8):
    """A decoder whose greedy token after t is (t + 1) mod vocab whatever the context: identity
    embedding, zero attention-output and MLP-down projections, permutation LM head (the closed
    form logits = rmsnorm(E[t]) W_lm^T pinned above)."""
    sh = small_shape(d_model=vocab, n_q_heads=2, n_kv_heads=1, head_dim=vocab // 2, d_ff=16, vocab=vocab)
    w = I.make_weights(sh, 91)
    w["tok_emb"] = np.eye(vocab, dtype=np.float32)
    w["final_norm"] = np.ones(vocab, dtype=np.float32)
    lm = np.zeros((vocab, vocab), dtype=np.float32)
    for t in range(vocab):
        lm[(t + 1) % vocab, t] = 1.0
    w["lm_head"] = lm
    w["wo"] = [np.zeros_like(a) for a in w["wo"]]
    w["w_down"] = [np.zeros_like(a) for a in w["w_down"]]
    return sh, w


def test_exspec_loop_counters_match_hand_worked_run():
    """rounds / fallbacks / drafted / accepted of the decode loop, exactly, on a run worked by hand
    (tests/golden/exspec_loop_example.txt): partial acceptance, a first-lookup miss that falls
    back, a later miss that still drafts, and the cut of the last round's draft length."""
    from oracle import exspec as X
    ex = _loop_example()
    sh, w = successor_model(ex["vocab"][0])
    assert O.greedy_decode(sh, w, new_kv(sh), ex["pending"][0], 10) == ex["tokens"]
    lut = X.build_lut(ex["stream"], ex["n"][0])
    assert len(lut) == 9
    kv = new_kv(sh)
    O.forward(sh, w, ex["history"], kv)
    out, st = X.generate(sh, w, kv, lut, ex["n"][0], ex["history"], ex["pending"][0], ex["max_new"][0], ex["k"][0],
                         True, seed=1)
    assert out == ex["tokens"]
    assert st == dict(rounds=ex["rounds"][0], fallbacks=ex["fallbacks"][0], drafted=ex["drafted"][0],
                      accepted=ex["accepted"][0])
    assert X.draft_accuracy(st) == ex["accuracy"][0]
    assert len(kv) == len(ex["history"]) + ex["max_new"][0]      # everything but the last emitted token
    full = X.build_lut(ex["full_stream"], ex["n"][0])
    for selective in (True, False):
        kv = new_kv(sh)
        O.forward(sh, w, ex["history"], kv)
        out, st = X.generate(sh, w, kv, full, ex["n"][0], ex["history"], ex["pending"][0], ex["max_new"][0], ex["k"][0],
                             selective, seed=1)
        assert out == ex["tokens"]
        assert st == dict(rounds=ex["full_rounds"][0], fallbacks=ex["full_fallbacks"][0], drafted=ex["full_drafted"][0],
                          accepted=ex["full_accepted"][0])
    # non-selective, first table: round 2 drafts three guesses instead of falling back, so no round
    # falls back and 3 more drafts are generated (whether a guess happens to be right is up to the generator)
    kv = new_kv(sh)
    O.forward(sh, w, ex["history"], kv)
    out, st = X.generate(sh, w, kv, lut, ex["n"][0], ex["history"], ex["pending"][0], ex["max_new"][0], ex["k"][0],
                         False, seed=1)
    assert out == ex["tokens"] and st["fallbacks"] == 0 and st["drafted"] >= st["accepted"] >= 0


@pytest.mark.parametrize("selective", [True, False])
def test_exspec_stream_equals_greedy_and_counts_drafts(selective):
    """The decode loop emits exactly the greedy stream (accuracy preservation); a table built
    from the greedy continuation itself predicts most of it, a table built from unrelated text
    predicts nothing; accuracy = accepted / drafted."""
    from oracle import exspec as X
    sh = small_shape(vocab=61)
    w = I.make_weights(sh, 71)
    prompt = I.templated_prompt(sh.vocab, 71, 40)
    kv = new_kv(sh)
    first = O.argmax_lowest(O.forward(sh, w, prompt, kv)[-1])
    greedy = O.greedy_decode(sh, w, kv.fork(), first, 48)
    good = X.build_lut(list(prompt) + [first] + greedy, 3)
    out, st = X.generate(sh, w, kv.fork(), good, 3, prompt, first, 48, 4, selective, seed=9)
    assert out == greedy
    assert st["accepted"] > 0 and st["drafted"] >= st["accepted"] and st["rounds"] < 48
    bad = X.build_lut(I.zipf_tokens(sh.vocab, 72, "other", 30) + 0, 3)
    out2, st2 = X.generate(sh, w, kv.fork(), bad, 3, prompt, first, 20, 4, selective, seed=9)
    assert out2 == greedy[:20]
    if selective:
        assert st2["fallbacks"] >= 1
    else:
        assert st2["fallbacks"] <= 1 and st2["drafted"] > 0     # only the last round (0 drafts left) falls back


def test_bf16_bit_patterns_widen_to_their_hand_decoded_values():
    """bfloat16 = sign, 8 exponent bits (bias 127), 7 fraction bits, stored as uint16: a handful of patterns decoded
    by hand (normal, negative, the value nearest 0.1, the largest finite, the smallest subnormal, zero) must come out
    exactly; float32 storage is passed through unchanged.  The memo cache must not hand a tensor the copy of another."""
    bits = np.array([[0x3F80, 0xC000, 0x3DCD, 0x7F7F], [0x0001, 0x0000, 0x8000, 0x4049]], dtype=np.uint16)
    want = np.array([[1.0, -2.0, (1 + 77 / 128) * 2.0 ** -4, (2 - 2.0 ** -7) * 2.0 ** 127],
                     [2.0 ** -133, 0.0, -0.0, (1 + 73 / 128) * 2.0]])
    O.clear_widen_cache()
    got = O.widen(bits)
    assert got.dtype == np.float64 and np.array_equal(got, want)
    assert np.signbit(got[1, 2]) and not np.signbit(got[1, 1])
    assert O.widen(bits) is got                                   # memoised for whole 2-D tensors
    other = bits.copy()
    other[0, 0] = 0x4000
    assert O.widen(other)[0, 0] == 2.0 and O.widen(bits)[0, 0] == 1.0
    f = np.array([[0.1, -3.5]], dtype=np.float32)
    assert np.array_equal(O.widen(f), f.astype(np.float64))
    O.clear_widen_cache()
    assert O.widen(bits) is not got and np.array_equal(O.widen(bits), want)
    O.clear_widen_cache()


def test_softmax_rows_closed_forms():
    """Rows of equal scores give 1/n each; two scores a, b give the logistic of their difference; adding a constant
    to a row changes nothing, also at magnitudes where a naive exp would overflow; -inf entries get exactly 0."""
    assert np.allclose(O.softmax_rows(np.full((3, 7), 4.2)), 1.0 / 7, rtol=0, atol=1e-16)
    a, b = 1.3, -0.4
    p = O.softmax_rows(np.array([[a, b]]))
    assert abs(p[0, 0] - 1.0 / (1.0 + math.exp(b - a))) < 1e-15 and abs(p.sum() - 1.0) < 1e-15
    s = np.array([[0.5, -2.0, 3.0, 0.0], [10.0, 9.0, -1.0, 2.5]])
    base = O.softmax_rows(s)
    for shift in (1000.0, -1000.0, 1e6):
        assert np.allclose(O.softmax_rows(s + shift), base, rtol=0, atol=1e-9)
    masked = O.softmax_rows(np.array([[0.0, -np.inf, 0.0, -np.inf]]))
    assert np.array_equal(masked, np.array([[0.5, 0.0, 0.5, 0.0]]))
