"""GPU vs the CPU oracle over seeded RANDOM decoder shapes and call patterns.

The hand-picked cases elsewhere sit on the shapes the kernels were written around; this sweep draws
what they were not tuned for - odd head counts and group sizes, d_model / d_ff / vocabulary at every
multiple the boundary accepts (64 for bf16 models, anything even-headed for fp32), prefixes built in
ragged chunks, extends of up to 700 rows that end inside a KV block, verify rounds at any k up to 16, a
batched pass over forks of unequal length, and every fifth bf16 case with split (hi + lo) activations.  Every logit of every compared row against the plain computation (paper
Sec. 2.3: an extend over a cached prefix equals the full forward; verification accepts exactly the
greedy continuation), tolerances as everywhere: 1e-4 (fp32) / 2e-2 (bf16) max-abs, decisions exact
wherever the oracle's top-2 margin exceeds 1e-2.
"""
import numpy as np
import pytest

from oracle import decoder as O
from paper_2605_10380_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
MARGIN = 1e-2


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_10380_amd import binding
    return binding


def draw_shape(rng, case):
    if case % 4 == 3:                                            # fp32: plain kernels, any sizes
        hd = int(rng.choice([16, 32, 48, 64, 96]))
        hkv = int(rng.integers(1, 4))
        g = int(rng.integers(1, 5))
        return I.DecoderShape(f"r{case}", int(rng.integers(1, 3)), int(rng.integers(5, 40)) * 4, hkv * g, hkv, hd,
                              int(rng.integers(20, 200)) * 2 + 1, int(rng.integers(50, 700)), "f32")
    hd = int(rng.choice([64, 128]))
    hkv = int(rng.integers(1, 5))
    g = int(rng.choice([1, 2, 3, 4, 5, 8]))
    return I.DecoderShape(f"r{case}", int(rng.integers(1, 4)), 64 * int(rng.integers(2, 11)), hkv * g, hkv, hd,
                          64 * int(rng.integers(3, 21)), 64 * int(rng.integers(5, 41)), "bf16")


def check(sh, got, ref, what):
    err = float(np.abs(got.astype(np.float64) - ref).max())
    assert err <= TOL[sh.dtype], (what, err)
    return err


@pytest.mark.parametrize("case", range(48))
def test_random_shape_and_call_pattern(B, case):
    rng = np.random.default_rng(7000 + case)
    sh = draw_shape(rng, case)
    P = int(rng.integers(0, 420))
    T = int(rng.integers(1, 230)) if case % 8 else int(rng.integers(257, 700))      # every eighth: the many-row kernels
    k_list = [int(rng.integers(0, 17)) for _ in range(3)]
    print(f"case {case}: {sh}, P={P} T={T} k={k_list}", flush=True)
    w = I.make_weights(sh, 7000 + case)
    toks = I.templated_prompt(sh.vocab, 7000 + case, P + T + 64)
    assert P + T + 3 * 17 + 60 <= 1536
    split = 1 if sh.dtype == "bf16" and case % 5 == 4 else 0
    dm = B.DeviceModel(sh, w, max_pos=1536, max_tokens=768, pool_tokens=6144, max_seqs=3, act_split=split)
    kv, ref_kv = dm.new_kv(), O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)

    # prefix in ragged chunks (the oracle takes it in one go: the result must not depend on the cut)
    at = 0
    while at < P:
        c = min(P - at, int(rng.integers(1, 200)))
        dm.extend(kv, toks[at:at + c])
        at += c
    if P:
        O.forward(sh, w, toks[:P], ref_kv, rows=[-1])
    got = dm.extend(kv, toks[P:P + T], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, toks[P:P + T], ref_kv)
    errs = [check(sh, got, ref, f"extend P={P} T={T}")]

    # verify rounds: the first j drafts are the greedy continuation, draft j is wrong (j seeded)
    pending = O.argmax_lowest(ref[-1])
    exempt = 0
    for r, k in enumerate(k_list):
        Pn = len(ref_kv)
        greedy = O.greedy_decode(sh, w, ref_kv.fork(), pending, k) if k else []
        drafts = I.seeded_accept_drafts(np.array(greedy[:k]), sh.vocab, 7000 + case, r, k)[0] if k else np.zeros(0, np.int32)
        a_ref, nxt_ref, logits = O.verify(sh, w, ref_kv, pending, drafts)
        a, nxt = dm.verify(kv, pending, drafts)
        assert B.ax_kv_len(kv) == Pn + 1 + a
        if (a, nxt) != (a_ref, nxt_ref):
            assert O.top2_margin(logits[min(a, a_ref)]) <= MARGIN, (r, k, a, a_ref, nxt, nxt_ref)
            exempt += 1
            if a > a_ref:
                B.ax_kv_truncate(kv, Pn + 1 + a_ref)
            elif a < a_ref:
                dm.extend(kv, np.asarray(drafts[a:a_ref], dtype=np.int32))
        pending = nxt_ref
    assert exempt <= 1

    # three forks of unequal length extended by unequal amounts in one batched pass
    n_now = len(ref_kv)
    cuts = [n_now, max(1, n_now - int(rng.integers(0, 20))), max(1, n_now // 2)]
    t_each = [int(rng.integers(1, 60)) for _ in range(3)]
    kvs, refs, news = [], [], []
    for s in range(3):
        kvs.append(B.ax_kv_fork(kv, cuts[s]))
        rk = ref_kv.fork()
        rk.truncate(cuts[s])
        refs.append(rk)
        news.append(I.zipf_tokens(sh.vocab, 7000 + case, f"n{s}", t_each[s]))
    gotb = dm.extend_batch(kvs, news, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    at = 0
    for s in range(3):
        refb = O.forward(sh, w, news[s], refs[s])
        errs.append(check(sh, gotb[at:at + t_each[s]], refb, f"batched fork {s} (len {cuts[s]} + {t_each[s]})"))
        assert B.ax_kv_len(kvs[s]) == len(refs[s])
        at += t_each[s]
    print(f"case {case}: max-abs logit errors {['%.2e' % e for e in errs]} (limit {TOL[sh.dtype]:.0e}), exempt rounds {exempt}", flush=True)
    for h in kvs + [kv]:
        B.ax_kv_free(h)
    assert B.ax_pool_stats(dm.pool)[0] == B.ax_pool_stats(dm.pool)[1]
    dm.close()


@pytest.mark.parametrize("case", range(16))
def test_random_sessions_batched(B, case):
    """2-12 sessions forked at random points of one prefix (long enough, in half of the cases, for the
    shared-prefix attention pass), private histories of random length, then rounds that alternate a batched
    extend of random lengths (last-row logits against the oracle) and a batched verify with a random draft
    count per session, 0 included; finally one session is exported, imported into fresh blocks and must
    continue exactly like the original."""
    rng = np.random.default_rng(9000 + case)
    sh = draw_shape(rng, case if case % 4 != 3 else case + 1)            # bf16 shapes only: the batched paths with MFMA attention
    n = int(rng.integers(2, 13))
    plen = int(rng.integers(40, 200)) if case % 2 else int(rng.integers(500, 900))
    print(f"case {case}: {sh}, {n} sessions, prefix {plen}", flush=True)
    w = I.make_weights(sh, 9000 + case)
    prefix = I.templated_prompt(sh.vocab, 9000 + case, plen)
    dm = B.DeviceModel(sh, w, max_pos=1536, max_tokens=512, pool_tokens=16384, max_seqs=n)
    root, root_ref = dm.new_kv(), O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    for at in range(0, plen, 256):
        dm.extend(root, prefix[at:at + 256])
    O.forward(sh, w, prefix, root_ref, rows=[-1])
    kvs, refs, pend = [], [], []
    for s in range(n):
        cut = plen if rng.random() < 0.7 else int(rng.integers(1, plen + 1))
        kv, ref = B.ax_kv_fork(root, cut), root_ref.fork()
        ref.truncate(cut)
        hl = int(rng.integers(0, 60))
        h = I.zipf_tokens(sh.vocab, 9000 + case, f"h{s}", hl + 1)
        if hl:
            dm.extend(kv, h[:hl])
            O.forward(sh, w, h[:hl], ref, rows=[-1])
        kvs.append(kv)
        refs.append(ref)
        pend.append(int(h[hl]))
    exempt = 0
    worst = 0.0
    for r in range(2):
        budget = 512 // n
        news = [I.zipf_tokens(sh.vocab, 9000 + case, f"n{r}/{s}", int(rng.integers(1, min(40, budget) + 1))) for s in range(n)]
        got = dm.extend_batch(kvs, news, B.AX_OUT_LAST_LOGITS).cpu().numpy()
        for s in range(n):
            worst = max(worst, check(sh, got[s], O.forward(sh, w, news[s], refs[s])[-1], f"round {r} session {s}"))
        ks = [int(rng.integers(0, 17)) for _ in range(n)]
        drafts = []
        for s in range(n):
            g = O.greedy_decode(sh, w, refs[s].fork(), pend[s], ks[s]) if ks[s] else []
            d = I.seeded_accept_drafts(np.array(g), sh.vocab, 9000 + case, 100 * r + s, ks[s])[0] if ks[s] else np.zeros(0, np.int32)
            drafts.append([int(t) for t in d])
        lens = [len(ref) for ref in refs]
        acc, nxt = dm.verify_batch(kvs, pend, drafts)
        for s in range(n):
            a_ref, n_ref, logits = O.verify(sh, w, refs[s], pend[s], drafts[s])
            assert B.ax_kv_len(kvs[s]) == lens[s] + 1 + acc[s]
            if (acc[s], nxt[s]) != (a_ref, n_ref):
                assert O.top2_margin(logits[min(acc[s], a_ref)]) <= MARGIN, (r, s, ks[s], acc[s], a_ref, nxt[s], n_ref)
                exempt += 1
                if acc[s] > a_ref:
                    B.ax_kv_truncate(kvs[s], lens[s] + 1 + a_ref)
                elif acc[s] < a_ref:
                    dm.extend(kvs[s], np.asarray(drafts[s][acc[s]:a_ref], dtype=np.int32))
            pend[s] = n_ref
    assert exempt <= max(2, n // 3)
    # stored prefix: export one session, import it into fresh blocks, both continue alike (bit for bit)
    s = int(rng.integers(0, n))
    image = dm.export_kv(kvs[s])
    twin = dm.import_kv(image)
    assert B.ax_kv_len(twin) == B.ax_kv_len(kvs[s]) and set(B.ax_kv_blocks(twin)).isdisjoint(B.ax_kv_blocks(kvs[s]))
    cont = I.zipf_tokens(sh.vocab, 9000 + case, "cont", 20)
    a1 = dm.extend(kvs[s], cont, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    a2 = dm.extend(twin, cont, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert np.array_equal(a1, a2)
    check(sh, a1, O.forward(sh, w, cont, refs[s]), "continuation after the round trip")
    print(f"case {case}: worst logit error {worst:.2e}, exempt {exempt}", flush=True)
    for h in kvs + [root, twin]:
        B.ax_kv_free(h)
    assert B.ax_pool_stats(dm.pool)[0] == B.ax_pool_stats(dm.pool)[1]
    dm.close()


EXTREME = {
    # name: (layers, d_model, Hq, Hkv, hd, d_ff, vocab) - ratios no real decoder has, all accepted by the boundary
    "wide-heads": (2, 64, 16, 2, 128, 64, 64),            # q/k/v columns = 40 d_model
    "one-head": (2, 1024, 1, 1, 64, 64, 64),              # q columns = d_model / 16
    "fat-mlp": (1, 64, 2, 1, 64, 4096, 128),              # d_ff = 64 d_model
    "thin-mlp": (2, 768, 12, 4, 64, 64, 192),             # d_ff = d_model / 12
    "big-vocab": (1, 64, 2, 2, 64, 128, 50048),           # vocabulary = 782 d_model
    "g16": (2, 256, 16, 1, 64, 256, 256),                 # 16 query heads per KV head
    "g32-hd128": (1, 128, 32, 1, 128, 192, 320),          # 32 query heads per KV head
    "many-kv-heads": (1, 128, 12, 12, 64, 128, 128),      # as many KV heads as query heads, more than 8
}


@pytest.mark.parametrize("split", [0, 1], ids=["single", "split"])
@pytest.mark.parametrize("name", list(EXTREME))
def test_extreme_ratios_at_every_row_count_class(B, name, split):
    """Shapes at the edges of what the boundary accepts, extended by row counts on both sides of every kernel
    choice (1, 16 | 17, 32 | 33, 64 | 65, 128 | 129, 192 | 193, 256 | 257, 512 | 513, 700), every logit against the
    oracle; then verify rounds at k = 0, 15, 16 and a last extend, which read everything the large calls may have
    overrun in the workspace.  Each shape with single and with split (hi + lo) activations."""
    L, d, hq, hkv, hd, F, V = EXTREME[name]
    sh = I.DecoderShape(name, L, d, hq, hkv, hd, F, V, "bf16")
    w = I.make_weights(sh, 8100)
    toks = I.templated_prompt(sh.vocab, 8100, 3200)
    dm = B.DeviceModel(sh, w, max_pos=3200, max_tokens=704, pool_tokens=4096, act_split=1 if split else -1)
    kv, ref_kv = dm.new_kv(), O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    at, worst = 0, 0.0
    for M in (1, 16, 17, 32, 33, 64, 65, 128, 129, 192, 193, 256, 257, 513, 700, 512, 1):
        got = dm.extend(kv, toks[at:at + M], B.AX_OUT_ALL_LOGITS).cpu().numpy()
        ref = O.forward(sh, w, toks[at:at + M], ref_kv)
        worst = max(worst, check(sh, got, ref, f"{name}: {M} rows over {at}"))
        at += M
    pending = O.argmax_lowest(ref[-1])
    for r, k in enumerate((0, 15, 16)):
        greedy = O.greedy_decode(sh, w, ref_kv.fork(), pending, k) if k else []
        drafts = I.seeded_accept_drafts(np.array(greedy[:k]), sh.vocab, 8100, r, k)[0] if k else np.zeros(0, np.int32)
        Pn = len(ref_kv)
        a_ref, nxt_ref, logits = O.verify(sh, w, ref_kv, pending, drafts)
        a, nxt = dm.verify(kv, pending, drafts)
        if (a, nxt) != (a_ref, nxt_ref):
            assert O.top2_margin(logits[min(a, a_ref)]) <= MARGIN, (name, k, a, a_ref, nxt, nxt_ref)
            if a > a_ref:
                B.ax_kv_truncate(kv, Pn + 1 + a_ref)
            elif a < a_ref:
                dm.extend(kv, np.asarray(drafts[a:a_ref], dtype=np.int32))
        pending = nxt_ref
    tail = I.zipf_tokens(sh.vocab, 8100, "tail", 9)
    worst = max(worst, check(sh, dm.extend(kv, tail, B.AX_OUT_ALL_LOGITS).cpu().numpy(), O.forward(sh, w, tail, ref_kv), f"{name}: tail"))
    print(f"{name}: worst max-abs logit error {worst:.2e}", flush=True)
    B.ax_kv_free(kv)
    dm.close()


@pytest.mark.parametrize("which,S", [("hd64-g4", 200), ("hd128-g3", 96), ("f32", 64)])
def test_many_sessions_at_the_configured_limits(B, which, S):
    """max_seqs sessions in every call and exactly max_tokens rows in the last one: one-token decode steps of all
    sessions batched, a batched verify with k = 0 / 1, and a batched extend whose row total equals max_tokens with
    one long sequence among one-token ones.  Last-row logits / acceptance of EVERY session against the oracle."""
    sh = {"hd64-g4": I.DecoderShape("m64", 2, 256, 8, 2, 64, 512, 512, "bf16"),
          "hd128-g3": I.DecoderShape("m128", 2, 384, 6, 2, 128, 384, 512, "bf16"),
          "f32": I.DecoderShape("mf32", 2, 96, 6, 3, 32, 200, 301, "f32")}[which]
    max_tokens = 256
    rng = np.random.default_rng(8800 + S)
    w = I.make_weights(sh, 8800)
    prefix = I.templated_prompt(sh.vocab, 8800, 100)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=max_tokens, pool_tokens=100 + S * 96 + 512, max_seqs=S)
    root, root_ref = dm.new_kv(), O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    dm.extend(root, prefix)
    O.forward(sh, w, prefix, root_ref, rows=[-1])
    kvs = [B.ax_kv_fork(root, 100 if s % 3 else 90 + s % 10) for s in range(S)]
    refs = []
    for s in range(S):
        r = root_ref.fork()
        r.truncate(100 if s % 3 else 90 + s % 10)
        refs.append(r)
    tol = TOL[sh.dtype]
    worst = 0.0
    # 1. one token per session
    news = [I.zipf_tokens(sh.vocab, 8800, f"a{s}", 1) for s in range(S)]
    got = dm.extend_batch(kvs, news, B.AX_OUT_LAST_LOGITS).cpu().numpy()
    pend = []
    for s in range(S):
        ref = O.forward(sh, w, news[s], refs[s])[-1]
        worst = max(worst, float(np.abs(got[s] - ref).max()))
        pend.append(O.argmax_lowest(ref))
    assert worst <= tol, worst
    # 2. batched verify, k = 0 or 1, as many rows as fit
    room = max_tokens - S
    ks = [1 if s < room and rng.random() < 0.5 else 0 for s in range(S)]
    drafts = []
    for s in range(S):
        g = O.greedy_decode(sh, w, refs[s].fork(), pend[s], 1) if ks[s] else []
        drafts.append([int(g[0]) if rng.random() < 0.6 else (int(g[0]) + 1) % sh.vocab] if ks[s] else [])
    lens = [len(r) for r in refs]
    acc, nxt = dm.verify_batch(kvs, pend, drafts)
    exempt = 0
    for s in range(S):
        a_ref, n_ref, logits = O.verify(sh, w, refs[s], pend[s], drafts[s])
        assert B.ax_kv_len(kvs[s]) == lens[s] + 1 + acc[s]
        if (acc[s], nxt[s]) != (a_ref, n_ref):
            assert O.top2_margin(logits[min(acc[s], a_ref)]) <= MARGIN, (s, ks[s], acc[s], a_ref, nxt[s], n_ref)
            exempt += 1
            if acc[s] > a_ref:
                B.ax_kv_truncate(kvs[s], lens[s] + 1 + a_ref)
            elif acc[s] < a_ref:
                dm.extend(kvs[s], np.asarray(drafts[s][acc[s]:a_ref], dtype=np.int32))
    assert exempt <= S // 20 + 1
    # 3. exactly max_tokens rows: one long sequence (at a random place) among one-token ones
    long_s = int(rng.integers(0, S))
    news = [I.zipf_tokens(sh.vocab, 8800, f"c{s}", max_tokens - (S - 1) if s == long_s else 1) for s in range(S)]
    got = dm.extend_batch(kvs, news, B.AX_OUT_LAST_LOGITS).cpu().numpy()
    for s in range(S):
        ref = O.forward(sh, w, news[s], refs[s])[-1]
        worst = max(worst, float(np.abs(got[s] - ref).max()))
    assert worst <= tol, worst
    # one row too many is refused and changes nothing
    lens = [B.ax_kv_len(k) for k in kvs]
    over = [np.array([1, 2], np.int32) if s == 0 else np.array([1], np.int32) for s in range(S)]
    over[long_s] = I.zipf_tokens(sh.vocab, 8800, "over", max_tokens - (S - 1))
    with pytest.raises(B.AxError):
        dm.extend_batch(kvs, over, B.AX_OUT_LAST_LOGITS)
    assert [B.ax_kv_len(k) for k in kvs] == lens
    print(f"{which}, {S} sessions: worst max-abs logit error {worst:.2e} (limit {tol:.0e}), exempt {exempt}", flush=True)
    for h in kvs + [root]:
        B.ax_kv_free(h)
    assert B.ax_pool_stats(dm.pool)[0] == B.ax_pool_stats(dm.pool)[1]
    dm.close()


@pytest.mark.parametrize("case", range(12))
def test_random_draft_verify_loops(B, case):
    """The library's draft / verify / rollback loop (paper Sec. 4.3: n-gram table, selective fallback, drafts
    produced regardless after a first hit) against the oracle's loop over random shapes, window lengths n = 2..5,
    draft counts k = 1..16, table contents (the model's own continuation, corrupted at a random rate) and
    generation lengths: same tokens and the same round / fallback / drafted / accepted counts, a first differing
    token only where the oracle's top-2 margin is at most 1e-2."""
    from oracle import exspec as X
    rng = np.random.default_rng(9500 + case)
    sh = draw_shape(rng, case)
    n, k = int(rng.integers(2, 6)), int(rng.integers(1, 17))
    max_new, plen = int(rng.integers(5, 70)), int(rng.integers(n, 120))
    selective = bool(rng.integers(0, 2))
    corrupt = float(rng.choice([0.0, 0.1, 0.3, 0.9]))
    print(f"case {case}: {sh}, n={n} k={k} max_new={max_new} prompt={plen} selective={selective} corrupt={corrupt}", flush=True)
    w = I.make_weights(sh, 9500 + case)
    prompt = I.templated_prompt(sh.vocab, 9500 + case, plen)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=128, pool_tokens=1024)
    kv, ref_kv = dm.new_kv(), O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    dm.extend(kv, prompt)
    pending = O.argmax_lowest(O.forward(sh, w, prompt, ref_kv)[-1])
    gkv = ref_kv.fork()
    greedy, margins, tok = [], [], pending
    for _ in range(max_new):
        lg = O.forward(sh, w, [tok], gkv)[-1]
        tok = O.argmax_lowest(lg)
        greedy.append(tok)
        margins.append(O.top2_margin(lg))
    example = np.array([pending] + greedy[:max(1, int(max_new * 0.8))])
    bad = rng.random(len(example)) < corrupt
    example = np.where(bad, rng.integers(0, sh.vocab, len(example)), example)
    stream = np.concatenate([prompt, example]).astype(np.int32)
    ref_lut = X.build_lut(stream, n)
    lut = B.ax_lut_build(stream, n, sh.vocab)
    assert B.ax_lut_size(lut) == len(ref_lut)
    want, wst = X.generate(sh, w, ref_kv, ref_lut, n, prompt, pending, max_new, k, selective, seed=case)
    assert want == greedy
    got, gst = B.ax_exspec_generate(dm.model, kv, lut, prompt, pending, max_new, k, selective, seed=case, stream=dm.stream)
    diff = next((i for i in range(max_new) if got[i] != want[i]), None)
    print(f"case {case}: stats {gst} oracle {wst} first difference {diff}", flush=True)
    if diff is not None:
        assert margins[diff] <= MARGIN, (diff, margins[diff])
    else:
        assert gst == wst
        assert B.ax_kv_len(kv) == len(prompt) + max_new
    B.ax_lut_free(lut)
    B.ax_kv_free(kv)
    dm.close()


@pytest.mark.parametrize("which", ["bf16-hd64", "bf16-hd128", "f32"])
def test_verify_with_many_drafts(B, which):
    """Draft counts far beyond the usual few: k = 17, 31, 32, 63, 127 and max_tokens - 1 = 255 (the row counts of the
    many-row kernels inside a verify call), with the first j drafts right (j seeded, so acceptance lengths from 0 to
    over a hundred) - accepted length, next token and the KV length after rollback against the oracle; k = max_tokens
    is refused and leaves the sequence as it was."""
    sh = {"bf16-hd64": I.DecoderShape("v64", 2, 256, 8, 2, 64, 512, 512, "bf16"),
          "bf16-hd128": I.DecoderShape("v128", 2, 384, 6, 2, 128, 384, 512, "bf16"),
          "f32": I.DecoderShape("vf32", 2, 96, 6, 3, 32, 200, 301, "f32")}[which]
    w = I.make_weights(sh, 8600)
    prompt = I.templated_prompt(sh.vocab, 8600, 70)
    dm = B.DeviceModel(sh, w, max_pos=2048, max_tokens=256, pool_tokens=4096)
    kv, ref_kv = dm.new_kv(), O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    dm.extend(kv, prompt)
    pending = O.argmax_lowest(O.forward(sh, w, prompt, ref_kv)[-1])
    exempt, hist = 0, []
    for r, k in enumerate((17, 31, 32, 63, 127, 255)):
        Pn = len(ref_kv)
        greedy = O.greedy_decode(sh, w, ref_kv.fork(), pending, k)
        drafts = I.seeded_accept_drafts(np.array(greedy[:k]), sh.vocab, 8600, r, k)[0]
        a_ref, nxt_ref, logits = O.verify(sh, w, ref_kv, pending, drafts)
        a, nxt = dm.verify(kv, pending, drafts)
        assert B.ax_kv_len(kv) == Pn + 1 + a
        if (a, nxt) != (a_ref, nxt_ref):
            assert O.top2_margin(logits[min(a, a_ref)]) <= MARGIN, (k, a, a_ref, nxt, nxt_ref)
            exempt += 1
            if a > a_ref:
                B.ax_kv_truncate(kv, Pn + 1 + a_ref)
            elif a < a_ref:
                dm.extend(kv, np.asarray(drafts[a:a_ref], dtype=np.int32))
        pending = nxt_ref
        hist.append((k, a_ref))
    print(f"{which}: (k, accepted) {hist}, exempt {exempt}", flush=True)
    assert exempt <= 1 and max(a for _, a in hist) >= 10
    n = B.ax_kv_len(kv)
    with pytest.raises(B.AxError):
        dm.verify(kv, pending, np.zeros(256, np.int32))
    assert B.ax_kv_len(kv) == n
    B.ax_kv_free(kv)
    dm.close()
