"""GPU: the extend / verify path through the C ABI against the CPU oracle, element by element.

Tolerances are the ones the benchmark spec fixes: max-abs logit error <= 1e-4 for fp32
weights and <= 2e-2 for bf16 weights (over every vocabulary entry of every compared row);
accepted lengths and token ids identical wherever the oracle's top-2 margin exceeds 1e-2.
"""
import numpy as np
import pytest

from oracle import decoder as O
from paper_2605_10380_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
MARGIN = 1e-2

SMALL = {
    "bf16-hd64-g4": I.DecoderShape("s64", 4, 512, 8, 2, 64, 1024, 2048, "bf16"),
    "bf16-hd128-g3": I.DecoderShape("s128", 3, 384, 6, 2, 128, 768, 1024, "bf16"),
    "bf16-hd128-g1": I.DecoderShape("s128g1", 2, 256, 2, 2, 128, 512, 1024, "bf16"),
    "f32-hd32": I.DecoderShape("f32s", 2, 96, 6, 3, 32, 200, 301, "f32"),
}


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_10380_amd import binding
    return binding


def okv(sh):
    return O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)


def check_logits(sh, got, ref, what):
    err = float(np.abs(got.astype(np.float64) - ref).max())
    print(f"{what}: max-abs logit error {err:.3e} (limit {TOL[sh.dtype]:.0e}), logit std {ref.std():.3f}")
    assert err <= TOL[sh.dtype], what
    return err


def assert_argmax_of(idx, logits, slack=1e-5):
    """idx[r] is the argmax of logits[r] up to summation-order noise: its logit is within
    `slack` of the row maximum, and it is the exact argmax wherever the top-2 gap is larger."""
    for r, i in enumerate(idx):
        row = logits[r]
        assert 0 <= i < len(row) and row[i] >= row.max() - slack, (r, int(i), int(np.argmax(row)))
        if O.top2_margin(row.astype(np.float64)) > slack:
            assert i == int(np.argmax(row))


def run_verify_rounds(B, dm, sh, w, kv, ref_kv, pending, rounds, k, make_drafts):
    """Feeds both sides the same (pending, drafts) each round.  Where the results differ and the
    oracle's deciding row has a top-2 margin <= MARGIN the round is exempt and the GPU sequence
    is put back on the oracle's state; any other difference fails."""
    exempt = 0
    hist = []
    for r in range(rounds):
        P = len(ref_kv)
        assert B.ax_kv_len(kv) == P
        drafts = make_drafts(r, ref_kv, pending)
        a_ref, nxt_ref, logits = O.verify(sh, w, ref_kv, pending, drafts)
        a, nxt = dm.verify(kv, pending, drafts)
        assert B.ax_kv_len(kv) == P + 1 + a
        if (a, nxt) != (a_ref, nxt_ref):
            deciding = min(a, a_ref)
            assert O.top2_margin(logits[deciding]) <= MARGIN, (r, a, a_ref, nxt, nxt_ref)
            exempt += 1
            if a > a_ref:
                B.ax_kv_truncate(kv, P + 1 + a_ref)
            elif a < a_ref:                                  # re-run the rows the GPU dropped
                dm.extend(kv, np.asarray(drafts[a:a_ref], dtype=np.int32))
        pending = nxt_ref
        hist.append(a_ref)
    return hist, exempt, pending


# ------------------------------------------------------------------ configuration 1 (fp32)

def test_config1_workload(B):
    """Tiny fp32 decoder: prefix 512 built by extends, extend of 64, then 20 verify rounds at
    k = 4 with prompt-copied drafts, all against the oracle."""
    wl = I.WORKLOADS[1]
    sh = wl.shape
    w = I.make_weights(sh, 1001)
    prompt = I.templated_prompt(sh.vocab, 1001, wl.P + wl.T)
    dm = B.DeviceModel(sh, w, max_pos=1024, max_tokens=256, pool_tokens=2048)
    kv = dm.new_kv()
    ref_kv = okv(sh)
    # prefix in ragged chunks (spans several blocks, ends inside one)
    at = 0
    for c in (200, 7, 256, 49):
        got = dm.extend(kv, prompt[at:at + c], B.AX_OUT_LAST_LOGITS).cpu().numpy()
        ref = O.forward(sh, w, prompt[at:at + c], ref_kv)
        check_logits(sh, got[0], ref[-1], f"prefix chunk at {at}")
        at += c
    assert at == wl.P
    got = dm.extend(kv, prompt[wl.P:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, prompt[wl.P:], ref_kv)
    check_logits(sh, got, ref, "extend T=64")
    am = dm  # argmax mode agrees with the logits it came from
    pending = O.argmax_lowest(ref[-1])
    hist, exempt, _ = run_verify_rounds(B, dm, sh, w, kv, ref_kv, pending, wl.rounds, wl.k,
                                        lambda r, _kv, _p: I.prompt_copied_drafts(prompt, 1001, r, wl.k))
    print("accepted per round", hist, "exempt rounds", exempt)
    assert exempt <= wl.rounds // 2
    B.ax_kv_free(kv)
    dm.close()


# ------------------------------------------------------------------ small models, both dtypes

@pytest.mark.parametrize("which", list(SMALL))
@pytest.mark.parametrize("P,T", [(0, 1), (0, 40), (33, 1), (300, 70), (129, 130)])
def test_extend_logits_small(B, which, P, T):
    sh = SMALL[which]
    w = I.make_weights(sh, 7)
    toks = I.templated_prompt(sh.vocab, 7, P + T)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=320, pool_tokens=1024)
    kv = dm.new_kv()
    ref_kv = okv(sh)
    if P:
        dm.extend(kv, toks[:P])
        O.forward(sh, w, toks[:P], ref_kv)
    got = dm.extend(kv, toks[P:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, toks[P:], ref_kv)
    check_logits(sh, got, ref, f"{which} P={P} T={T}")
    # the other output modes agree with these logits
    B.ax_kv_truncate(kv, P)
    last = dm.extend(kv, toks[P:], B.AX_OUT_LAST_LOGITS).cpu().numpy()
    # (a different row count picks a different GEMM kernel, hence a different summation order)
    np.testing.assert_allclose(last[0], got[-1], rtol=0, atol=1e-5)
    B.ax_kv_truncate(kv, P)
    am = dm.extend(kv, toks[P:], B.AX_OUT_ALL_ARGMAX).cpu().numpy()
    assert_argmax_of(am, got)
    B.ax_kv_truncate(kv, P)
    la = dm.extend(kv, toks[P:], B.AX_OUT_LAST_ARGMAX).cpu().numpy()
    assert_argmax_of(la, got[-1:])
    B.ax_kv_free(kv)
    dm.close()


@pytest.mark.parametrize("which,P,T", [("bf16-hd64-g4", 40, 520), ("bf16-hd128-g3", 10, 700)])
def test_very_long_extend_uses_eight_tile_blocks(B, which, P, T):
    """T * G >= 2048 stacked rows: the attention launches blocks of 8 q tiles."""
    sh = SMALL[which]
    w = I.make_weights(sh, 8)
    toks = I.templated_prompt(sh.vocab, 8, P + T)
    dm = B.DeviceModel(sh, w, max_pos=1024, max_tokens=768, pool_tokens=2048)
    kv, ref_kv = dm.new_kv(), okv(sh)
    dm.extend(kv, toks[:P])
    O.forward(sh, w, toks[:P], ref_kv)
    got = dm.extend(kv, toks[P:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    check_logits(sh, got, O.forward(sh, w, toks[P:], ref_kv), f"{which} P={P} T={T}")
    B.ax_kv_free(kv)
    dm.close()


@pytest.mark.parametrize("which", ["bf16-hd64-g4", "bf16-hd128-g3", "f32-hd32"])
@pytest.mark.parametrize("k", [0, 1, 4, 8, 16])
def test_verify_rounds_seeded_acceptance(B, which, k):
    """Drafts whose first j tokens are the oracle's greedy tokens (j uniform in 0..k): partial
    acceptance and rollback every round; the emitted stream equals plain greedy decoding."""
    sh = SMALL[which]
    w = I.make_weights(sh, 9)
    prompt = I.templated_prompt(sh.vocab, 9, 90)
    rounds = 10
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=128, pool_tokens=1024)
    kv, ref_kv = dm.new_kv(), okv(sh)
    dm.extend(kv, prompt)
    pending = O.argmax_lowest(O.forward(sh, w, prompt, ref_kv)[-1])
    greedy_kv = ref_kv.fork()
    greedy = O.greedy_decode(sh, w, greedy_kv, pending, rounds * (k + 1) + k)
    emitted = [0]

    def drafts(r, kv_now, p):
        at = len(kv_now) - len(prompt)            # tokens emitted so far = index of next greedy token
        return I.seeded_accept_drafts(np.array(greedy[at:at + k] + [0]), sh.vocab, 9, r, k)[0] if k else np.zeros(0, np.int32)

    hist, exempt, _ = run_verify_rounds(B, dm, sh, w, kv, ref_kv, pending, rounds, k, drafts)
    print(which, "k", k, "accepted", hist, "exempt", exempt)
    if k >= 4:
        assert 0 < sum(hist) < k * rounds
    assert exempt <= 3
    B.ax_kv_free(kv)
    dm.close()


# ------------------------------------------------------------------ properties on the GPU itself

@pytest.mark.parametrize("which", ["bf16-hd64-g4", "f32-hd32"])
def test_prefix_reuse_fork_cow_and_rollback(B, which):
    """Extend over a cached prefix equals recomputation; forks share the prefix and diverge
    without disturbing each other (copy on write inside a shared block); a rolled-back sequence
    continues as if the rejected rows had never been there."""
    sh = SMALL[which]
    w = I.make_weights(sh, 11)
    toks = I.templated_prompt(sh.vocab, 11, 200)
    tol = TOL[sh.dtype]
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=256, pool_tokens=2048)
    full = dm.new_kv()
    ref_all = dm.extend(full, toks, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    # chunked
    ch = dm.new_kv()
    outs, at = [], 0
    for c in (1, 64, 17, 118):
        outs.append(dm.extend(ch, toks[at:at + c], B.AX_OUT_ALL_LOGITS).cpu().numpy())
        at += c
    assert np.abs(np.concatenate(outs) - ref_all).max() <= tol
    # fork inside a block (100 = 6*16 + 4), both continue differently
    f1, f2 = B.ax_kv_fork(full, 100), B.ax_kv_fork(full, 100)
    assert list(B.ax_kv_blocks(f1)) == list(B.ax_kv_blocks(full))[:7]
    alt = I.zipf_tokens(sh.vocab, 11, "alt", 30)
    o1 = dm.extend(f1, toks[100:130], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    o2 = dm.extend(f2, alt, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert B.ax_kv_blocks(f1)[6] != B.ax_kv_blocks(full)[6] and B.ax_kv_blocks(f2)[6] != B.ax_kv_blocks(f1)[6]
    assert np.abs(o1 - ref_all[100:130]).max() <= tol
    fresh = dm.new_kv()
    dm.extend(fresh, toks[:100])
    o2_ref = dm.extend(fresh, alt, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert np.abs(o2 - o2_ref).max() <= tol
    # the source still reads its own data after the forks wrote theirs
    again = dm.extend(full, toks[:5], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    B.ax_kv_truncate(full, 200)
    chk = dm.new_kv()
    dm.extend(chk, toks)
    again_ref = dm.extend(chk, toks[:5], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert np.abs(again - again_ref).max() <= tol
    # rollback: wrong drafts, then continue == continuing without them
    a, nxt = dm.verify(f1, int(toks[130]), (toks[131:135] + 1) % sh.vocab)
    assert B.ax_kv_len(f1) == 131 + a
    B.ax_kv_truncate(f1, 131)
    cont = dm.extend(f1, toks[131:150], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert np.abs(cont - ref_all[131:150]).max() <= tol
    for k in (full, ch, f1, f2, fresh, chk):
        B.ax_kv_free(k)
    assert B.ax_pool_stats(dm.pool)[0] == B.ax_pool_stats(dm.pool)[1]
    dm.close()


# 113, 143 and 180 rows in all: row counts on both sides of the 128-row block shapes
@pytest.mark.parametrize("T_each", [[33, 1, 70, 9], [33, 1, 100, 9], [60, 1, 110, 9]], ids=["113rows", "143rows", "180rows"])
@pytest.mark.parametrize("which", ["bf16-hd64-g4", "bf16-hd128-g3", "f32-hd32"])
def test_batched_mixed_length_equals_separate(B, which, T_each):
    """Several sessions with different cached lengths and different T in one pass, sharing a
    forked prefix, against the oracle and against one-at-a-time calls."""
    sh = SMALL[which]
    w = I.make_weights(sh, 13)
    prefix = I.templated_prompt(sh.vocab, 13, 72)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=256, pool_tokens=4096, max_seqs=4)
    root = dm.new_kv()
    dm.extend(root, prefix)
    hist_len = [0, 19, 40, 5]
    kvs, refs, news = [], [], []
    for s in range(4):
        kv = B.ax_kv_fork(root, 72 if s != 2 else 50)             # one session shares less
        ref = okv(sh)
        base = prefix[:72 if s != 2 else 50]
        O.forward(sh, w, base, ref)
        if hist_len[s]:
            h = I.zipf_tokens(sh.vocab, 13, f"h{s}", hist_len[s])
            dm.extend(kv, h)
            O.forward(sh, w, h, ref)
        kvs.append(kv)
        refs.append(ref)
        news.append(I.zipf_tokens(sh.vocab, 13, f"n{s}", T_each[s]))
    got = dm.extend_batch(kvs, news, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    at = 0
    for s in range(4):
        ref = O.forward(sh, w, news[s], refs[s])
        check_logits(sh, got[at:at + T_each[s]], ref, f"batched session {s}")
        assert B.ax_kv_len(kvs[s]) == len(refs[s])
        at += T_each[s]
    last = None
    for s in range(4):
        B.ax_kv_truncate(kvs[s], B.ax_kv_len(kvs[s]) - T_each[s])
    last = dm.extend_batch(kvs, news, B.AX_OUT_LAST_ARGMAX).cpu().numpy()
    ends = np.cumsum(T_each) - 1
    assert_argmax_of(last, got[ends])
    for kv in kvs + [root]:
        B.ax_kv_free(kv)
    dm.close()


def test_errors_leave_kv_untouched(B):
    sh = SMALL["f32-hd32"]
    w = I.make_weights(sh, 15)
    dm = B.DeviceModel(sh, w, max_pos=64, max_tokens=32, pool_tokens=48)
    kv = dm.new_kv()
    dm.extend(kv, [1, 2, 3])
    for bad, status in [([], B.AX_ERR_INVALID), ([sh.vocab], B.AX_ERR_INVALID), ([-1], B.AX_ERR_INVALID),
                        (list(range(33)), B.AX_ERR_INVALID), (list(range(30)) * 3, B.AX_ERR_INVALID)]:
        with pytest.raises(B.AxError) as e:
            dm.extend(kv, bad, B.AX_OUT_LAST_ARGMAX)
        assert e.value.status == status and B.ax_kv_len(kv) == 3
    other = dm.new_kv()
    dm.extend(other, list(range(30)))               # 2 of 3 blocks
    with pytest.raises(B.AxError) as e:
        dm.extend(kv, list(range(32)))              # needs 2 more, 0 free
    assert e.value.status == B.AX_ERR_OOM and B.ax_kv_len(kv) == 3 and len(B.ax_kv_blocks(kv)) == 1
    with pytest.raises(B.AxError):
        dm.verify(kv, 1, [sh.vocab + 5])
    assert B.ax_kv_len(kv) == 3
    B.ax_kv_free(kv)
    B.ax_kv_free(other)
    dm.close()


@pytest.mark.parametrize("which", ["bf16-hd64-g4", "f32-hd32"])
def test_limits_are_reachable(B, which):
    """Exactly max_tokens rows in one call, a sequence filled to exactly max_pos, a verify round
    with the most drafts a call can carry, max_seqs sequences in one batch, one token on an empty
    sequence - each against the oracle; one past each limit is refused."""
    sh = SMALL[which]
    w = I.make_weights(sh, 71)
    MT, MP, MS = 96, 208, 3
    dm = B.DeviceModel(sh, w, max_pos=MP, max_tokens=MT, pool_tokens=1024, max_seqs=MS)
    toks = I.templated_prompt(sh.vocab, 71, MP)
    kv, ref = dm.new_kv(), okv(sh)
    got = dm.extend(kv, toks[:1], B.AX_OUT_ALL_LOGITS).cpu().numpy()             # one token, empty cache
    check_logits(sh, got, O.forward(sh, w, toks[:1], ref), "T=1 on an empty sequence")
    got = dm.extend(kv, toks[1:1 + MT], B.AX_OUT_LAST_LOGITS).cpu().numpy()      # max_tokens rows
    check_logits(sh, got[0], O.forward(sh, w, toks[1:1 + MT], ref)[-1], "T = max_tokens")
    with pytest.raises(B.AxError):
        dm.extend(kv, toks[:MT + 1])
    got = dm.extend(kv, toks[1 + MT:MP - 16], B.AX_OUT_LAST_LOGITS).cpu().numpy()
    O.forward(sh, w, toks[1 + MT:MP - 16], ref)
    got = dm.extend(kv, toks[MP - 16:MP], B.AX_OUT_LAST_LOGITS).cpu().numpy()     # ends exactly at max_pos
    check_logits(sh, got[0], O.forward(sh, w, toks[MP - 16:MP], ref)[-1], "P + T = max_pos")
    assert B.ax_kv_len(kv) == MP
    with pytest.raises(B.AxError):
        dm.extend(kv, toks[:1])
    with pytest.raises(B.AxError):
        dm.verify(kv, int(toks[0]), [])                                           # no room for the pending token
    B.ax_kv_truncate(kv, 100)
    ref.truncate(100)
    drafts = I.zipf_tokens(sh.vocab, 71, "d", MT - 1)                             # 1 + k = max_tokens rows
    a_ref, n_ref, lg = O.verify(sh, w, ref, int(toks[100]), drafts)
    a, nxt = dm.verify(kv, int(toks[100]), drafts)
    if O.top2_margin(lg[min(a, a_ref)]) > MARGIN:
        assert (a, nxt) == (a_ref, n_ref)
    with pytest.raises(B.AxError):
        dm.verify(kv, int(toks[100]), I.zipf_tokens(sh.vocab, 71, "d", MT))
    # max_seqs sequences in one call; one more is refused
    kvs = [dm.new_kv() for _ in range(MS + 1)]
    news = [toks[10 * s:10 * s + 7 + s] for s in range(MS + 1)]
    got = dm.extend_batch(kvs[:MS], news[:MS], B.AX_OUT_LAST_LOGITS).cpu().numpy()
    for s in range(MS):
        check_logits(sh, got[s], O.forward(sh, w, news[s], okv(sh))[-1], f"batch of max_seqs, sequence {s}")
    with pytest.raises(B.AxError):
        dm.extend_batch(kvs, news)
    assert B.ax_kv_len(kvs[MS]) == 0
    for k_ in kvs + [kv]:
        B.ax_kv_free(k_)
    dm.close()


# ------------------------------------------------------------------ full-size shapes

@pytest.mark.parametrize("name,P,T,k", [("1b", 4096, 256, 8)])
def test_full_width_two_layers(B, name, P, T, k):
    """(The ~3B and ~8B widths at their own P and T: tests/test_gpu_config_sizes.py.)
    The real per-layer shape and vocabulary of the ~1B decoder, cut to two layers so
    that the oracle finishes in seconds: the launch shapes (GEMM tiles, attention splits, LM
    head) are the ones the benchmark times.  Full prefix P, extend T, then verify rounds."""
    sh = I.SHAPES[name].with_layers(2)
    w = I.make_weights(sh, 2002)
    prompt = I.templated_prompt(sh.vocab, 2002, P + T)
    dm = B.DeviceModel(sh, w, max_pos=P + T + 256, max_tokens=512, pool_tokens=P + T + 512)
    kv, ref_kv = dm.new_kv(), okv(sh)
    for at in range(0, P, 512):
        dm.extend(kv, prompt[at:at + 512])
    O.forward(sh, w, prompt[:P], ref_kv)
    got = dm.extend(kv, prompt[P:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, prompt[P:], ref_kv)
    check_logits(sh, got, ref, f"{sh.name} extend P={P} T={T}")
    pending = O.argmax_lowest(ref[-1])
    greedy = O.greedy_decode(sh, w, ref_kv.fork(), pending, 3 * (k + 1) + k)

    def drafts(r, kv_now, p):
        at = len(kv_now) - (P + T)
        return I.seeded_accept_drafts(np.array(greedy[at:at + k]), sh.vocab, 2002, r, k)[0]

    hist, exempt, _ = run_verify_rounds(B, dm, sh, w, kv, ref_kv, pending, 3, k, drafts)
    print(sh.name, "accepted", hist, "exempt", exempt)
    B.ax_kv_free(kv)
    dm.close()


def test_graph_replays_match_eager_verify(B):
    """Verify rounds replay a captured graph.  Several replays, with eager extends and
    synchronisations in between and the cache growing across a block boundary and across a
    change of the key-slice count, must give exactly what the uncaptured path gives."""
    sh = SMALL["bf16-hd64-g4"]
    w = I.make_weights(sh, 17)
    prompt = I.templated_prompt(sh.vocab, 17, 400)
    eager = B.DeviceModel(sh, w, max_pos=1024, max_tokens=128, pool_tokens=2048)
    B.ax_dbg_use_graphs(eager.model, False)
    graph = B.DeviceModel(sh, w, max_pos=1024, max_tokens=128, pool_tokens=2048)
    ke, kg = eager.new_kv(), graph.new_kv()
    eager.extend(ke, prompt[:100])
    graph.extend(kg, prompt[:100])
    pending = int(prompt[100])
    at = 101
    for r in range(24):
        k = (4, 8, 0, 4)[r % 4]
        drafts = prompt[at:at + k].copy()
        if r % 3 == 0 and k:
            drafts[k // 2] = (drafts[k // 2] + 1) % sh.vocab
        res_e = eager.verify(ke, pending, drafts)
        res_g = graph.verify(kg, pending, drafts)
        assert res_e == res_g, (r, res_e, res_g)
        assert B.ax_kv_len(ke) == B.ax_kv_len(kg)
        if r % 5 == 4:                                   # eager work between replays
            chunk = prompt[at:at + 37]
            le = eager.extend(ke, chunk, B.AX_OUT_LAST_LOGITS).cpu().numpy()
            lg = graph.extend(kg, chunk, B.AX_OUT_LAST_LOGITS).cpu().numpy()
            np.testing.assert_array_equal(le, lg)
            at += 37
        pending = res_e[1]
    le = eager.extend(ke, prompt[300:310], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    lg = graph.extend(kg, prompt[300:310], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    np.testing.assert_array_equal(le, lg)
    for dm, kv in ((eager, ke), (graph, kg)):
        B.ax_kv_free(kv)
        dm.close()


# ------------------------------------------------------------------ example-based drafter + decode loop

@pytest.mark.parametrize("which", ["bf16-hd64-g4", "f32-hd32"])
@pytest.mark.parametrize("selective", [True, False])
def test_exspec_loop_equals_oracle_loop(B, which, selective):
    """The library's draft-verify-rollback loop against the oracle's loop: same tokens, same
    round / fallback / drafted / accepted counts.  The table is built from the prompt plus a
    partly corrupted copy of the model's own greedy continuation, so rounds hit, miss and are
    partially accepted.  A first differing token is tolerated only where the oracle's top-2
    margin is <= MARGIN; otherwise tokens and counts are identical."""
    from oracle import exspec as X
    sh = SMALL[which]
    w = I.make_weights(sh, 21)
    prompt = I.templated_prompt(sh.vocab, 21, 75)
    n, k, max_new = 3, 6, 48
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=128, pool_tokens=1024)
    kv, ref_kv = dm.new_kv(), okv(sh)
    dm.extend(kv, prompt)
    pending = O.argmax_lowest(O.forward(sh, w, prompt, ref_kv)[-1])
    # greedy continuation with margins
    gkv = ref_kv.fork()
    greedy, margins, tok = [], [], pending
    for _ in range(max_new):
        lg = O.forward(sh, w, [tok], gkv)[-1]
        tok = O.argmax_lowest(lg)
        greedy.append(tok)
        margins.append(O.top2_margin(lg))
    rng = np.random.default_rng(21)
    example = np.array([pending] + greedy[:40])
    bad = rng.random(len(example)) < 0.15
    example = np.where(bad, rng.integers(0, sh.vocab, len(example)), example)
    stream = np.concatenate([prompt, example]).astype(np.int32)
    ref_lut = X.build_lut(stream, n)
    lut = B.ax_lut_build(stream, n, sh.vocab)
    assert B.ax_lut_size(lut) == len(ref_lut)
    want, wst = X.generate(sh, w, ref_kv, ref_lut, n, prompt, pending, max_new, k, selective, seed=3)
    assert want == greedy                                     # the oracle loop itself is lossless
    got, gst = B.ax_exspec_generate(dm.model, kv, lut, prompt, pending, max_new, k, selective, seed=3, stream=dm.stream)
    diff = next((i for i in range(max_new) if got[i] != want[i]), None)
    print(which, "selective", selective, "stats", gst, "oracle", wst, "first difference", diff)
    if diff is not None:                                      # only a near-tie may decide differently
        assert margins[diff] <= MARGIN, (diff, margins[diff])
    else:
        assert gst == wst
        assert B.ax_kv_len(kv) == len(prompt) + max_new
        assert 0 < gst["accepted"] < gst["drafted"] and gst["rounds"] < max_new
    B.ax_lut_free(lut)
    B.ax_kv_free(kv)
    dm.close()


def test_exspec_loop_is_lossless_on_the_gpu(B):
    """Whatever the table holds (here: built from unrelated text, non-selective, so mostly wrong
    drafts), the loop emits the GPU's own one-token-at-a-time greedy stream."""
    sh = SMALL["f32-hd32"]
    w = I.make_weights(sh, 22)
    prompt = I.templated_prompt(sh.vocab, 22, 60)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=128, pool_tokens=1024)
    kv = dm.new_kv()
    pending = int(dm.extend(kv, prompt, B.AX_OUT_LAST_ARGMAX).cpu().numpy()[0])
    base = B.ax_kv_fork(kv)
    plain, tok = [], pending
    for _ in range(30):
        _, tok = dm.verify(base, tok, [])
        plain.append(tok)
    lut = B.ax_lut_build(I.zipf_tokens(sh.vocab, 5, "other", 500), 2, sh.vocab)
    got, st = B.ax_exspec_generate(dm.model, kv, lut, prompt, pending, 30, 5, False, seed=1, stream=dm.stream)
    print("stats", st)
    assert got == plain and st["drafted"] > 0
    assert B.ax_exspec_generate(dm.model, kv, lut, prompt, got[-1], 0, 5, stream=dm.stream)[0] == []
    B.ax_lut_free(lut)
    B.ax_kv_free(base)
    B.ax_kv_free(kv)
    dm.close()


# ------------------------------------------------------------------ batched verify, two resident models

def _batched_rounds(B, dm, sh, w, kvs, refs, pend, rounds, k_of, seed):
    """`rounds` batched verify rounds over the sessions; drafts carry a seeded number of the
    oracle's own greedy tokens.  Every session's (accepted, next) must equal the oracle's unless
    the oracle's deciding row is a near-tie, in which case the session is re-synchronised."""
    exempt = 0
    accepted_total = 0
    for r in range(rounds):
        drafts, want = [], []
        for s, ref in enumerate(refs):
            k = k_of(r, s)
            g = O.greedy_decode(sh, w, ref.fork(), pend[s], k) if k else []
            d = I.seeded_accept_drafts(np.array(g), sh.vocab, seed, 100 * r + s, k)[0] if k else np.zeros(0, np.int32)
            drafts.append([int(t) for t in d])
        P = [len(ref) for ref in refs]
        acc, nxt = dm.verify_batch(kvs, pend, drafts)
        for s, ref in enumerate(refs):
            a_ref, n_ref, logits = O.verify(sh, w, ref, pend[s], drafts[s])
            assert B.ax_kv_len(kvs[s]) == P[s] + 1 + acc[s]
            if (acc[s], nxt[s]) != (a_ref, n_ref):
                assert O.top2_margin(logits[min(acc[s], a_ref)]) <= MARGIN, (r, s, acc[s], a_ref, nxt[s], n_ref)
                exempt += 1
                if acc[s] > a_ref:
                    B.ax_kv_truncate(kvs[s], P[s] + 1 + a_ref)
                elif acc[s] < a_ref:
                    dm.extend(kvs[s], np.asarray(drafts[s][acc[s]:a_ref], dtype=np.int32))
            pend[s] = n_ref
            accepted_total += a_ref
    return accepted_total, exempt


@pytest.mark.parametrize("which", ["bf16-hd64-g4", "bf16-hd128-g3", "f32-hd32"])
def test_batched_verify_mixed_k(B, which):
    """Sessions with different cached lengths and draft counts (0 included) verified in one
    forward: per-session acceptance and rollback equal the oracle's."""
    sh = SMALL[which]
    w = I.make_weights(sh, 31)
    prefix = I.templated_prompt(sh.vocab, 31, 70)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=128, pool_tokens=4096, max_seqs=5)
    root = dm.new_kv()
    dm.extend(root, prefix)
    kvs, refs, pend = [], [], []
    for s, hl in enumerate([0, 13, 37, 90, 1]):
        kv, ref = B.ax_kv_fork(root, -1), okv(sh)
        h = np.concatenate([prefix, I.zipf_tokens(sh.vocab, 31, f"h{s}", hl)]).astype(np.int32)
        if hl:
            dm.extend(kv, h[70:])
        pend.append(O.argmax_lowest(O.forward(sh, w, h, ref)[-1]))
        kvs.append(kv)
        refs.append(ref)
    ks = [[8, 0, 3, 16, 1], [0, 0, 0, 0, 0], [4, 4, 4, 4, 4], [1, 16, 0, 2, 9]]
    total, exempt = _batched_rounds(B, dm, sh, w, kvs, refs, pend, 4, lambda r, s: ks[r][s], 31)
    print(which, "accepted", total, "exempt", exempt)
    assert total > 0 and exempt <= 4
    # a batch of one equals the single-sequence call
    f = B.ax_kv_fork(kvs[0], -1)
    d = [int(t) for t in I.zipf_tokens(sh.vocab, 31, "d", 5)]
    one = dm.verify(kvs[0], pend[0], d)
    acc, nxt = dm.verify_batch([f], [pend[0]], [d])
    assert (acc[0], nxt[0]) == one and B.ax_kv_len(f) == B.ax_kv_len(kvs[0])
    # all or nothing: a bad draft token in the last session leaves every session as it was
    lens = [B.ax_kv_len(kv) for kv in kvs]
    with pytest.raises(B.AxError):
        dm.verify_batch(kvs, pend, [[1], [2], [3], [4], [sh.vocab]])
    assert [B.ax_kv_len(kv) for kv in kvs] == lens
    for kv in kvs + [root, f]:
        B.ax_kv_free(kv)
    dm.close()


@pytest.mark.parametrize("which", ["bf16-hd64-g4", "bf16-hd128-g3"])
def test_batched_verify_over_a_long_shared_prefix(B, which):
    """Sessions forked from one 600-token prefix (it ends inside a block, so the last shared
    block is copied on the first private write): the batched verify applies the prefix keys to all
    sessions' rows in one shared pass and the rest per session.  Acceptance per session equals
    the oracle's; a batched extend with LAST_LOGITS over the same forks also matches."""
    sh = SMALL[which]
    w = I.make_weights(sh, 33)
    prefix = I.templated_prompt(sh.vocab, 33, 600)
    dm = B.DeviceModel(sh, w, max_pos=1024, max_tokens=320, pool_tokens=8192, max_seqs=6)
    root, root_ref = dm.new_kv(), okv(sh)
    dm.extend(root, prefix[:300])
    dm.extend(root, prefix[300:])
    O.forward(sh, w, prefix, root_ref)
    kvs, refs, pend = [], [], []
    for s, hl in enumerate([0, 5, 40, 17, 90, 33]):
        kv, ref = B.ax_kv_fork(root, -1), root_ref.fork()
        h = I.zipf_tokens(sh.vocab, 33, f"h{s}", hl + 1)
        if hl:
            dm.extend(kv, h[:hl])
            O.forward(sh, w, h[:hl], ref)
        kvs.append(kv)
        refs.append(ref)
        pend.append(int(h[hl]))
    # short batched extend (single-tile path): logits of every session against the oracle
    news = [I.zipf_tokens(sh.vocab, 33, f"n{s}", 3 + s) for s in range(6)]
    got = dm.extend_batch(kvs, news, B.AX_OUT_LAST_LOGITS).cpu().numpy()
    for s in range(6):
        check_logits(sh, got[s], O.forward(sh, w, news[s], refs[s])[-1], f"shared-prefix batch, session {s}")
    ks = [[8, 0, 3, 16, 1, 5], [4, 4, 4, 4, 4, 4], [1, 16, 0, 2, 9, 7]]
    total, exempt = _batched_rounds(B, dm, sh, w, kvs, refs, pend, 3, lambda r, s: ks[r][s], 33)
    print(which, "accepted", total, "exempt", exempt)
    assert total > 0 and exempt <= 3
    for kv in kvs + [root]:
        B.ax_kv_free(kv)
    dm.close()


def test_two_resident_models_forked_sessions(B):
    """The plan-out agent's shape at a size the oracle can follow: two decoders with their own
    weights and pools resident together; per model, sessions fork one shared prefix, build
    private histories, then interleave batched mixed-length extends with batched verify rounds
    at k = 8.  Forks must not disturb each other or the shared prefix (copy on write)."""
    sh = SMALL["bf16-hd64-g4"]
    models = []
    for mi in range(2):
        w = I.make_weights(sh, 500 + mi)
        dm = B.DeviceModel(sh, w, max_pos=1024, max_tokens=512, pool_tokens=8192, max_seqs=6)
        prefix = I.templated_prompt(sh.vocab, 500 + mi, 200)          # ends inside a block: forks copy on write
        root, root_ref = dm.new_kv(), okv(sh)
        dm.extend(root, prefix)
        O.forward(sh, w, prefix, root_ref)
        kvs, refs = [], []
        for s in range(6):
            kv, ref = B.ax_kv_fork(root, -1), root_ref.fork()
            kvs.append(kv)
            refs.append(ref)
        models.append((dm, w, root, root_ref, kvs, refs, prefix))
    rng = np.random.default_rng(5)
    pend = [[0] * 6, [0] * 6]
    for step in range(3):
        for mi, (dm, w, root, root_ref, kvs, refs, prefix) in enumerate(models):      # interleave the two models
            T_each = [int(rng.integers(2, 80)) for _ in kvs]
            news = [I.zipf_tokens(sh.vocab, 500 + mi, f"s{step}-{s}", T_each[s]) for s in range(6)]
            got = dm.extend_batch(kvs, news, B.AX_OUT_LAST_LOGITS).cpu().numpy()
            for s in range(6):
                ref = O.forward(sh, w, news[s], refs[s])
                check_logits(sh, got[s], ref[-1], f"model {mi} step {step} session {s}")
                pend[mi][s] = O.argmax_lowest(ref[-1])
            total, exempt = _batched_rounds(B, dm, sh, w, kvs, refs, pend[mi], 2, lambda r, s: 8, 500 + mi)
            assert exempt <= 3
    for dm, w, root, root_ref, kvs, refs, prefix in models:
        # the shared prefix is intact: extending a fresh fork of it reproduces the oracle
        f, fr = B.ax_kv_fork(root, -1), root_ref.fork()
        t = I.zipf_tokens(sh.vocab, 9, "probe", 20)
        check_logits(sh, dm.extend(f, t, B.AX_OUT_ALL_LOGITS).cpu().numpy(), O.forward(sh, w, t, fr), "shared prefix probe")
        for kv in kvs + [root, f]:
            B.ax_kv_free(kv)
        free, total_blocks, live = B.ax_pool_stats(dm.pool)
        assert free == total_blocks and live == 0
        dm.close()


def test_full_width_3b_batched_sessions(B):
    """The ~3B per-layer shape (two layers): four sessions over a shared 1024-token prefix with
    private histories, one batched extend and batched verify rounds at k = 8 - the launch shapes
    of the two-model workload at a depth the oracle finishes."""
    sh = I.SHAPES["3b"].with_layers(2)
    w = I.make_weights(sh, 5005)
    prefix = I.templated_prompt(sh.vocab, 5005, 1024)
    dm = B.DeviceModel(sh, w, max_pos=4096, max_tokens=1024, pool_tokens=8192, max_seqs=4)
    root, root_ref = dm.new_kv(), okv(sh)
    for at in range(0, 1024, 512):
        dm.extend(root, prefix[at:at + 512])
    O.forward(sh, w, prefix, root_ref)
    kvs, refs, pend = [], [], [0] * 4
    T_each = [300, 32, 150, 77]
    news = [I.zipf_tokens(sh.vocab, 5005, f"n{s}", T_each[s]) for s in range(4)]
    for s in range(4):
        kvs.append(B.ax_kv_fork(root, -1))
        refs.append(root_ref.fork())
    got = dm.extend_batch(kvs, news, B.AX_OUT_LAST_LOGITS).cpu().numpy()
    for s in range(4):
        ref = O.forward(sh, w, news[s], refs[s])
        check_logits(sh, got[s], ref[-1], f"3b session {s}")
        pend[s] = O.argmax_lowest(ref[-1])
    total, exempt = _batched_rounds(B, dm, sh, w, kvs, refs, pend, 2, lambda r, s: 8, 5005)
    print("3b batched: accepted", total, "exempt", exempt)
    # 155 rows in one pass: the row count of 16 sessions verified together (160-row blocks, K slices
    # in the down projection, 160-row blocks in the LM head when all logits are asked for)
    more = [I.zipf_tokens(sh.vocab, 5005, f"m{s}", t) for s, t in enumerate([40, 50, 30, 35])]
    for kv, ref in zip(kvs, refs):
        assert B.ax_kv_len(kv) == len(ref)
    got = dm.extend_batch(kvs, more, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    at = 0
    for s in range(4):
        ref = O.forward(sh, w, more[s], refs[s])
        check_logits(sh, got[at:at + len(more[s])], ref, f"3b session {s}, 155-row pass")
        at += len(more[s])
    # 256 rows in one pass: 128-row blocks everywhere, the QKV GEMM over three K slices
    more = [I.zipf_tokens(sh.vocab, 5005, f"q{s}", t) for s, t in enumerate([60, 70, 66, 60])]
    got = dm.extend_batch(kvs, more, B.AX_OUT_LAST_LOGITS).cpu().numpy()
    for s in range(4):
        ref = O.forward(sh, w, more[s], refs[s])
        check_logits(sh, got[s], ref[-1], f"3b session {s}, 256-row pass")
    for kv in kvs + [root]:
        B.ax_kv_free(kv)
    dm.close()


# ------------------------------------------------------------------ the benchmark workload at full depth

@pytest.mark.timeout(1200)
def test_config2_full_depth_extend_and_verify(B):
    """The ~1B decoder with all 16 layers at the benchmark's sizes and launch configuration:
    prefix P = 4096 built in chunks of 512, the extend of T = 256 compared on every logit of
    every row, then verify rounds at k = 8 (prompt-copied drafts, then drafts carrying a seeded
    number of the oracle's greedy tokens) compared on accepted length and next token."""
    wl = I.WORKLOADS[2]
    sh = wl.shape
    w = I.make_weights(sh, 2000)
    prompt = I.templated_prompt(sh.vocab, 2000, wl.P + wl.T)
    dm = B.DeviceModel(sh, w, max_pos=wl.P + wl.T + 1024, max_tokens=512, pool_tokens=wl.P + wl.T + 1024)
    kv, ref_kv = dm.new_kv(), okv(sh)
    for at in range(0, wl.P, 512):
        dm.extend(kv, prompt[at:at + 512])
    for at in range(0, wl.P, 1024):                     # the oracle's prefix, in pieces to bound its memory
        O.forward(sh, w, prompt[at:at + 1024], ref_kv, rows=[-1])
        print(f"oracle prefix {at + 1024}/{wl.P}", flush=True)
    got = dm.extend(kv, prompt[wl.P:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, prompt[wl.P:], ref_kv)
    check_logits(sh, got, ref, f"config 2 full depth, extend T={wl.T} over P={wl.P}")
    B.ax_kv_truncate(kv, wl.P)
    am = dm.extend(kv, prompt[wl.P:], B.AX_OUT_ALL_ARGMAX).cpu().numpy()
    assert_argmax_of(am, got)
    pending = O.argmax_lowest(ref[-1])
    hist, exempt, pending = run_verify_rounds(B, dm, sh, w, kv, ref_kv, pending, 3, wl.k,
                                              lambda r, _kv, _p: I.prompt_copied_drafts(prompt, 2000, r, wl.k))
    print("prompt-copied drafts: accepted", hist, "exempt", exempt, flush=True)
    greedy = O.greedy_decode(sh, w, ref_kv.fork(), pending, 3 * (wl.k + 1) + wl.k)
    base = len(ref_kv)

    def drafts(r, kv_now, p):
        at = len(kv_now) - base
        return I.seeded_accept_drafts(np.array(greedy[at:at + wl.k]), sh.vocab, 2000, r, wl.k)[0]

    hist2, exempt2, _ = run_verify_rounds(B, dm, sh, w, kv, ref_kv, pending, 3, wl.k, drafts)
    print("seeded drafts: accepted", hist2, "exempt", exempt2, flush=True)
    assert sum(hist2) > 0 and exempt + exempt2 <= 2
    B.ax_kv_free(kv)
    dm.close()
    O.clear_widen_cache()


# ------------------------------------------------------------------ automatic prefix reuse

@pytest.mark.parametrize("which", ["bf16-hd64-g4", "f32-hd32"])
def test_prefix_index_reuses_cached_combination(B, which):
    """A cached prompt "static part, cluster 1, cluster 3, cluster 2" serves a prompt that
    activates only clusters 1 and 3: the index finds the common prefix (token granular, here
    inside a block), the tail is cut, only the rest is computed - and the logits equal the
    oracle's full recomputation.  The cached entry itself stays intact."""
    sh = SMALL[which]
    w = I.make_weights(sh, 61)
    static = I.templated_prompt(sh.vocab, 61, 70)
    c1, c3, c2 = (I.zipf_tokens(sh.vocab, 61, f"cluster{i}", n) for i, n in ((1, 23), (3, 31), (2, 18)))
    cached = np.concatenate([static, c1, c3, c2]).astype(np.int32)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=256, pool_tokens=2048)
    idx = B.ax_index_create(dm.pool)
    kv = dm.new_kv()
    dm.extend(kv, cached)
    B.ax_index_insert(idx, kv, cached)
    B.ax_kv_free(kv)
    dynamic = I.zipf_tokens(sh.vocab, 61, "query", 27)
    prompts = {"1-3": np.concatenate([static, c1, c3, dynamic]), "1-3-2": np.concatenate([cached, dynamic]),
               "1 only": np.concatenate([static, c1, dynamic]), "other": np.concatenate([dynamic, static])}
    expect = {"1-3": 70 + 23 + 31, "1-3-2": len(cached), "1 only": 70 + 23, "other": 0}
    for name, p in prompts.items():
        p = p.astype(np.int32)
        got_kv, m = B.ax_index_match(idx, p, max_reuse=len(p) - 1)
        assert m == expect[name], name
        got = dm.extend(got_kv, p[m:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
        ref = O.forward(sh, w, p, okv(sh))[m:]
        check_logits(sh, got, ref, f"prompt '{name}' reusing {m} of {len(p)} tokens")
        B.ax_kv_free(got_kv)
    # a prompt that IS a cached sequence keeps one token to run
    got_kv, m = B.ax_index_match(idx, cached, max_reuse=len(cached) - 1)
    assert m == len(cached) - 1
    B.ax_kv_free(got_kv)
    B.ax_index_destroy(idx)
    free, total, live = B.ax_pool_stats(dm.pool)
    assert free == total and live == 0
    dm.close()
