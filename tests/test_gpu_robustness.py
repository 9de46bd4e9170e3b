"""GPU: preconditions the library must not have, and the range its 16-bit activations cover -
each against the CPU oracle through the C ABI."""
import numpy as np
import pytest

from oracle import decoder as O
from paper_2605_10380_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_10380_amd import binding
    return binding


def okv(sh):
    return O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)


def test_one_long_extend_among_many_short_sequences(B):
    """A call whose longest sequence runs on 4-tile attention blocks pads every sequence of the call
    to whole blocks: 80 two-row sequences beside one of 96 rows need 83 groups x 4 tiles x 8 KV heads
    = 2 656 partial records, more than the 2 048 a workspace once held.  Every sequence's last-row
    logits against the oracle, and the buffers next to the partial records (K-slice slabs, logits)
    unharmed: a second, ordinary call still matches."""
    sh = I.DecoderShape("heads8", 2, 256, 32, 8, 64, 512, 1024, "bf16")
    w = I.make_weights(sh, 23)
    n_short, T_long, T_short = 80, 96, 2
    dm = B.DeviceModel(sh, w, max_pos=256, max_tokens=T_long + n_short * T_short, pool_tokens=16 * 4 * (n_short + 2) + 256,
                       max_seqs=n_short + 1)
    kvs, refs, news = [], [], []
    for s in range(n_short + 1):
        kv, ref = dm.new_kv(), okv(sh)
        P = 5 + (s * 7) % 40
        hist = I.zipf_tokens(sh.vocab, 23, f"h{s}", P)
        dm.extend(kv, hist)
        O.forward(sh, w, hist, ref, rows=[-1])
        kvs.append(kv)
        refs.append(ref)
        news.append(I.zipf_tokens(sh.vocab, 23, f"n{s}", T_long if s == 40 else T_short))   # the long one sits in the middle
    got = dm.extend_batch(kvs, news, B.AX_OUT_LAST_LOGITS).cpu().numpy()
    worst = 0.0
    for s in range(n_short + 1):
        ref = O.forward(sh, w, news[s], refs[s], rows=[-1])
        worst = max(worst, float(np.abs(got[s] - ref[0]).max()))
        assert B.ax_kv_len(kvs[s]) == len(refs[s])
    print(f"81 sequences (one of 96 rows): max-abs logit error {worst:.3e}")
    assert worst <= TOL["bf16"]
    more = I.zipf_tokens(sh.vocab, 23, "more", 70)
    got = dm.extend(kvs[3], more, B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert np.abs(got - O.forward(sh, w, more, refs[3])).max() <= TOL["bf16"]
    for kv in kvs:
        B.ax_kv_free(kv)
    dm.close()


@pytest.mark.parametrize("which", ["bf16-hd64", "bf16-hd128", "f32"])
def test_pool_memory_may_hold_anything(B, which):
    """The pool is created over memory filled with 0xFF bytes (every 16-bit and 32-bit slot a NaN).
    Slots past the end of a sequence must never reach a result: extends of ragged lengths (one
    wavefront per tile and 4-tile blocks), verify rounds with rollback (rejected rows leave stale
    slots behind) and a fork with copy on write, all against the oracle."""
    sh = {"bf16-hd64": I.DecoderShape("s64", 3, 512, 8, 2, 64, 1024, 2048, "bf16"),
          "bf16-hd128": I.DecoderShape("s128", 2, 384, 6, 2, 128, 768, 1024, "bf16"),
          "f32": I.DecoderShape("f32s", 2, 96, 6, 3, 32, 200, 301, "f32")}[which]
    w = I.make_weights(sh, 29)
    toks = I.templated_prompt(sh.vocab, 29, 400)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=256, pool_tokens=2048, pool_fill=0xFF)
    kv, ref = dm.new_kv(), okv(sh)
    at = 0
    for T in (37, 1, 150, 9):                               # ends inside blocks; 150 rows: 4-tile blocks (bf16)
        got = dm.extend(kv, toks[at:at + T], B.AX_OUT_ALL_LOGITS).cpu().numpy()
        refl = O.forward(sh, w, toks[at:at + T], ref)
        assert np.isfinite(got).all(), f"T={T}"
        assert np.abs(got - refl).max() <= TOL[sh.dtype], f"T={T}"
        at += T
    pending = int(toks[at])
    for r in range(4):                                      # all drafts wrong: 1 row kept, k rows left stale
        drafts = [(int(t) + 1) % sh.vocab for t in toks[at + 1:at + 1 + 6]]
        a_ref, nxt_ref, lg = O.verify(sh, w, ref, pending, drafts)
        a, nxt = dm.verify(kv, pending, drafts)
        if min(O.top2_margin(row) for row in lg[:a_ref + 1]) > 1e-2:
            assert (a, nxt) == (a_ref, nxt_ref)
        else:
            B.ax_kv_truncate(kv, len(ref))
        pending = nxt_ref
    f, fref = B.ax_kv_fork(kv, len(ref) - 3), ref.fork(len(ref) - 3)          # shared partly filled block: copied on write
    got = dm.extend(f, toks[300:320], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert np.abs(got - O.forward(sh, w, toks[300:320], fref)).max() <= TOL[sh.dtype]
    B.ax_kv_free(f)
    B.ax_kv_free(kv)
    dm.close()


@pytest.mark.parametrize("scale", [1.0e3, 1.0e4])
def test_large_residual_stream_within_the_stated_range(B, scale):
    """bf16-weight models keep fp16(x * gain) between kernels, so the residual stream times the norm
    gain must stay below 65 504 (stated in the header).  Embeddings scaled so that |x| reaches ~1e3
    and ~1e4 (a real model's outlier channels) must still meet the tolerance; beyond the range the
    result is not finite - checked here so that the clause in the header stays true."""
    sh = I.DecoderShape("s64", 4, 512, 8, 2, 64, 1024, 2048, "bf16")
    w = I.make_weights(sh, 31)
    emb = I.bf16_bits_to_f32(w["tok_emb"])
    # a few outlier channels carry the large values, as in trained models; the rest stay O(0.02)
    big = np.zeros(sh.d_model, dtype=np.float32)
    big[[3, 100, 257, 500]] = scale / 0.02 / 4.0           # |E| ~ 0.02 * this ~ scale / 4 .. scale
    w["tok_emb"] = I.f32_to_bf16_bits(emb * (1.0 + big)[None, :])
    toks = I.templated_prompt(sh.vocab, 31, 120)
    dm = B.DeviceModel(sh, w, max_pos=256, max_tokens=128, pool_tokens=512)
    kv, ref = dm.new_kv(), okv(sh)
    trace = {}
    got = dm.extend(kv, toks[:90], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    refl = O.forward(sh, w, toks[:90], ref, trace=trace)
    peak = float(np.abs(trace["x"]).max())
    err = float(np.abs(got - refl).max())
    print(f"residual stream peak {peak:.3g}: max-abs logit error {err:.3e}, logit std {refl.std():.3f}")
    assert scale / 8 < peak < 65504 / 1.2
    assert np.isfinite(got).all() and err <= TOL["bf16"]
    a_ref, nxt_ref, lg = O.verify(sh, w, ref, int(toks[90]), toks[91:95])
    a, nxt = dm.verify(kv, int(toks[90]), toks[91:95])
    if min(O.top2_margin(row) for row in lg[:a_ref + 1]) > 1e-2:
        assert (a, nxt) == (a_ref, nxt_ref)
    B.ax_kv_free(kv)
    dm.close()


SPLIT_SHAPES = {
    "hd64-g4": I.DecoderShape("s64", 4, 512, 8, 2, 64, 1024, 2048, "bf16"),
    "hd128-g3": I.DecoderShape("s128", 3, 384, 6, 2, 128, 768, 1024, "bf16"),
    "wide": I.DecoderShape("wide", 2, 1024, 16, 4, 64, 4096, 4096, "bf16"),
}


@pytest.mark.parametrize("which", list(SPLIT_SHAPES))
def test_split_activations_every_kernel_family(B, which):
    """ax_model_config.act_split = 1: activations between kernels as hi + lo fp16 pairs.  Row counts
    chosen so that every GEMM family (few-row, LDS tiles with and without K slices, streaming blocks)
    and both attention kernels run with two-part operands, one sequence and several; against the
    oracle, and against the same calls on a model without the split: the split must not be worse,
    and over the run its worst error must be clearly smaller."""
    sh = SPLIT_SHAPES[which]
    w = I.make_weights(sh, 37)
    toks = I.templated_prompt(sh.vocab, 37, 1500)
    worst = {}
    for mode in (-1, 1):
        dm = B.DeviceModel(sh, w, max_pos=2048, max_tokens=640, pool_tokens=8192, max_seqs=4, act_split=mode)
        kv, ref = dm.new_kv(), okv(sh)
        errs, at = [], 0
        for T in (9, 1, 40, 17, 150, 300, 600, 64, 130):
            got = dm.extend(kv, toks[at:at + T], B.AX_OUT_ALL_LOGITS).cpu().numpy()
            errs.append(float(np.abs(got - O.forward(sh, w, toks[at:at + T], ref)).max()))
            at += T
        # verify rounds (graph replays), partly accepted
        pending = int(toks[at])
        for r in range(3):
            greedy = O.greedy_decode(sh, w, ref.fork(), pending, 6)
            drafts = greedy[:3] + [(greedy[3] + 1) % sh.vocab] + greedy[4:]
            a_ref, nxt_ref, lg = O.verify(sh, w, ref, pending, drafts)
            a, nxt = dm.verify(kv, pending, drafts)
            if min(O.top2_margin(row) for row in lg[:a_ref + 1]) > 1e-2:
                assert (a, nxt) == (a_ref, nxt_ref) == (3, greedy[3])
            else:
                B.ax_kv_truncate(kv, len(ref))
            pending = nxt_ref
        # several sequences in one pass, forked from the long one (shared prefix)
        kvs = [B.ax_kv_fork(kv, len(ref) - 5 * s) for s in range(3)]
        refs = [ref.fork(len(ref) - 5 * s) for s in range(3)]
        news = [toks[1400 + 10 * s:1400 + 10 * s + t] for s, t in enumerate((33, 9, 70))]
        got = dm.extend_batch(kvs, news, B.AX_OUT_ALL_LOGITS).cpu().numpy()
        row = 0
        for s in range(3):
            errs.append(float(np.abs(got[row:row + len(news[s])] - O.forward(sh, w, news[s], refs[s])).max()))
            row += len(news[s])
        for k_ in kvs + [kv]:
            B.ax_kv_free(k_)
        dm.close()
        worst[mode] = errs
        print(f"{which} act_split={mode}: max-abs logit error per call", " ".join(f"{e:.2e}" for e in errs))
    assert max(worst[1]) <= TOL["bf16"]
    assert all(s_ <= u * 1.25 + 1e-4 for s_, u in zip(worst[1], worst[-1]))
    assert max(worst[1]) < 0.7 * max(worst[-1])


def test_weights_outside_fp16_range_are_refused(B):
    """bf16 weights are multiplied as fp16: a matrix entry that is not finite in fp16 (here 1e5, and
    a NaN) must make ax_model_create fail with AX_ERR_UNSUPPORTED instead of producing infinities."""
    sh = I.DecoderShape("s64", 2, 256, 4, 2, 64, 512, 512, "bf16")
    for name, layer, value in (("w_down", 1, 1.0e5), ("lm_head", None, float("nan"))):
        w = I.make_weights(sh, 33)
        t = w[name] if layer is None else w[name][layer]
        t[3, 5] = I.f32_to_bf16_bits(np.array([value], dtype=np.float32))[0]
        with pytest.raises(B.AxError) as e:
            B.DeviceModel(sh, w, max_pos=64, max_tokens=16, pool_tokens=64)
        assert e.value.status == B.AX_ERR_UNSUPPORTED, name
    w = I.make_weights(sh, 33)
    w["wo"][0][1, 1] = I.f32_to_bf16_bits(np.array([6.0e4], dtype=np.float32))[0]      # large but representable
    dm = B.DeviceModel(sh, w, max_pos=64, max_tokens=16, pool_tokens=64)
    dm.close()


def test_workspace_guards_notice_a_write_past_a_region(B):
    """Every workspace region is followed by 256 guard bytes (DeviceModel.close checks them after every test that
    closes its model).  The check itself: intact after ordinary calls; a single byte written just behind the first
    region (the rotary cosine table, max_pos * head_dim / 2 floats rounded up to 256 bytes) or into the very last
    guard (the end of the workspace) is reported with the region's index; restored, the check passes again."""
    sh = I.DecoderShape("g", 2, 256, 8, 2, 64, 512, 512, "bf16")
    w = I.make_weights(sh, 77)
    dm = B.DeviceModel(sh, w, max_pos=300, max_tokens=64, pool_tokens=512)
    kv = dm.new_kv()
    dm.extend(kv, I.templated_prompt(sh.vocab, 77, 60))
    dm.verify(kv, 5, [1, 2, 3])
    assert B.ax_dbg_check_guards(dm.model) == -1
    first = -(-(300 * 32 * 4) // 256) * 256
    assert bytes(dm.ws[first:first + 256].cpu().numpy()) == b"\xa5" * 256
    dm.ws[first + 17] = 0
    assert B.ax_dbg_check_guards(dm.model) == 0
    dm.ws[first + 17] = 0xA5
    assert B.ax_dbg_check_guards(dm.model) == -1
    assert bytes(dm.ws[-256:].cpu().numpy()) == b"\xa5" * 256
    dm.ws[-1] = 1
    assert B.ax_dbg_check_guards(dm.model) == len(B.WORKSPACE_REGIONS) - 1
    dm.ws[-1] = 0xA5
    B.ax_kv_free(kv)
    dm.close()
