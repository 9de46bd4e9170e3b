"""GPU vs the CPU oracle at the sizes the workload configurations name, element by element.

  * the ~3B width (two layers) at its own P = 6144 with T in {64, 256, 1024} - every logit of every
    row - and verify rounds at k in {1, 4, 16};
  * the ~8B width (two layers) at its own P = 8192, T = 512 and verify rounds at k = 8;
  * both decoders at FULL depth (28 / 32 layers) over a 1024-token prefix: extend of 128 rows, every
    logit, then verify rounds at k = 8.

Weights are drawn on the device (torch generator, the distribution of inputs.make_weights) and the
same bits are handed to the oracle, as bench.py does: the host-side Philox draw of 3-8 G parameters
would take longer than the comparison.  Extend over a cached prefix must equal the plain computation
(paper Sec. 2.3, prefix caching), verification must accept exactly what greedy decoding would emit
(Sec. 2.3, speculative decoding; Sec. 4.3).  Tolerances as everywhere: 2e-2 max-abs over all logits,
exact accepted length / next token wherever the oracle's top-2 margin exceeds 1e-2.
"""
import time

import numpy as np
import pytest

from oracle import decoder as O
from paper_2605_10380_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL = 2e-2
MARGIN = 1e-2


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_10380_amd import binding
    return binding


def device_and_host_weights(sh, seed):
    import torch
    from bench import torch_weights, to_numpy_storage
    w_dev = torch_weights(torch, sh, seed, torch.device("cuda:0"))
    w_host = {k: ([to_numpy_storage(torch, t) for t in v] if isinstance(v, list) else to_numpy_storage(torch, v))
              for k, v in w_dev.items()}
    return w_dev, w_host


def okv(sh):
    return O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)


def build_prefix(dm, kv, ref_kv, sh, w, prompt, P, piece):
    for at in range(0, P, 512):
        dm.extend(kv, prompt[at:min(at + 512, P)])
    t0 = time.perf_counter()
    for at in range(0, P, piece):                          # in pieces: bounded memory, and a progress line per piece
        O.forward(sh, w, prompt[at:min(at + piece, P)], ref_kv, rows=[-1])
        print(f"  oracle prefix {min(at + piece, P)}/{P} ({time.perf_counter() - t0:.0f} s)", flush=True)


def check(got, ref, what):
    err = float(np.abs(got.astype(np.float64) - ref).max())
    print(f"{what}: max-abs logit error {err:.3e} (limit {TOL:.0e}), logit std {ref.std():.3f}", flush=True)
    assert err <= TOL, what
    return err


def verify_rounds(B, dm, sh, w, kv, ref_kv, pending, k, rounds, seed, prompt, seeded=True):
    """Rounds alternate prompt-copied drafts (nearly always all rejected) and drafts whose first j
    tokens are the oracle's greedy continuation (partial acceptance, j seeded).  Returns the
    accepted counts and the number of exempt rounds (oracle margin <= 1e-2 at the deciding row)."""
    hist, exempt = [], 0
    for r in range(rounds):
        P = len(ref_kv)
        assert B.ax_kv_len(kv) == P
        if r % 2 == 0 or not seeded:
            drafts = I.prompt_copied_drafts(prompt, seed, r, k)
        else:
            greedy = O.greedy_decode(sh, w, ref_kv.fork(), pending, k) if k else []
            drafts = I.seeded_accept_drafts(np.array(greedy[:k]), sh.vocab, seed, r, k)[0] if k else np.zeros(0, np.int32)
        a_ref, nxt_ref, logits = O.verify(sh, w, ref_kv, pending, drafts)
        a, nxt = dm.verify(kv, pending, drafts)
        assert B.ax_kv_len(kv) == P + 1 + a
        if (a, nxt) != (a_ref, nxt_ref):
            assert O.top2_margin(logits[min(a, a_ref)]) <= MARGIN, (r, a, a_ref, nxt, nxt_ref)
            exempt += 1
            if a > a_ref:
                B.ax_kv_truncate(kv, P + 1 + a_ref)
            elif a < a_ref:
                dm.extend(kv, np.asarray(drafts[a:a_ref], dtype=np.int32))
        pending = nxt_ref
        hist.append(a_ref)
    return hist, exempt, pending


def test_3b_width_at_its_own_P_and_T(B):
    """~3B width, two layers, P = 6144: extends of T = 64 / 256 / 1024 (every logit of every row; the
    three lengths run the few-row tiles, the 128-row tiles with K slices and the streaming kernels
    with 8-tile attention blocks) and verify rounds at k = 1, 4, 16 (2, 5 and 17 rows)."""
    sh = I.SHAPES["3b"].with_layers(2)
    P = 6144
    w_dev, w = device_and_host_weights(sh, 3000)
    prompt = I.templated_prompt(sh.vocab, 3000, P + 1024)
    dm = B.DeviceModel(sh, w_dev, max_pos=P + 1024 + 256, max_tokens=1024, pool_tokens=P + 1024 + 512)
    kv, ref_kv = dm.new_kv(), okv(sh)
    build_prefix(dm, kv, ref_kv, sh, w, prompt, P, 2048)
    last_ref = None
    for T in (64, 256, 1024):
        got = dm.extend(kv, prompt[P:P + T], B.AX_OUT_ALL_LOGITS).cpu().numpy()
        ref = O.forward(sh, w, prompt[P:P + T], ref_kv)
        check(got, ref, f"3b width, L=2, P={P}, extend T={T}")
        last_ref = ref[-1].copy()
        del got, ref
        if T != 1024:
            B.ax_kv_truncate(kv, P)
            ref_kv.truncate(P)
    pending = O.argmax_lowest(last_ref)
    for k in (1, 4, 16):
        hist, exempt, pending = verify_rounds(B, dm, sh, w, kv, ref_kv, pending, k, 4, 3000 + k, prompt)
        print(f"3b width verify k={k}: accepted {hist}, exempt {exempt}", flush=True)
        assert exempt <= 1
    B.ax_kv_free(kv)
    dm.close()
    O.clear_widen_cache()


def test_8b_width_at_its_own_P_and_T(B):
    """~8B width, two layers, P = 8192, extend T = 512 (every logit), verify rounds at k = 8.  The
    full-depth ~8B model keeps its activations as hi + lo pairs (ax_model_config.act_split, automatic
    for deep wide models); the two-layer cut is created with that mode on, so that it launches what
    the full model launches."""
    sh = I.SHAPES["8b"].with_layers(2)
    P, T, k = 8192, 512, 8
    w_dev, w = device_and_host_weights(sh, 4000)
    prompt = I.templated_prompt(sh.vocab, 4000, P + T)
    dm = B.DeviceModel(sh, w_dev, max_pos=P + T + 256, max_tokens=512, pool_tokens=P + T + 512, act_split=1)
    kv, ref_kv = dm.new_kv(), okv(sh)
    build_prefix(dm, kv, ref_kv, sh, w, prompt, P, 2048)
    got = dm.extend(kv, prompt[P:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, prompt[P:], ref_kv)
    check(got, ref, f"8b width, L=2, P={P}, extend T={T}, split activations")
    pending = O.argmax_lowest(ref[-1])
    del got, ref
    hist, exempt, _ = verify_rounds(B, dm, sh, w, kv, ref_kv, pending, k, 4, 4000, prompt)
    print(f"8b width verify k={k}: accepted {hist}, exempt {exempt}", flush=True)
    assert exempt <= 1
    B.ax_kv_free(kv)
    dm.close()
    O.clear_widen_cache()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,P", [("3b", 1024), ("8b", 1024)])
def test_full_depth_extend_and_verify(B, name, P, monkeypatch):
    """All 28 / 32 layers of the ~3B / ~8B decoder: prefix P built in chunks of 512, extend of
    T = 128 compared on every logit of every row, then verify rounds at k = 8."""
    import psutil
    sh = I.SHAPES[name]
    T, k = 128, 8
    # float64 copies of every matrix (26 / 60 GB): kept across the oracle's calls where the host has the memory
    f64_bytes = (sh.n_layers * sh.layer_params + 2 * sh.vocab * sh.d_model) * 8
    cached = f64_bytes <= O.WIDE_CACHE_LIMIT
    if not cached and psutil.virtual_memory().available > 2 * f64_bytes + (32 << 30):
        monkeypatch.setattr(O, "WIDE_CACHE_LIMIT", f64_bytes + (1 << 30))
        cached = True
    w_dev, w = device_and_host_weights(sh, 5000)
    prompt = I.templated_prompt(sh.vocab, 5000, P + T)
    dm = B.DeviceModel(sh, w_dev, max_pos=P + T + 256, max_tokens=512, pool_tokens=P + T + 512)
    kv, ref_kv = dm.new_kv(), okv(sh)
    build_prefix(dm, kv, ref_kv, sh, w, prompt, P, 256)
    got = dm.extend(kv, prompt[P:], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, prompt[P:], ref_kv)
    check(got, ref, f"{name} at full depth ({sh.n_layers} layers), P={P}, extend T={T}")
    pending = O.argmax_lowest(ref[-1])
    # the round with greedy-seeded drafts costs k more oracle forwards: only where the float64 weights stay cached
    hist, exempt, _ = verify_rounds(B, dm, sh, w, kv, ref_kv, pending, k, 2, 5000, prompt, seeded=cached)
    print(f"{name} full depth verify k={k}: accepted {hist}, exempt {exempt}", flush=True)
    assert exempt <= 1
    B.ax_kv_free(kv)
    dm.close()
    O.clear_widen_cache()
