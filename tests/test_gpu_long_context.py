"""GPU vs the CPU oracle over very long cached prefixes (50 000 - 100 000 tokens), without paying for a
prefill of that length on the CPU: the prefix's K and V are drawn at random, written as a KV image in the
documented format (64-byte header, blocks in logical order, per block [layer][K|V][kv head] planes, a K plane
[slot][hd], a V plane [hd][slot]) by a writer of this file's own, loaded with ax_kv_import, and handed to the
oracle's cache as the same fp16 values.  What follows - an extend of the uncached suffix, verify rounds, a
rollback - runs over that cache on both sides (paper Sec. 2.3 / 4.2: a stored prefix is loaded and only the
suffix is computed; Sec. 5.5 measures the cost of attending to a long cached prefix).  This reaches what short
prefixes cannot: block tables of thousands of entries read in several pieces per key slice, key slices of
more than 1024 keys, rotary angles at positions near 100 000."""
import struct

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


def write_image(K, V, hd):
    """K, V: fp16 [layer][token, kv_head, hd] -> image bytes (uint8)."""
    L, n_tok, Hkv = len(K), K[0].shape[0], K[0].shape[1]
    nb = (n_tok + 15) // 16
    body = np.zeros((nb, L, 2, Hkv, 16 * hd), np.float16)
    for l in range(L):
        k = np.zeros((nb * 16, Hkv, hd), np.float16)
        v = np.zeros((nb * 16, Hkv, hd), np.float16)
        k[:n_tok], v[:n_tok] = K[l], V[l]
        body[:, l, 0] = k.reshape(nb, 16, Hkv, hd).transpose(0, 2, 1, 3).reshape(nb, Hkv, 16 * hd)
        body[:, l, 1] = v.reshape(nb, 16, Hkv, hd).transpose(0, 2, 3, 1).reshape(nb, Hkv, 16 * hd)
    payload = body.nbytes
    header = struct.pack("<IIiiiiiiqq", int.from_bytes(b"AXKV", "little"), 1, L, Hkv, hd, 1, 16, 0, n_tok, payload)
    return np.concatenate([np.frombuffer(header.ljust(64, b"\0"), np.uint8), body.reshape(-1).view(np.uint8)])


@pytest.mark.parametrize("name,P,T", [("hd64", 100000, 64), ("hd128", 50003, 40), ("hd64-long-extend", 40000, 300)])
def test_extend_and_verify_over_a_long_imported_prefix(B, name, P, T):
    import torch
    if name.startswith("hd64"):
        sh = I.DecoderShape(name, 2, 256, 8, 2, 64, 512, 1024, "bf16")
    else:
        sh = I.DecoderShape(name, 2, 384, 12, 4, 128, 768, 1024, "bf16")
    w = I.make_weights(sh, 6100)
    rng = np.random.default_rng(6100)
    K = [(rng.standard_normal((P, sh.n_kv_heads, sh.head_dim)) * 0.5).astype(np.float16) for _ in range(sh.n_layers)]
    V = [(rng.standard_normal((P, sh.n_kv_heads, sh.head_dim)) * 0.5).astype(np.float16) for _ in range(sh.n_layers)]
    ref_kv = O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    ref_kv.K = [k.astype(np.float64) for k in K]
    ref_kv.V = [v.astype(np.float64) for v in V]
    dm = B.DeviceModel(sh, w, max_pos=P + T + 256, max_tokens=max(T, 64), pool_tokens=P + T + 512)
    img = torch.from_numpy(write_image(K, V, sh.head_dim)).pin_memory()
    assert img.numel() == B.ax_kv_image_bytes(dm.pool, P)
    kv = dm.import_kv(img)
    assert B.ax_kv_len(kv) == P
    print(f"{name}: {P} cached tokens imported ({img.numel() / 2**20:.0f} MiB image, {len(B.ax_kv_blocks(kv))} blocks)", flush=True)

    toks = I.templated_prompt(sh.vocab, 6100, T + 8)
    got = dm.extend(kv, toks[:T], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    ref = O.forward(sh, w, toks[:T], ref_kv)
    err = float(np.abs(got - ref).max())
    print(f"{name}: extend of {T} rows over {P} keys: max-abs logit error {err:.2e} (limit {TOL:.0e}), logit std {ref.std():.3f}", flush=True)
    assert err <= TOL

    pending = O.argmax_lowest(ref[-1])
    exempt = 0
    for r, k in enumerate((8, 16, 1)):
        Pn = len(ref_kv)
        greedy = O.greedy_decode(sh, w, ref_kv.fork(), pending, k)
        drafts = I.seeded_accept_drafts(np.array(greedy[:k]), sh.vocab, 6100, r, k)[0]
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
    # rollback to the imported prefix, then the same suffix again: the same logits
    B.ax_kv_truncate(kv, P)
    again = dm.extend(kv, toks[:T], B.AX_OUT_ALL_LOGITS).cpu().numpy()
    assert np.array_equal(again, got)
    B.ax_kv_free(kv)
    dm.close()
