"""GPU: single kernels and per-stage intermediates against the CPU oracle (localises faults)."""
import numpy as np
import pytest

from oracle import decoder as O
from paper_2605_10380_amd import inputs as I

pytestmark = pytest.mark.gpu


def _bf16_round(x):
    return I.bf16_bits_to_f32(I.f32_to_bf16_bits(x.astype(np.float32))).astype(np.float64)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


# M values: skinny path (<= 16, and to 32 rows for some epilogues) and tile path (ragged); K / N pick
# different wavefront counts in the skinny kernel and both tile shapes; M >= 257 (and 193-256 for
# wide matrices) takes the streaming SwiGLU kernel (steady-state loop and drain, ragged rows and columns)
GEMM_CASES = [(1, 64, 64), (9, 3072, 2048), (9, 2048, 8192), (17, 512, 256), (33, 128, 1024), (64, 2064, 192),
              (65, 384, 128), (100, 200 * 16, 320), (256, 3072, 2048), (300, 1024, 512), (512, 33 * 128, 256),
              (400, 1040, 1024), (384, 2048, 576), (300, 2048, 256), (230, 14336, 128), (257, 8192, 128), (640, 8192, 192), (320, 14336, 128),
              # thousands of rows: every epilogue through the streaming kernel (ragged rows and columns, drain path)
              (1600, 7712, 192), (1664, 7680, 448),
              (144, 65600, 128), (131, 65536, 192), (17, 65600, 128), (40, 65536, 192), (100, 65568, 128), (190, 65536, 128), (300, 65600, 128),   # streaming blocks for wide outputs (logits) from 17 rows
              (144, 8192, 3072), (190, 4096, 1536), (150, 4112, 1536),  # 17-192 rows: SwiGLU over K slices (32- to 192-row blocks)
              (40, 8192, 2048), (96, 4112, 1536), (128, 4096, 3072), (17, 8192, 2048), (30, 4112, 1536)]


@pytest.mark.parametrize("M,N,K", GEMM_CASES)
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_bf16_gemm(torch_cuda, M, N, K, epi):
    torch = torch_cuda
    from paper_2605_10380_amd import binding as B
    rng = np.random.default_rng(M * 7 + N + K + epi)
    A = rng.standard_normal((M, K), dtype=np.float32).astype(np.float16)      # activations are fp16
    W = I.f32_to_bf16_bits(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    W2 = I.f32_to_bf16_bits(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    C0 = rng.standard_normal((M, N), dtype=np.float32)
    dev = lambda a: torch.from_numpy(a).view(torch.bfloat16).cuda() if a.dtype == np.uint16 else torch.from_numpy(a).cuda()
    dA, dW, dW2 = dev(A), dev(W), dev(W2)
    A64 = A.astype(np.float64)
    ref = A64 @ O.widen(W).T
    if epi == 2:
        dC = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    else:
        dC = dev(C0.copy())
    B.ax_dbg_gemm(B.AX_BF16, epi, dA.data_ptr(), dW.data_ptr(), dW2.data_ptr(), dC.data_ptr(), M, N, K)
    got = dC.float().cpu().numpy().astype(np.float64)
    scale = np.abs(ref).max()
    if epi == 0:
        assert np.abs(got - ref).max() <= 2e-5 * scale + 1e-6
    elif epi == 1:
        assert np.abs(got - (C0 + ref)).max() <= 2e-5 * scale + 1e-5
    else:
        want = O.silu(ref) * (A64 @ O.widen(W2).T)
        assert np.abs(got - want).max() <= 2 ** -11 * np.abs(want).max() + 1e-6


def _random_gemm_cases(n, seed=20260517):
    """Seeded shapes around the launcher's row-count crossovers (16/17, 32/33, 64/65, 128/129, 192/193, 256/257,
    512/513) with ragged column counts (multiples of 16) and K a multiple of 64: every (kernel, epilogue)
    pair is reached at shapes nobody picked by hand."""
    rng = np.random.default_rng(seed)
    edges = [16, 17, 32, 33, 64, 65, 128, 129, 160, 161, 192, 193, 256, 257, 384, 512, 513, 640]
    cases = []
    for i in range(n):
        M = int(rng.choice(edges)) if i % 2 == 0 else int(rng.integers(1, 700))
        N = 16 * int(rng.integers(4, 560))
        K = 64 * int(rng.integers(1, 40))
        cases.append((M, N, K, i % 3))
    return cases


@pytest.mark.parametrize("M,N,K,epi", _random_gemm_cases(36))
def test_bf16_gemm_seeded_random_shapes(torch_cuda, M, N, K, epi):
    test_bf16_gemm(torch_cuda, M, N, K, epi)


# the residual GEMM with the next norm's preparation, through every kernel that implements it:
# skinny with 8 / 12 / 16 columns per block (to 16 rows, and to 32 rows when K is short), tile kernels
# unsplit and with K slices (64- and 128-row
# blocks), streaming kernel
RESIDUAL_CASES = [(9, 2048, 512, False), (9, 3072, 256, False), (33, 4096, 192, False), (16, 1040, 128, False),
                  (24, 2048, 256, False), (24, 1024, 4096, True), (64, 1024, 128, False),
                  (100, 512, 256, False), (256, 2048, 2048, True), (256, 2048, 2048, False), (300, 1024, 4096, True),
                  (512, 4096, 4096, True), (520, 3072, 8192, True), (300, 4096, 14336, True), (1600, 7712, 192, True),
                  (1030, 5088, 8192, True),        # long K and one even round of blocks: streaming kernel
                  (144, 3072, 8192, True), (131, 2048, 8192, True), (190, 2048, 8192, True), (161, 1024, 12288, True)]   # 160- / 192-row streaming blocks, K slices


@pytest.mark.parametrize("M,N,K,split", RESIDUAL_CASES)
def test_bf16_residual_gemm_with_norm_preparation(torch_cuda, M, N, K, split):
    torch = torch_cuda
    from paper_2605_10380_amd import binding as B
    rng = np.random.default_rng(M * 3 + N + K)
    A = (rng.standard_normal((M, K), dtype=np.float32) * 0.5).astype(np.float16)
    W = I.f32_to_bf16_bits(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    gain = I.f32_to_bf16_bits(1.0 + 0.1 * rng.standard_normal(N, dtype=np.float32))
    x0 = rng.standard_normal((M, N), dtype=np.float32)
    bf = lambda a: torch.from_numpy(a).view(torch.bfloat16).cuda()
    dA, dW, dg, dx = torch.from_numpy(A).cuda(), bf(W), bf(gain), torch.from_numpy(x0.copy()).cuda()
    da16 = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    dssq = torch.full((M, N // 8), float("nan"), dtype=torch.float32, device="cuda")
    ws_bytes = 8 * M * N * 4 if split else 0
    dws = torch.empty(max(ws_bytes, 4), dtype=torch.uint8, device="cuda")
    parts = B.ax_dbg_gemm_residual(dA.data_ptr(), dW.data_ptr(), dg.data_ptr(), dx.data_ptr(), da16.data_ptr(),
                                   dssq.data_ptr(), M, N, K, dws.data_ptr() if split else 0, ws_bytes)
    assert 1 <= parts <= N // 8
    want = x0.astype(np.float64) + A.astype(np.float64) @ O.widen(W).T
    got = dx.cpu().numpy().astype(np.float64)
    assert np.abs(got - want).max() <= 2e-5 * np.abs(want).max() + 1e-5
    a16 = da16.float().cpu().numpy().astype(np.float64)
    want16 = want * O.widen(gain)[None, :]
    assert np.abs(a16 - want16).max() <= 2 ** -10 * np.abs(want16).max() + 1e-6
    ssq = dssq.cpu().numpy().reshape(-1)[:M * parts].reshape(M, parts)        # rows are `parts` apart
    assert np.isfinite(ssq).all()
    assert np.allclose(ssq.astype(np.float64).sum(axis=1), (want ** 2).sum(axis=1), rtol=2e-5)


def _random_residual_cases(n, seed=20260518):
    """Seeded shapes for the residual GEMM with norm preparation: N a multiple of 64 (K slices and the
    streaming kernels need it), long and short K, rows around the launcher's crossovers."""
    rng = np.random.default_rng(seed)
    edges = [9, 16, 17, 32, 33, 64, 128, 129, 160, 161, 192, 193, 256, 257, 512, 640]
    cases = []
    for i in range(n):
        M = int(rng.choice(edges)) if i % 2 == 0 else int(rng.integers(1, 700))
        N = 64 * int(rng.integers(2, 70))
        K = 64 * int(rng.integers(1, 40)) if i % 3 else 1024 * int(rng.integers(8, 15))
        cases.append((M, N, K, True))
    return cases


@pytest.mark.parametrize("M,N,K,split", _random_residual_cases(18))
def test_bf16_residual_gemm_seeded_random_shapes(torch_cuda, M, N, K, split):
    test_bf16_residual_gemm_with_norm_preparation(torch_cuda, M, N, K, split)


@pytest.mark.parametrize("M,N,K", [(5, 37, 19), (64, 688, 256), (70, 256, 688), (130, 4096, 256)])
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_f32_gemm(torch_cuda, M, N, K, epi):
    torch = torch_cuda
    from paper_2605_10380_amd import binding as B
    rng = np.random.default_rng(M + N + K + epi)
    A = rng.standard_normal((M, K), dtype=np.float32)
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05)
    W2 = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05)
    C0 = rng.standard_normal((M, N), dtype=np.float32)
    dA, dW, dW2, dC = (torch.from_numpy(a.copy()).cuda() for a in (A, W, W2, C0))
    B.ax_dbg_gemm(B.AX_F32, epi, dA.data_ptr(), dW.data_ptr(), dW2.data_ptr(), dC.data_ptr(), M, N, K)
    got = dC.cpu().numpy().astype(np.float64)
    ref = A.astype(np.float64) @ W.astype(np.float64).T
    want = ref if epi == 0 else C0 + ref if epi == 1 else O.silu(ref) * (A.astype(np.float64) @ W2.astype(np.float64).T)
    assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(want).max())


STAGE_SHAPES = {
    "f32": I.DecoderShape("st-f32", 1, 256, 4, 2, 64, 688, 512, "f32"),
    "bf16-hd64": I.DecoderShape("st-b64", 1, 256, 8, 2, 64, 512, 512, "bf16"),
    "bf16-hd128-g3": I.DecoderShape("st-b128", 1, 384, 6, 2, 128, 512, 512, "bf16"),
}


@pytest.mark.parametrize("which", list(STAGE_SHAPES))
@pytest.mark.parametrize("P,T", [(0, 5), (37, 9), (100, 70)])
def test_single_layer_stages(torch_cuda, which, P, T):
    """Each stage of a one-layer model against the oracle's intermediates: pre-rotary qkv,
    rotated q, attention output, SwiGLU activations, residual stream, normed LM-head input."""
    from paper_2605_10380_amd import binding as B
    sh = STAGE_SHAPES[which]
    w = I.make_weights(sh, 5)
    toks = I.templated_prompt(sh.vocab, 5, P + T)
    dm = B.DeviceModel(sh, w, max_pos=512, max_tokens=128, pool_tokens=1024)
    kv = dm.new_kv()
    if P:
        dm.extend(kv, toks[:P])
    logits = dm.extend(kv, toks[P:], B.AX_OUT_ALL_LOGITS).cpu().numpy().astype(np.float64)
    okv = O.KVCache(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    if P:
        O.forward(sh, w, toks[:P], okv)
    tr = {}
    ref = O.forward(sh, w, toks[P:], okv, trace=tr)
    bf = sh.dtype == "bf16"
    Hq, hd = sh.n_q_heads, sh.head_dim

    def read(which_buf, cols, act):
        if act and bf:
            a = np.zeros((T, cols), dtype=np.float16)
            B.ax_dbg_read(dm.model, which_buf, a)
            return a.astype(np.float64)
        a = np.zeros((T, cols), dtype=np.float32)
        B.ax_dbg_read(dm.model, which_buf, a)
        return a.astype(np.float64)

    tol = 4e-3 if bf else 2e-5      # relative to the stage's largest magnitude
    stages = [("q", read(2, Hq * hd, True), tr["q"].reshape(T, -1)),
              ("attn", read(3, Hq * hd, True), tr["attn"].reshape(T, -1)),
              ("ffn", read(4, sh.d_ff, True), tr["ffn"]),
              ("x", read(0, sh.d_model, False), tr["x"]),
              ("logits", logits, ref)]
    if bf:      # the norm's division happens inside the consuming GEMM: buffer 5 is x * gain
        stages.append(("x*gain", read(5, sh.d_model, True), tr["x"] * O.widen(w["final_norm"])))
    else:
        stages += [("qkv", read(1, sh.qkv_rows, False), tr["qkv"]),
                   ("h_out", read(5, sh.d_model, True), tr["h_out"])]
    errs = {name: float(np.abs(g - r).max() / np.abs(r).max()) for name, g, r in stages}
    print(which, P, T, {k: f"{v:.2e}" for k, v in errs.items()})
    for name, e in errs.items():
        assert e <= tol, (name, errs)
    dm.close()


def test_measured_peaks_probe(torch_cuda):
    """The machine-rate probes leave their buffer's first half untouched (the read-only stream writes
    nothing, the copy kernel fills the second half with the first) and report rates that a working
    MI355X-class device delivers and that do not exceed the nominal peaks."""
    torch = torch_cuda
    from paper_2605_10380_amd import binding as B
    n = 256 << 20
    buf = torch.arange(n // 4, dtype=torch.int32, device="cuda")
    before = buf[: n // 8].clone()
    torch.cuda.synchronize()
    read_gbs, copy_gbs, mfma_tf = B.ax_dbg_peaks(buf.data_ptr(), n, 3)
    assert torch.equal(buf[: n // 8], before) and torch.equal(buf[n // 8:], before)
    assert 1000.0 < read_gbs <= 8000.0 and 1000.0 < copy_gbs <= 8000.0
    assert 500.0 < mfma_tf <= 2520.0
    with pytest.raises(B.AxError):
        B.ax_dbg_peaks(buf.data_ptr(), 48, 3)


def test_phase_order_probe(torch_cuda):
    """Kernel boundary against in-kernel barrier: both times are positive and finite, the barrier kernel
    crosses all its rounds (a workgroup that gave up would come back as an error), bytes of the buffer
    past the first 4096 are untouched, and bad shapes are refused."""
    torch = torch_cuda
    from paper_2605_10380_amd import binding as B
    buf = torch.full((2048,), 7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    for blocks in (8, 64, 256):
        boundary_us, barrier_us = B.ax_dbg_phase_order(buf.data_ptr(), buf.numel() * 4, blocks, 50)
        print(f"{blocks} workgroups: {boundary_us:.2f} us per kernel boundary, {barrier_us:.2f} us per grid barrier", flush=True)
        assert 0.0 < boundary_us < 1000.0 and 0.0 < barrier_us < 1000.0
    assert bool((buf[1024:] == 7).all())
    for bad in (0, 12, 264):
        with pytest.raises(B.AxError):
            B.ax_dbg_phase_order(buf.data_ptr(), buf.numel() * 4, bad, 50)


def test_cu_fill_probe(torch_cuda):
    """What one compute unit pulls out of L2 and out of HBM: rates that a working device delivers, L2 above HBM, the
    chip-wide memory figure (256 x per-CU) of the order of the nominal 8 TB/s; the buffer is only read; bad sizes are refused."""
    torch = torch_cuda
    from paper_2605_10380_amd import binding as B
    n = 256 << 20
    buf = torch.arange(n // 4, dtype=torch.int32, device="cuda")
    ref = buf.clone()
    torch.cuda.synchronize()
    l2, hbm = B.ax_dbg_cu_fill(buf.data_ptr(), n)
    print(f"one compute unit pulls {l2:.1f} GB/s from L2, {hbm:.1f} GB/s from HBM (x 256 = {hbm * 256 / 1e3:.2f} TB/s)", flush=True)
    assert torch.equal(buf, ref)
    assert 10.0 < hbm < l2 < 400.0 and hbm * 256 <= 12000.0      # (a 256 MiB buffer may sit in the memory-side cache)
    for bad in (n - 16, 1 << 20):
        with pytest.raises(B.AxError):
            B.ax_dbg_cu_fill(buf.data_ptr(), bad)
