"""Host logic of bench.py that needs no GPU: the refusal of more than one GPU, the algorithmic bytes /
flops its roofline fractions divide by (checked against figures worked out by hand from the ~1B shape),
and the parsing of the committed profile tables it quotes."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and not r.stdout.strip()


def test_algorithmic_bytes_and_flops_of_the_headline_workload():
    import bench
    from paper_2605_10380_amd import inputs as I
    wl = I.WORKLOADS[2]
    sh = wl.shape
    assert (sh.n_layers, sh.d_model, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.d_ff, sh.vocab) == (16, 2048, 32, 8, 64, 8192, 128256)
    assert (wl.P, wl.T, wl.k) == (4096, 256, 8)
    alg = bench.algorithmic(sh, wl.P, wl.T, wl.k)
    # SwiGLU gate/up: two [8192, 2048] bf16 matrices + the rows in (fp16) + the rows out (fp16)
    assert alg["verify"]["swiglu_gate_up"]["bytes"] == 67108864 + 9 * 2048 * 2 + 9 * 8192 * 2 == 67293184
    assert alg["extend"]["swiglu_gate_up"]["bytes"] == 67108864 + 256 * 2048 * 2 + 256 * 8192 * 2 == 72351744
    assert alg["extend"]["swiglu_gate_up"]["flops"] == 4 * 256 * 8192 * 2048 == 17179869184
    # QKV: [(32 + 16) * 64, 2048]
    assert alg["verify"]["qkv_proj"]["bytes"] == 3072 * 2048 * 2 + 9 * 2048 * 2 + 9 * 3072 * 4
    # K and V of every cached position of one layer: (P + T) * 2 * 8 heads * 64 * 2 B, plus q in and out rows
    assert alg["verify"]["attention"]["bytes"] == 4352 * 2 * 8 * 64 * 2 + 2 * 9 * 2048 * 2
    # causal extend: row i of T sees P + i + 1 keys -> T * (P + (T + 1) / 2) scores, 4 flops per score and channel
    assert alg["extend"]["attention"]["flops"] == 4.0 * 256 * (4096 + 128.5) * 64 * 32
    # whole verify step: every layer matrix and the LM head once, 32 KiB of K,V per cached token
    layer_params = 3072 * 2048 + 2048 * 2048 + 3 * 8192 * 2048
    kv_tok = 2 * 16 * 8 * 64 * 2
    assert kv_tok == 32768
    expect = 16 * layer_params * 2 + 128256 * 2048 * 2 + (4352 + 9) * kv_tok + 9 * kv_tok + 9 * 2048 * 2
    assert abs(alg["verify_bytes"] - expect) <= 16 * 2 * 2048 * 2 * 2          # the two gain vectors per layer, if counted
    assert alg["extend_flops"] == pytest.approx(2 * 256 * 16 * sh.layer_params + 2 * 128256 * 2048 + 16 * alg["extend"]["attention"]["flops"])


def test_committed_profile_tables_parse():
    import bench
    dur = bench.load_rocprof_durations(2)
    for phase in ("verify", "extend"):
        us, kernel = dur[(phase, "swiglu_gate_up")]
        assert 1.0 < us < 1000.0 and "gemm_bf16" in kernel
    traffic = bench.load_traffic(2)
    alg = bench.algorithmic(*[getattr(__import__("paper_2605_10380_amd.inputs", fromlist=["x"]).WORKLOADS[2], n) for n in ("shape", "P", "T", "k")])
    for phase in ("verify", "extend"):
        t = traffic[(phase, "swiglu_gate_up")]
        a = alg[phase]["swiglu_gate_up"]["bytes"]
        assert 0.9 * a < t < 1.5 * a, (phase, t, a)        # measured HBM traffic of the dominant kernels stays near the algorithmic bytes
