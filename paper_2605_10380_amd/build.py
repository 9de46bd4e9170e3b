"""Builds libagentx.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2605_10380_amd.build [--force]

Objects go to paper_2605_10380_amd/_build/, the library next to this file.  hipcc
cross-compiles without a GPU.  Packed-fp32 instruction selection is switched off for all
device code (a requirement of the target machines).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libagentx.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Per-file extras.  Attention: keep the MFMA accumulators in ordinary vector registers; the score
# tile and the output accumulators are read and rescaled by vector instructions on every key
# step, and with accumulation registers each such access costs an extra move (about a third of
# the instructions of the key-step loop).
EXTRA_FLAGS = {"k_attn.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


# `python -m paper_2605_10380_amd.build --tuning` compiles the dispatch thresholds as environment-overridable
# knobs (kernel tuning sessions only; the product build has them as constants)
TUNING_FLAGS = []


def sources():
    """HIP sources (kernels, GPU half of the ABI) and plain C++ sources (host-only half of the ABI)."""
    return sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def _newest_header():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(HERE, "..", "include", "agentx.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    spath = os.path.join(CSRC, src)
    if (not force and os.path.exists(obj)
            and os.path.getmtime(obj) > max(os.path.getmtime(spath), _newest_header())):
        return obj
    if src.endswith(".cpp"):        # no device code: host compiler flags only
        cmd = [HIPCC, "-O2", "-std=c++17", "-fPIC", "-Wall", "-c", spath, "-o", obj]
    else:
        cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), *TUNING_FLAGS, "-c", spath, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), sources()))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    if "--tuning" in sys.argv:
        TUNING_FLAGS.append("-DAX_TUNING_KNOBS")
    print(build(force="--force" in sys.argv or "--tuning" in sys.argv))
