"""Build the C-ABI library (HIP, gfx950 only) in-tree: paper_2505_14708_amd/lib/libdraftattn.so, and beside it the
bench's measuring sticks as a library of their own (lib/libdaprobe.so: not part of the product)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libdraftattn.so")
PROBE_LIB_PATH = os.path.join(LIB_DIR, "libdaprobe.so")

SOURCES = ["da_api.hip", "k_permute.hip", "k_pool.hip", "k_draft.hip", "k_select.hip", "k_select_global.hip", "k_attn_f32.hip",
           "k_attn_bf16_ring.hip"]
PROBE_SOURCES = ["probe/k_probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 instructions are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", os.path.join(CSRC, "probe")]


# files whose float32 results must be reproducible bit for bit on a CPU: no contraction
STRICT_FP = {"k_pool.hip", "k_draft.hip"}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(os.path.basename(src))[0] + ".o")
    extra = ["-ffp-contract=off"] if src in STRICT_FP else []
    if src == "k_attn_bf16_ring.hip":
        # all MFMA results in ordinary vector registers: the softmax reads the scores many times and
        # a 32-query wave has the registers for it
        extra += ["-mllvm", "-amdgpu-mfma-vgpr-form"]
    if src == "k_attn_bf16_ring.hip":
        extra.append("-fno-honor-nans")   # no NaN canonicalisation around max(); infinities stay exact
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES + PROBE_SOURCES))
    for path, part in ((LIB_PATH, objs[:len(SOURCES)]), (PROBE_LIB_PATH, objs[len(SOURCES):])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", path, *part]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        if verbose:
            print("built", path)
    return LIB_PATH


if __name__ == "__main__":
    build()
