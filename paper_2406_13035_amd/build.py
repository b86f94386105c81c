"""Builds libd2o.so (HIP, gfx950) in-tree next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["d2o_host.hip", "prefill_f32.hip", "prefill_bf16.hip", "tokens.hip", "decode.hip", "decode_split.hip", "append.hip", "qkv.hip", "fp8.hip"]
LIB = os.environ.get("D2O_LIB", os.path.join(HERE, "libd2o.so"))
# Matrix-core results straight into vector registers: the kernels of these files post-process
# every accumulator element on the vector ALU, and a copy out of the accumulation registers per
# element is a sizeable part of their instruction count.
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
EXTRA_FLAGS = {"tokens.hip": VGPR_FORM}


def build(verbose: bool = False) -> str:
    """Compiles every source (in parallel, one hipcc per file) and links libd2o.so."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
             "-Wno-unused-value"] + os.environ.get("D2O_EXTRA_FLAGS", "").split()

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        res = subprocess.run([hipcc, "-c"] + flags + EXTRA_FLAGS.get(src, []) + ["-o", obj, os.path.join(HERE, "csrc", src)],
                             capture_output=True, text=True)
        return src, obj, res

    msgs = []
    objs = []
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), int(os.environ.get("MAX_JOBS", "8")))) as ex:
        for src, obj, res in ex.map(compile_one, SOURCES):
            out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
            if res.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n" + out)
            if out.strip():
                msgs.append(out)
            objs.append(obj)
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs,
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    if verbose and msgs:
        print("\n".join(msgs), file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
