"""Builds libspiral.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2506_24119_amd.build [--act bf16|f16]

hipcc cross-compiles without a GPU.  The packed-fp32 target feature is switched
off for every device compile.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspiral.so")
SOURCES = ["spiral_api.hip", "kernels_misc.hip", "kernels_gemm.hip", "kernels_gemm_stream.hip", "kernels_gemm_tile.hip", "kernels_attn.hip", "kernels_sample.hip", "kernels_score.hip", "spiral_static_ws.hip", "spiral_rae.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _flags(act_f16: bool):
    return ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            f"-DSPIRAL_ACT_F16={1 if act_f16 else 0}",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(args):
    src, obj, flags = args
    cmd = [HIPCC] + flags + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    return src, r.returncode, out


def build(act_f16: bool = True, lib: str = LIB, verbose: bool = True) -> str:
    objdir = os.path.join(HERE, "_build", "f16" if act_f16 else "bf16")
    os.makedirs(objdir, exist_ok=True)
    flags = _flags(act_f16)
    jobs = [(s, os.path.join(objdir, s.rsplit(".", 1)[0] + ".o"), flags) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(jobs), 8)) as ex:
        results = list(ex.map(_compile, jobs))
    for src, rc, out in results:
        if verbose and out.strip():
            print(f"[{src}]\n{out}")
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + [j[1] for j in jobs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    act = "f16"
    if "--act" in sys.argv:
        act = sys.argv[sys.argv.index("--act") + 1]
    out = LIB
    if "--out" in sys.argv:
        out = sys.argv[sys.argv.index("--out") + 1]
    build(act_f16=(act == "f16"), lib=out)
