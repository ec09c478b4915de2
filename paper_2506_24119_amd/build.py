"""Builds libspiral.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2506_24119_amd.build [--asan] [--out PATH]

hipcc cross-compiles without a GPU.  The packed-fp32 target feature is switched
off for every device compile.

--asan builds libspiral_asan.so with AddressSanitizer and UndefinedBehaviorSanitizer on the
HOST code only (argument checks, page bookkeeping, workspace carving, RAE; device code is
compiled as usual), for running the host-only tests under the sanitizers on a CPU machine:

    LD_PRELOAD="$LD_PRELOAD:$(python -m paper_2506_24119_amd.build --asan-runtime)" \
    ASAN_OPTIONS=verify_asan_link_order=0:detect_leaks=0 SPIRAL_LIB=paper_2506_24119_amd/libspiral_asan.so \
        python -m pytest tests/test_abi_host.py -q
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


ASAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
              "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def _flags(asan: bool = False):
    return ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC] + (ASAN_FLAGS if asan else [])


def asan_runtime() -> str:
    """Path of the shared AddressSanitizer runtime that matches hipcc's clang."""
    r = subprocess.run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True)
    return os.path.realpath(r.stdout.strip())


def _compile(args):
    src, obj, flags = args
    cmd = [HIPCC] + flags + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    return src, r.returncode, out


def build(lib: str = LIB, verbose: bool = True, asan: bool = False) -> str:
    objdir = os.path.join(HERE, "_build", "asan" if asan else "f16")
    os.makedirs(objdir, exist_ok=True)
    flags = _flags(asan)
    jobs = [(s, os.path.join(objdir, s.rsplit(".", 1)[0] + ".o"), flags) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(jobs), 8)) as ex:
        results = list(ex.map(_compile, jobs))
    for src, rc, out in results:
        if verbose and out.strip():
            print(f"[{src}]\n{out}")
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + [j[1] for j in jobs]
    if asan:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-fno-gpu-sanitize"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    if "--asan-runtime" in sys.argv:
        print(asan_runtime())
        sys.exit(0)
    asan = "--asan" in sys.argv
    out = os.path.join(HERE, "libspiral_asan.so") if asan else LIB
    if "--out" in sys.argv:
        out = sys.argv[sys.argv.index("--out") + 1]
    build(lib=out, asan=asan)
