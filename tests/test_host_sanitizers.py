"""The host side of the C ABI (argument checks, page bookkeeping, workspace carving, repack planning, RAE) under
AddressSanitizer and UndefinedBehaviorSanitizer: builds the sanitizer variant of the library (host code
instrumented, device code as usual) and runs tests/test_abi_host.py against it in a child process that has the
sanitizer runtime preloaded.  No GPU is needed."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2506_24119_amd import build as B
    if not os.path.exists(B.HIPCC):
        pytest.skip("no hipcc")
    runtime = B.asan_runtime()
    if not os.path.exists(runtime):
        pytest.skip("the compiler ships no shared sanitizer runtime")
    lib = B.build(lib=str(tmp_path / "libspiral_asan.so"), verbose=False, asan=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD", ""), runtime) if x)     # appended to what is there
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    env["SPIRAL_LIB"] = lib
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi_host.py"), "-q", "-x",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=600)
    out = r.stdout
    assert r.returncode == 0, out[-3000:]
    assert " passed" in out and "AddressSanitizer" not in out and "runtime error:" not in out, out[-3000:]
