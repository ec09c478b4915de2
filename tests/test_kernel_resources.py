"""Host-only guard on the register budget of the decode attention kernel: it runs three workgroups per compute unit
(three waves per SIMD), which holds only while a wave needs at most 168 vector registers and spills nothing.  An
innocent-looking source change can cost that occupancy (and a fifth of the kernel's bandwidth) without failing any
numerical test, so the compiler's own resource report is checked here."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_decode_attention_fits_three_waves_per_simd(tmp_path):
    from paper_2506_24119_amd import build as B
    if not (os.path.exists(B.HIPCC) or shutil.which(B.HIPCC)):
        pytest.skip("hipcc not available")
    src = os.path.join(B.CSRC, "kernels_attn.hip")
    cmd = [B.HIPCC] + B._flags() + ["-x", "hip", "--cuda-device-only", "-S", src, "-o", str(tmp_path / "attn.s")]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    asm = open(tmp_path / "attn.s").read()
    found = {}
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)\n\s+\.vgpr_spill_count:\s+(\d+)", asm):
        found[m.group(1)] = (int(m.group(2)), int(m.group(3)))
    stream = {k: v for k, v in found.items() if "attn_stream_kernel" in k}
    assert len(stream) >= 6, sorted(found)                      # head_dim 32 / 64 / 128 x two activation types
    for name, (vgprs, spills) in stream.items():
        assert vgprs <= 168 and spills == 0, (name, vgprs, spills)
