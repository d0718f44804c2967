"""Host-side check of the compiled gfx950 code: no matrix instruction may sit under an EXEC mask without a branch.

The matrix (MFMA) instructions ignore EXEC.  Where a kernel leaves k-tiles out of a product by a condition, the
compiler must branch around the MFMAs; if it takes the condition for divergent it can turn a short block into
"s_and_saveexec ... s_or exec" with no branch, and the MFMAs inside then run although every lane is masked off.
The kernels avoid this by deriving such conditions from scalar values (wave index through readfirstlane); this test
compiles the bf16 kernels to assembly and looks for the pattern, so that a later change cannot bring it back unseen.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2510_01336_amd", "csrc", "kernels_bf16.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def masked_mfma(asm_text):
    """Names of the functions in which an MFMA follows an s_and_saveexec / s_andn2_saveexec with no branch, label or
    restore of EXEC in between, with the count of such places."""
    name, pending, bad = None, False, {}
    for line in asm_text.splitlines():
        m = re.match(r"^(_Z\S+):", line)
        if m:
            name, pending = m.group(1), False
            continue
        t = line.strip()
        if t.startswith(("s_and_saveexec", "s_andn2_saveexec", "s_or_saveexec")):
            pending = True
        elif pending and t.startswith(("s_cbranch", "s_or_b64 exec", "s_mov_b64 exec", ".LBB", "s_endpgm")):
            pending = False
        elif pending and t.startswith("v_mfma"):
            bad[name] = bad.get(name, 0) + 1
            pending = False
    return bad


def test_scanner_sees_the_pattern():
    good = "_Zk:\n s_and_saveexec_b64 s[0:1], vcc\n s_cbranch_execz .LBB0_1\n v_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]\n.LBB0_1:\n s_or_b64 exec, exec, s[0:1]\n"
    bad = "_Zk:\n s_and_saveexec_b64 s[0:1], vcc\n v_add_u32 v1, v2, v3\n v_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]\n s_or_b64 exec, exec, s[0:1]\n"
    assert masked_mfma(good) == {}
    assert masked_mfma(bad) == {"_Zk": 1}


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_no_mfma_under_an_exec_mask(tmp_path):
    out = tmp_path / "kernels_bf16.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "--cuda-device-only", "-S", SRC, "-o", str(out)]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    text = out.read_text()
    assert text.count("v_mfma_f32_16x16x32_bf16") > 1000          # the kernels are in there
    bad = masked_mfma(text)
    assert not bad, f"MFMA under an EXEC mask without a branch in: {bad}"
    shutil.rmtree(tmp_path, ignore_errors=True)
