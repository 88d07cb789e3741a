"""Host-side guard on the generated gfx950 code (no GPU): a matrix-core instruction runs for the whole
wave whatever the lane mask says, so it must never sit in a block that is only masked off (EXEC saved
and narrowed, no branch around the block).  The compiler leaves out the skip branch of short masked
blocks; a decode GEMM whose k range it took for lane-dependent once added the products of a skipped
register batch that way.  The kernels keep such conditions wave-uniform (scalar); this test compiles
the device code of every kernel source and scans the assembly for the pattern."""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2311_15566_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = ["stream_gemm.hip", "gemm.hip", "attention.hip"]


def device_asm(src, out_dir):
    out = os.path.join(out_dir, src + ".s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "--cuda-device-only", "-S", "-o", out, os.path.join(CSRC, src)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return open(out).read()


def masked_mfma(asm):
    """(kernel, count) for every kernel with matrix-core instructions inside a masked block that no branch skips."""
    found, kernels = [], 0
    for name in re.findall(r"^(_ZN2ss\w+):", asm, re.M):
        start = asm.index("\n" + name + ":")
        body = asm[start:asm.index("s_endpgm", start)]
        lines = [l.strip() for l in body.split("\n") if l.strip() and not l.strip().startswith((".", ";"))]
        if not any(l.startswith("v_mfma") for l in lines):
            continue
        kernels += 1
        masked, n = False, 0
        for l in lines:
            if "saveexec" in l:
                masked = True                      # EXEC narrowed ...
            elif l.startswith(("s_cbranch_execz", "s_cbranch_execnz", "s_or_b64 exec", "s_mov_b64 exec")):
                masked = False                     # ... and either skipped when empty, or restored
            elif l.startswith("v_mfma") and masked:
                n += 1
        if n:
            found.append((name, n))
    return found, kernels


def test_scanner_sees_the_pattern():
    bad = "\n_ZN2ss4testEv:\n s_and_saveexec_b64 s[0:1], vcc\n v_mfma_f32_16x16x32_f16 v[0:3], v[4:7], v[8:11], v[0:3]\n s_or_b64 exec, exec, s[0:1]\n s_endpgm\n"
    good = bad.replace(" v_mfma", " s_cbranch_execz .L1\n v_mfma")
    assert masked_mfma(bad) == ([("_ZN2ss4testEv", 1)], 1)
    assert masked_mfma(good) == ([], 1)


def test_no_matrix_core_instruction_in_a_masked_block(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc is not installed")
    with ThreadPoolExecutor(max_workers=3) as ex:
        asms = list(ex.map(lambda s: device_asm(s, str(tmp_path)), SOURCES))
    total = 0
    for src, asm in zip(SOURCES, asms):
        found, kernels = masked_mfma(asm)
        assert not found, (src, found[:5])
        total += kernels
    assert total >= 40          # the scan saw the GEMM and attention kernels
