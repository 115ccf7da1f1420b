"""The grouped GEMM issues its MFMAs through inline statements, which the compiler does not see as MFMAs: it inserts
no wait states between the last MFMA of a K loop and the first read of an accumulator.  The source provides them
(a pair of `s_nop 15` behind the loop) and ties every accumulator to a point behind them.  This test compiles the
kernel to a listing and checks that the compiler kept it that way: between the last MFMA ahead of each such pair
and the pair itself nothing reads an accumulator (no v_accvgpr_read/mov, no accumulator spill)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_13920_amd", "csrc")


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    return None


@pytest.mark.skipif(hipcc() is None, reason="hipcc not found")
def test_no_accumulator_read_between_the_last_mfma_and_the_wait_states(tmp_path):
    out = tmp_path / "ffn.s"
    cmd = [hipcc(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-x", "hip", "--cuda-device-only", "-S", os.path.join(CSRC, "ffn.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln.strip() for ln in out.read_text().split("\n")]
    reads = re.compile(r"^(v_accvgpr_read|v_accvgpr_mov|scratch_store\w* off, a\[)")
    pairs = bad = 0
    for i in range(len(lines) - 1):
        if lines[i] == "s_nop 15" and lines[i + 1] == "s_nop 15":
            pairs += 1
            j = i - 1
            while j > 0 and "v_mfma" not in lines[j]:
                if reads.match(lines[j]):
                    bad += 1
                j -= 1
    # M0 carries the LDS base of the direct-to-LDS copies across several instructions: the only lines that name
    # it are the kernels' own writes
    named = [ln for ln in lines if re.search(r"\bm0\b", ln) and not ln.startswith(";")]
    assert named and all(ln.startswith("s_mov_b32 m0,") for ln in named), [ln for ln in named if not ln.startswith("s_mov_b32 m0,")][:5]
    # eight row-count variants of the K loop in each of the four epilogue forms of the persistent kernel and of the
    # one-tile-per-group kernel
    assert pairs >= 32, pairs
    assert bad == 0, f"{bad} accumulator reads ahead of the wait states"
