"""Host-side check of the compiled persistent matrix-core kernel (no GPU needed; hipcc cross-compiles).

conv_mfma_persistent_kernel issues its operand loads and waits for them with its own s_waitcnt
counts.  That is only sound if nothing the compiler emits can sit between such a load and its wait.
The kernel guarantees it by construction: the whole contraction of an item -- ring fill, MFMA loop,
chunk hand-over, drain -- is ONE asm statement, and the registers its loads land in are fixed
registers that the statement lists as clobbers.  This test compiles the kernel to assembly and
checks the construction for every instance: all MFMAs of a kernel lie in one asm region, the region
ends with everything drained, and the fixed registers are the ones the source says.
"""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2007_14178_amd", "csrc", "conv_mfma_persistent.hip")


@pytest.fixture(scope="module")
def asm_text():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(SRC),
               "--cuda-device-only", "-S", "-o", out, SRC]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


def _regs(text):
    out = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(a), int(b) + 1))
    out.update(int(a) for a in re.findall(r"\bv(\d+)\b", text))
    return out


@pytest.mark.parametrize("chain", [0, 1])
@pytest.mark.parametrize("vw", [4, 2, 1])
def test_contraction_is_one_asm_region(asm_text, vw, chain):
    name = f"conv_mfma_persistent_kernelILi{vw}ELb{chain}EEE"
    start = next(m.start() for m in re.finditer(r"^_ZN\S*" + name + r"\S*:", asm_text, re.M))
    lines = asm_text[start:asm_text.index("s_endpgm", start)].split("\n")
    mfma = [i for i, l in enumerate(lines) if l.strip().startswith("v_mfma")]
    # the eight that set the accumulators to zero (0 x 0 + 0), the normal turn, the half-item turn,
    # and the two turns that carry the chunk expansion
    zeroing = [i for i in mfma if re.search(r"\], 0 cbsz", lines[i])]
    assert len(zeroing) == 8 and zeroing == mfma[:8]
    mfma = mfma[8:]
    assert len(mfma) == 32 + 16 + 32 + 16
    begin = max(i for i in range(zeroing[0]) if "ASMSTART" in lines[i])
    end = min(i for i in range(mfma[-1], len(lines)) if "ASMEND" in lines[i])
    inside = lines[begin + 1:end]
    assert not any("ASMSTART" in l or "ASMEND" in l for l in inside), "the MFMAs lie in more than one asm statement"
    # every load the statement issues lands in v168..v255, and it leaves with nothing in flight
    for l in inside:
        t = l.strip()
        if t.startswith(("global_load", "ds_read")):
            dst = _regs(t.split(",")[0])
            assert dst and min(dst) >= 168, t
    text = "\n".join(inside)
    assert "s_waitcnt vmcnt(0) lgkmcnt(0)" in text
    drain = max(i for i, l in enumerate(inside) if "s_waitcnt vmcnt(0) lgkmcnt(0)" in l)
    # ... and from the drain the statement goes straight to its end (what follows in the text are
    # the out-of-line turns and hooks)
    after = [l.strip() for l in inside[drain + 1:]]
    jump = next(i for i, t in enumerate(after) if t.startswith("s_branch"))
    assert not any(t.startswith(("v_mfma", "global_load", "ds_read")) for t in after[:jump])
    # A / B operands of every MFMA are the fixed registers
    for i in mfma:
        tuples = re.findall(r"v\[(\d+):(\d+)\]", lines[i])
        for a, b in tuples[1:3]:
            assert 168 <= int(a) and int(b) <= 231, lines[i]
