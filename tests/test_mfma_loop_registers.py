"""Host-side check of the compiled matrix-core kernel (no GPU needed; hipcc cross-compiles).

conv_mfma_kernel issues its operand loads from inline-asm statements and waits for them with its
own s_waitcnt counts.  The compiler does not know that those registers have loads in flight, so
the kernel is only correct if no compiler-generated instruction reads one of them before the asm
statement that waits.  This test compiles the kernel to assembly and checks exactly that, for the
three staging widths and both epilogues: inside the MFMA loop region

  * no instruction outside the asm statements reads a register that an MFMA uses as an A / B operand
    (the filter ring, the pixel operands), and
  * between an asm fetch of staged input words and the asm wait that covers it, no instruction
    outside the asm statements reads the fetched registers.
"""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2007_14178_amd", "csrc", "conv_mfma.hip")


def _regs(text):
    out = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(a), int(b) + 1))
    out.update(int(a) for a in re.findall(r"\bv(\d+)\b", text))
    return out


def _sources(instr):
    """Registers an instruction reads (all operands but the destination; stores read everything)."""
    parts = instr.split(None, 1)
    if len(parts) < 2:
        return set()
    op, rest = parts
    if op.startswith(("ds_write", "global_store", "scratch_store", "buffer_store", "v_cmp", "s_")):
        return _regs(rest)
    ops = rest.split(",")
    return _regs(",".join(ops[1:]))


@pytest.fixture(scope="module")
def asm_text():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "conv_mfma.s")
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(SRC),
               "--cuda-device-only", "-S", "-o", out, SRC]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


@pytest.mark.parametrize("chain", [0, 1])
@pytest.mark.parametrize("vw", [4, 2, 1])
def test_no_compiler_read_of_registers_with_loads_in_flight(asm_text, vw, chain):
    name = f"conv_mfma_kernelILi{vw}ELb{chain}EEE"
    start = next(m.start() for m in re.finditer(r"^_ZN\S*" + name + r"\S*:", asm_text, re.M))
    body = asm_text[start:asm_text.index("s_endpgm", start)]
    lines = body.split("\n")
    mfma = [i for i, l in enumerate(lines) if l.strip().startswith("v_mfma")]
    assert len(mfma) >= 32, "the hand-placed loop should hold 4 steps x 8 MFMAs"
    operand_regs = set()
    for i in mfma:
        tuples = re.findall(r"v\[(\d+):(\d+)\]", lines[i])
        for a, b in tuples[1:3]:                       # dst, A, B, C
            operand_regs.update(range(int(a), int(b) + 1))
    assert 64 <= len(operand_regs) <= 80

    # region: from the barrier that ends the first staging to the last MFMA
    region_start = max(i for i in range(mfma[0]) if lines[i].strip().startswith("s_barrier"))
    # Linear scan in program order.  A register is "loaded" from the asm load that writes it until a
    # compiler-generated instruction overwrites it (the compiler reuses the pixel / ring registers as
    # temporaries while they are dead, which is fine: nothing is in flight to them then); reading a
    # "loaded" register outside the asm statements is the offence.  At the region's start every
    # operand register counts as loaded.
    in_asm = False
    loaded = set(operand_regs)
    fetched = set()                                    # staged input words with a fetch in flight
    offenders = []
    for i in range(region_start, mfma[-1] + 1):
        text = lines[i].strip()
        if "ASMSTART" in text:
            in_asm = True
            continue
        if "ASMEND" in text:
            in_asm = False
            continue
        if not text or text.startswith(";") or text.endswith(":") or text.startswith("."):
            continue
        if in_asm:
            if text.startswith(("global_load", "ds_read")):
                dst = _regs(text.split(",")[0])
                if text.startswith("global_load") and not dst & operand_regs:
                    fetched |= dst                     # staged input words, not the filter ring
                else:
                    loaded |= dst
            elif text.startswith("s_waitcnt") and ("vmcnt(6)" in text or "vmcnt(0)" in text):
                fetched = set()
            continue
        src = _sources(text)
        if i >= mfma[0] and src & loaded:
            offenders.append((i, text, "reads a register loaded by an asm statement"))
        if src & fetched:
            offenders.append((i, text, "reads a staged-word register before its wait"))
        parts = text.split(None, 1)
        if len(parts) == 2 and not parts[0].startswith(("ds_write", "global_store", "scratch_store", "s_", "v_cmp")):
            loaded -= _regs(parts[1].split(",")[0])    # overwritten by the compiler: a temporary now
    assert not offenders, offenders[:10]
