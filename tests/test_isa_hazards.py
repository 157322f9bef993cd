"""Two kernels (the software-pipelined prefix kernel and the 128-row absorb kernel) write their
MFMAs in assembly, so nothing inserts the wait states the hardware needs between a vector-ALU
write of a register and a matrix-core read of it.  The kernels are arranged so that no such pair
is ever adjacent; this test compiles them to assembly and checks that: no MFMA of those kernels
reads a register that one of the few instructions in front of it wrote with the vector ALU
(copies the register allocator may have placed there included), and no vector-ALU instruction
reads an MFMA's result right behind it."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2509_21081_amd import build as B

KERNELS = [("tmla_prefix_mfma.hip", "prefix_attn_pipelined_kernel"),
           ("tmla_absorb128_mfma.hip", "absorb128_kernel")]
LOOKBACK = 3      # instructions in front of an MFMA that must not write its operands


def _regs(tok):
    """'v[12:15]' -> ('v', {12..15}); 'a3' -> ('a', {3}); anything else -> None."""
    m = re.fullmatch(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return m.group(1), set(range(int(m.group(2)), int(m.group(3)) + 1))
    m = re.fullmatch(r"([va])(\d+)", tok)
    if m:
        return m.group(1), {int(m.group(2))}
    return None


def _operands(line):
    body = line.split(None, 1)[1] if len(line.split(None, 1)) > 1 else ""
    return [t.strip() for t in body.split(",")]


_cache = {}


def _kernel_instructions(source, kernel):
    if (source, kernel) not in _cache:
        src = os.path.join(B.CSRC, source)
        with tempfile.TemporaryDirectory() as tmp:
            out = os.path.join(tmp, "k.s")
            subprocess.run([B.HIPCC, *B.FLAGS, "-S", "--cuda-device-only", "-o", out, src],
                           check=True, capture_output=True)
            text = open(out).read()
        start = text.index("\n_ZN4tmla" + str(len(kernel)) + kernel)
        end = text.index("\n.Lfunc_end", start)     # (early exits put s_endpgm in the middle)
        instrs = []
        for raw in text[start:end].split("\n"):
            t = raw.strip()
            if not t or t.startswith(";") or t.startswith(".") or t.endswith(":"):
                continue
            instrs.append(t.split(";")[0].strip())
        _cache[(source, kernel)] = instrs
    return _cache[(source, kernel)]


@pytest.mark.parametrize("source,kernel", KERNELS)
@pytest.mark.skipif(not os.path.exists(B.HIPCC), reason="hipcc not available")
def test_no_vector_write_right_in_front_of_an_assembly_mfma(source, kernel):
    instrs = _kernel_instructions(source, kernel)
    n_mfma = 0
    for i, ins in enumerate(instrs):
        if not ins.startswith("v_mfma"):
            continue
        n_mfma += 1
        reads = [r for r in map(_regs, _operands(ins)[1:]) if r]     # A, B, C
        for prev in instrs[max(0, i - LOOKBACK):i]:
            op = prev.split()[0]
            if not op.startswith("v_") or op.startswith("v_mfma") or op.startswith("v_cmp"):
                continue
            dst = _regs(_operands(prev)[0])
            if not dst:
                continue
            for kind, regs in reads:
                assert not (kind == dst[0] and regs & dst[1]), (
                    f"'{prev}' writes an operand of '{ins}' {LOOKBACK} or fewer instructions "
                    f"in front of it")
    assert n_mfma > 100     # the loop bodies were found


@pytest.mark.parametrize("source,kernel", KERNELS)
@pytest.mark.skipif(not os.path.exists(B.HIPCC), reason="hipcc not available")
def test_no_vector_read_right_behind_an_assembly_mfma(source, kernel):
    """The other direction: a vector-ALU instruction (a register copy, say) that reads what an
    MFMA a few instructions in front of it writes would see the old contents.  The kernel's own
    reads come a whole period later or behind a long run of idle slots."""
    instrs = _kernel_instructions(source, kernel)
    behind = 8
    for i, ins in enumerate(instrs):
        op = ins.split()[0]
        if not op.startswith("v_") or op.startswith("v_mfma"):
            continue
        reads = [r for r in map(_regs, _operands(ins)[1:]) if r]
        for prev in reversed(instrs[max(0, i - behind):i]):
            if prev.startswith("s_nop 15"):
                break     # a drain
            if not prev.startswith("v_mfma"):
                continue
            dst = _regs(_operands(prev)[0])
            for kind, regs in reads:
                assert not (kind == dst[0] and regs & dst[1]), (
                    f"'{ins}' reads the result of '{prev}' {behind} or fewer instructions behind it")
