"""Two kernels (the software-pipelined prefix kernel and the 128-row absorb kernel) write their
MFMAs in assembly, so nothing inserts the wait states the hardware needs around them.  The
kernels are arranged so that no dependent pair is ever close; this test compiles them to
assembly and checks it by counting wait states between producer and consumer: an ordinary
instruction counts 1, `s_nop N` counts N + 1, an MFMA in between counts its 8 passes (the matrix
pipe takes the next one only when the previous one has gone through them).

  * a vector-ALU write of a register (copies placed by the register allocator included) must
    lie at least VALU_TO_MFMA wait states in front of an assembly MFMA that reads it;
  * the result of a v_mfma_f32_32x32x16_bf16 (8 passes) may be read -- by the vector ALU, by a
    store, by an LDS write, or as the A/B operand of a later MFMA -- or overwritten only
    MFMA_RESULT wait states behind it (passes + 3, one more on gfx950).  An MFMA that
    accumulates into the registers of the one before it is the chained case the hardware
    handles itself and is not checked.

Both directions are also checked across the back edge of every loop (the tail of the loop body
followed by its head)."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2509_21081_amd import build as B

KERNELS = [("tmla_prefix_mfma.hip", "prefix_attn_pipelined_kernel"),
           ("tmla_absorb128_mfma.hip", "absorb128_kernel")]
VALU_TO_MFMA = 4      # wait states between a vector-ALU write and an assembly MFMA reading it
MFMA_RESULT = 12      # wait states between an 8-pass MFMA and any other use of its result
MFMA_PASSES = 8
WINDOW = 48           # instructions looked at on either side of a loop's back edge


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
    parts = line.split(None, 1)
    body = parts[1] if len(parts) > 1 else ""
    return [t.strip().split()[0] if t.strip() else "" for t in body.split(",")]


def _wait_states(ins):
    op = ins.split()[0]
    if op == "s_nop":
        return int(ins.split()[1], 0) + 1
    if op.startswith("v_mfma"):
        return MFMA_PASSES
    return 1


def _overlap(a, b):
    return a is not None and b is not None and a[0] == b[0] and bool(a[1] & b[1])


_cache = {}


def _kernel_text(source, kernel):
    """(instructions, labels): instructions in text order; labels maps a label to the index of the
    instruction that follows it."""
    if (source, kernel) not in _cache:
        src = os.path.join(B.CSRC, source)
        with tempfile.TemporaryDirectory() as tmp:
            out = os.path.join(tmp, "k.s")
            subprocess.run([B.HIPCC, *B.FLAGS, "-S", "--cuda-device-only", "-o", out, src],
                           check=True, capture_output=True)
            text = open(out).read()
        start = text.index("\n_ZN4tmla" + str(len(kernel)) + kernel)
        end = text.index("\n.Lfunc_end", start)     # (early exits put s_endpgm in the middle)
        instrs, labels = [], {}
        for raw in text[start:end].split("\n"):
            t = raw.split(";")[0].strip()
            if not t:
                continue
            if t.endswith(":"):
                labels[t[:-1]] = len(instrs)
                continue
            if t.startswith("."):
                continue
            instrs.append(t)
        _cache[(source, kernel)] = (instrs, labels)
    return _cache[(source, kernel)]


def _sequences(instrs, labels):
    """The straight-line text, then for every backward branch the tail of the loop body followed
    by its head."""
    yield "text order", instrs
    for j, ins in enumerate(instrs):
        op = ins.split()[0]
        if op.startswith("s_cbranch") or op == "s_branch":
            target = _operands(ins)[0]
            k = labels.get(target)
            if k is not None and k <= j:
                yield f"back edge to {target}", instrs[max(k, j - WINDOW):j + 1] + instrs[k:k + WINDOW]


def _check_valu_to_mfma(seq, where):
    n_mfma = 0
    for i, ins in enumerate(seq):
        if not ins.startswith("v_mfma"):
            continue
        n_mfma += 1
        reads = [_regs(t) for t in _operands(ins)[1:]]     # A, B, C
        waited = 0
        for prev in reversed(seq[max(0, i - 4 * VALU_TO_MFMA):i]):
            if waited >= VALU_TO_MFMA:
                break
            op = prev.split()[0]
            if op.startswith("v_") and not op.startswith("v_mfma") and not op.startswith("v_cmp"):
                dst = _regs(_operands(prev)[0])
                for r in reads:
                    assert not _overlap(r, dst), (
                        f"{where}: '{prev}' writes an operand of '{ins}' only {waited} wait "
                        f"states in front of it")
            waited += _wait_states(prev)
    return n_mfma


def _check_mfma_result(seq, where):
    for i, ins in enumerate(seq):
        op = ins.split()[0]
        if op.startswith("s_"):
            continue
        ops = [_regs(t) for t in _operands(ins)]
        if op.startswith("v_mfma"):
            touched = ops[1:3]            # A and B; C / D in the same registers is the chained case
        else:
            touched = ops                 # sources, and the destination (write after write)
        waited = 0
        for prev in reversed(seq[max(0, i - MFMA_RESULT):i]):
            if waited >= MFMA_RESULT:
                break
            if prev.startswith("v_mfma"):
                dst = _regs(_operands(prev)[0])
                for r in touched:
                    assert not _overlap(r, dst), (
                        f"{where}: '{ins}' touches the result of '{prev}' only {waited} wait "
                        f"states behind it")
            waited += _wait_states(prev)


@pytest.mark.parametrize("source,kernel", KERNELS)
@pytest.mark.skipif(not os.path.exists(B.HIPCC), reason="hipcc not available")
def test_no_vector_write_close_in_front_of_an_assembly_mfma(source, kernel):
    instrs, labels = _kernel_text(source, kernel)
    n_loops = -1
    for where, seq in _sequences(instrs, labels):
        n = _check_valu_to_mfma(seq, where)
        if where == "text order":
            assert n > 100     # the loop bodies were found
        n_loops += 1
    assert n_loops >= 1        # and at least one loop's back edge


@pytest.mark.parametrize("source,kernel", KERNELS)
@pytest.mark.skipif(not os.path.exists(B.HIPCC), reason="hipcc not available")
def test_nothing_touches_an_mfma_result_before_it_is_written(source, kernel):
    """A register copy, a store or the A/B operand of a later MFMA that reads what an MFMA a few
    instructions in front of it writes would see the old contents.  The kernels' own reads come
    a whole period later or behind a long run of idle slots."""
    instrs, labels = _kernel_text(source, kernel)
    for where, seq in _sequences(instrs, labels):
        _check_mfma_result(seq, where)


def test_the_checker_itself_sees_a_planted_hazard():
    ok = ["v_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], a[0:3], v[0:15]", "s_nop 7", "s_nop 3",
          "v_add_f32 v40, v0, v1"]
    _check_mfma_result(ok, "planted")
    with pytest.raises(AssertionError):
        _check_mfma_result(ok[:2] + ok[3:], "planted")           # only 8 wait states
    with pytest.raises(AssertionError):                          # result used as a later A operand
        _check_mfma_result([ok[0], "v_mfma_f32_32x32x16_bf16 v[40:55], v[0:3], a[0:3], v[40:55]"],
                           "planted")
    _check_mfma_result([ok[0], ok[0]], "planted")                # chained accumulation is fine
    bad = ["v_mov_b32 v20, 0", "s_nop 1", ok[0]]
    with pytest.raises(AssertionError):
        _check_valu_to_mfma(bad, "planted")
    _check_valu_to_mfma(["v_mov_b32 v20, 0", "s_nop 3", ok[0]], "planted")
