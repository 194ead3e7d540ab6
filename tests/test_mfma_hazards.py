"""Static check of the hand-written MFMAs in the matrix-core streaming kernel (no GPU needed).

The kernel with four row blocks writes its score MFMAs as inline assembly so that their results land
in vector registers.  The compiler does not look inside inline assembly, so it neither knows that
these are matrix instructions nor inserts the wait a vector instruction needs before it may touch an
MFMA's result registers.  The source keeps every reader far away from its MFMA (or ends the
statement with an s_nop); this test compiles the file to assembly and checks the generated code
itself: after every hand-written MFMA no instruction other than an MFMA accumulating into the same
registers touches its destination before the distance the compiler keeps after its OWN MFMAs of the
same opcode (calibrated on the same file, from the kernels whose MFMAs it schedules itself).
"""
import os
import re
import subprocess

import pytest

from paper_2408_04093_amd import build as B

SRC = os.path.join(B.CSRC, "decode_partial_mfma.hip")
OPCODE = "v_mfma_f32_16x16x32_bf16"


def _regs(tok):
    tok = tok.rstrip(",")
    m = re.match(r"^[|-]*v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"^[|-]*v(\d+)\b", tok)
    return {int(m.group(1))} if m else set()


def _instructions(text):
    """(line number, text, inside inline assembly) for every instruction line."""
    out, in_asm = [], False
    for n, line in enumerate(text.split("\n"), 1):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
        elif t.startswith(";;#ASMEND"):
            in_asm = False
        elif t and not t.startswith((";", ".")) and not t.endswith(":"):
            out.append((n, t, in_asm))
    return out


def _distance_to_first_touch(ins, i, limit=64):
    """Wait states between MFMA ins[i] and the first later instruction that touches its destination
    other than another MFMA taking it as C operand or result (None if a branch or `limit` wait
    states come first).  Every instruction counts one wait state, s_nop N counts N + 1."""
    dst = _regs(ins[i][1].split()[1])
    ws = 0
    for n, t, _ in ins[i + 1:]:
        op = t.split()[0]
        if op.startswith(("s_cbranch", "s_branch", "s_endpgm", "s_setpc")):
            return None
        toks = t.split()[1:]
        touched = set()
        for x in toks:
            touched |= _regs(x)
        if touched & dst:
            # an MFMA that takes the result as its C operand (or writes over it) is interlocked by the
            # hardware: the compiler chains them back to back; as A or B operand it counts
            as_c_only = op.startswith("v_mfma") and not ((_regs(toks[1]) | _regs(toks[2])) & dst)
            if not as_c_only:
                return ws, n, t
        m = re.match(r"s_nop (\d+)", t)
        ws += int(m.group(1)) + 1 if m else 1
        if ws >= limit:
            return None
    return None


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    out = tmp_path_factory.mktemp("asm") / "decode_partial_mfma.s"
    flags = [f for f in B.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc] + flags + ["-S", "--cuda-device-only", "-I", B.CSRC, "-I", os.path.join(B.HERE, "..", "include"),
                              SRC, "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return out.read_text()


def test_hand_written_mfmas_keep_the_compilers_own_distance(assembly):
    ins = _instructions(assembly)
    own, hand = [], []
    for i, (n, t, in_asm) in enumerate(ins):
        if t.startswith(OPCODE + " v["):          # result in vector registers
            (hand if in_asm else own).append(i)
    assert len(hand) >= 64, "the inline-assembly MFMAs were not found: has the kernel changed?"
    assert len(own) >= 64, "no compiler-scheduled MFMAs with vector-register results to calibrate on"

    # the distance the compiler keeps: the smallest one it ever leaves after its own MFMAs
    dists = [d[0] for d in (_distance_to_first_touch(ins, i) for i in own) if d is not None]
    assert dists, "compiler-scheduled MFMAs never had their results read in straight-line code"
    required = min(dists)
    assert 4 <= required <= 20, required          # a sanity band around the 8 seen with ROCm 7.2

    bad = []
    for i in hand:
        d = _distance_to_first_touch(ins, i)
        if d is not None and d[0] < required:
            bad.append((ins[i][0], ins[i][1], d))
    assert not bad, "result of a hand-written MFMA touched after fewer than %d wait states: %r" % (required, bad[:5])


def test_no_kernel_spills_to_scratch(assembly):
    """No kernel of the file spills registers to scratch memory."""
    scratch = [int(x) for x in re.findall(r"; ScratchSize: (\d+)", assembly)]
    assert scratch and max(scratch) == 0, scratch
