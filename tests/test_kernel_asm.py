"""Static check of the dK/dV kernel's hand-issued MFMAs.

The kernel accumulates S and dP in ordinary vector registers with MFMAs written in `asm`, which
the compiler's hazard tracking does not see.  The source promises three things for them; this
test compiles the file to assembly text (no GPU needed) and checks the promises on every
instantiation of the kernel, so that a rebuild with another schedule cannot break them silently:
  1. no vector instruction writes an operand or the result registers of such an MFMA within the
     two wait states before it (an instruction is one wait state, `s_nop n` is n + 1);
  2. the result registers of an MFMA whose C operand is the literal 0 overlap neither A nor B;
  3. between such an MFMA and the `s_nop 15` that follows the chain, no other instruction
     names one of its result registers.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def vregs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


@pytest.fixture(scope="module")
def bwd_asm(tmp_path_factory):
    if not os.path.exists(HIPCC) and shutil.which(HIPCC) is None:
        pytest.skip("hipcc not available")
    import sys
    sys.path.insert(0, ROOT)
    from paper_2506_19852_amd import build as hip_build
    out = tmp_path_factory.mktemp("asm") / "radial_attn_bwd.s"
    cmd = [HIPCC, *hip_build.FLAGS, "--cuda-device-only", "-S", os.path.join(hip_build.CSRC, "radial_attn_bwd.hip"), "-o", str(out)]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    return out.read_text().split("\n")


def kernels(lines, name):
    cur, body = None, []
    for l in lines:
        m = re.match(r"^(_ZN[^\s.]*" + name + r"[^\s.]*):", l)   # the function's label, not its descriptor's
        if m:
            cur, body = m.group(1), []
        elif cur is not None:
            body.append(l)
            if l.startswith(".Lfunc_end"):   # (a kernel may hold more than one s_endpgm)
                yield cur, body
                cur = None


def instructions(body):
    for l in body:
        code = l.split(";")[0].strip()
        if code and l.startswith("\t") and not code.startswith("."):
            yield code


def is_hand_mfma(ins):
    return ins.startswith("v_mfma") and ins.split(None, 1)[1].lstrip().startswith("v[")


def check_kernel(name, code):
    """Asserts the three promises on one kernel's instruction list; returns the number of hand-issued MFMAs."""
    in_flight = set()   # result registers of hand-issued MFMAs since the last settle
    n_mfma = 0
    for i, ins in enumerate(code):
        if is_hand_mfma(ins):
            n_mfma += 1
            dst, a, b, c = [t.strip() for t in ins.split(None, 1)[1].split(",")]
            used = vregs(dst) | vregs(a) | vregs(b)
            waited, j = 0, i - 1
            while waited < 2 and j >= 0:
                prev = code[j]
                if prev.startswith("v_") and not prev.startswith("v_mfma"):
                    written = vregs(prev.split(None, 1)[1].split(",")[0])
                    assert not (written & used), (name, "operand written right before", prev, ins)
                waited += int(prev.split()[1]) + 1 if prev.startswith("s_nop") else 1
                j -= 1
            if c == "0":
                assert not (vregs(dst) & (vregs(a) | vregs(b))), (name, "result overlaps an operand", ins)
            else:
                assert c == dst, (name, ins)
            in_flight |= vregs(dst)
        elif ins == "s_nop 15":
            in_flight = set()
        elif in_flight:
            assert not (vregs(ins) & in_flight), (name, "accumulator named before the settle", ins, sorted(vregs(ins) & in_flight))
    assert not in_flight, (name, "no settle after the last chain")
    return n_mfma


def test_hand_issued_mfmas_keep_their_promises(bwd_asm):
    found = 0
    for name, body in kernels(bwd_asm, "radial_bwd_dkdv_kernel"):
        found += 1
        assert check_kernel(name, list(instructions(body))) > 0, name
    assert found == 8, found   # D in {64, 128} x block in {64, 128} x token rule on / off


GOOD = ["ds_read_b128 v[16:19], v20", "s_waitcnt lgkmcnt(0)", "v_mfma_f32_32x32x16_bf16 v[48:63], v[16:19], v[68:71], 0",
        "v_mfma_f32_32x32x16_bf16 v[32:47], v[22:25], v[64:67], 0", "v_add_u32_e32 v1, s4, v2",
        "v_mfma_f32_32x32x16_bf16 v[48:63], v[26:29], v[72:75], v[48:63]", "s_nop 15", "v_exp_f32_e32 v3, v48"]


@pytest.mark.parametrize("edit, what", [
    (lambda c: c[:2] + ["v_accvgpr_read_b32 v71, a3"] + c[2:], "operand written right before"),
    (lambda c: c[:2] + ["v_mfma_f32_32x32x16_bf16 v[16:31], v[16:19], v[68:71], 0"] + c[3:], "result overlaps an operand"),
    (lambda c: c[:4] + ["v_mov_b32_e32 v5, v33"] + c[4:], "accumulator named before the settle"),
    (lambda c: c[:6], "no settle after the last chain"),
])
def test_the_checker_sees_planted_violations(edit, what):
    assert check_kernel("good", GOOD) == 3
    with pytest.raises(AssertionError, match=what):
        check_kernel("planted", edit(list(GOOD)))
