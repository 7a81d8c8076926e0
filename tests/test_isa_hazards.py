"""The d_h = 256 attention kernels (forward and backward) issue MFMAs as inline assembly (so that the score / dP
accumulators stay in ordinary vector registers and the output accumulators in the accumulation registers), and the
compiler does not track matrix-core hazards through inline assembly: the result of an 8-pass MFMA must not be
touched by another kind of instruction for 11 issue slots after it (12 for a write).  These tests compile the
attention sources to ISA and measure, for every such MFMA, the number of instructions issued before the first
non-MFMA instruction that touches its destination registers; the kernels' schedules are required to keep at least
16.  The backward kernels also rely on the compiler leaving the accumulation registers alone inside the main loop
(no copies in or out between the MFMAs): checked here as well."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NEED = 16


def _regs(tok):
    """Registers named by an operand: ordinary ones as non-negative numbers, accumulation registers as -(n + 1)."""
    m = re.fullmatch(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        r = range(int(m.group(2)), int(m.group(3)) + 1)
        return set(r) if m.group(1) == "v" else {-(x + 1) for x in r}
    m = re.fullmatch(r"([va])(\d+)", tok)
    if not m:
        return set()
    return {int(m.group(2))} if m.group(1) == "v" else {-(int(m.group(2)) + 1)}


def _parse(lines):
    out, in_asm = [], False
    for ln in lines:
        t = ln.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t[0] in ";." or t.endswith(":"):
            continue
        t = t.split(";")[0].strip()
        if not t:
            continue
        op, _, rest = t.partition(" ")
        out.append((op, [x for x in re.split(r"[ ,]+", rest) if x], in_asm, t))
    return out


def _min_distance(ins):
    """Smallest number of issue slots between an inline-assembly MFMA and the next non-MFMA instruction that reads
    or writes its destination (a later MFMA on the same registers is the next link of the chain: checked from
    there).  s_nop N counts N + 1.  An MFMA on other registers issued in between counts 1, or 8 if it reads the
    result of another MFMA issued in between: it then waits for that one, which entered the matrix core behind
    the MFMA under test and runs 8 slots.  (Whether MFMAs that do not depend on one another are held back at issue is
    not documented, so they are not relied on.)"""
    worst, where = None, None
    for i, (op, toks, in_asm, text) in enumerate(ins):
        if not (in_asm and op.startswith("v_mfma")):
            continue
        dst, dist, later = _regs(toks[0]), 0, set()
        for op2, toks2, _, text2 in ins[i + 1:i + 400]:
            touched = set().union(*[_regs(x) for x in toks2]) if toks2 else set()
            if touched & dst:
                if not op2.startswith("v_mfma") and (worst is None or dist < worst):
                    worst, where = dist, (text, text2)
                break
            if op2.startswith("v_mfma"):
                dist += 8 if touched & later else 1
                later |= _regs(toks2[0])
            else:
                dist += int(toks2[0]) + 1 if op2 == "s_nop" else 1
    return worst, where


def _isa(source):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    src = os.path.join(ROOT, "paper_2510_04476_amd", "csrc", source)
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attn.s")
        subprocess.run([hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only", "-S", "-Xclang",
                        "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I",
                        os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2510_04476_amd", "csrc"), src,
                        "-o", out], check=True, stderr=subprocess.DEVNULL)
        return open(out).read()


def _min_operand_age(ins):
    """Smallest number of issue slots between a vector-ALU instruction that writes a register and an
    inline-assembly MFMA that reads it as an operand.  The compiler pads this distance for the MFMAs it selects
    itself, not for inline assembly.  Seen on the GPU: an MFMA issued one slot after the v_mov_b64 pair that
    wrote its (zero) operand, and one issued directly behind the v_cvt_pk_bf16_f32 that packed its operand, gave
    wrong or non-finite results now and then.  Copies out of the accumulation registers (v_accvgpr_read, the
    compiler's spill reloads) one slot ahead are exempt: the forward kernel has them in its loop and its results
    are bit-identical from run to run."""
    worst, where = None, None
    for i, (op, toks, in_asm, text) in enumerate(ins):
        if not (in_asm and op.startswith("v_mfma")):
            continue
        src = set().union(*[_regs(x) for x in toks[1:]])
        dist = 0
        for op2, toks2, _, text2 in reversed(ins[max(0, i - 12):i]):
            valu = op2.startswith("v_") and not op2.startswith("v_mfma") and not op2.startswith("v_accvgpr_read")
            if valu and toks2 and _regs(toks2[0]) & src:
                if worst is None or dist < worst:
                    worst, where = dist, (text2, text)
                break
            dist += int(toks2[0]) + 1 if op2 == "s_nop" else 1
    return worst, where


@pytest.mark.parametrize("source,kernel,count", [("cca_attention.hip", "attn_fwd_wide_kernel", 4),
                                                 ("cca_attention_bwd.hip", "attn_bwd_dq_wide_kernel", 2),
                                                 ("cca_attention_bwd.hip", "attn_bwd_dkdv_wide_kernel", 4)])
def test_inline_mfma_results_are_not_read_too_early(source, kernel, count):
    text = _isa(source)
    kernels = re.findall(r"^(_ZN3cca\S*" + kernel + r"\S*):.*?s_endpgm", text, flags=re.S | re.M)
    bodies = re.findall(r"^_ZN3cca\S*" + kernel + r"\S*:.*?s_endpgm", text, flags=re.S | re.M)
    assert len(bodies) >= count, kernels
    checked = 0
    for name, body in zip(kernels, bodies):
        ins = _parse(body.splitlines())
        n_inline = sum(1 for op, _, a, _ in ins if a and op.startswith("v_mfma"))
        assert n_inline > 0, name
        loops = [i for i, ln in enumerate(body.splitlines()) if "Inner Loop Header" in ln]
        worst, where = _min_distance(ins)
        assert worst is not None and worst >= NEED, (name, worst, where)
        age, which = _min_operand_age(ins)  # operands written by the vector ALU: at least 4 slots old
        assert age is None or age >= 4, (name, age, which)
        # the steady-state loop wraps around: scan it twice
        lines = body.splitlines()
        for start in loops[:1]:
            end = next(i for i in range(start, len(lines)) if "s_cbranch_execnz" in lines[i])
            loop = _parse(lines[start:end + 1])
            w2, wh2 = _min_distance(loop + loop)
            assert w2 is None or w2 >= NEED, (name, w2, wh2)
        checked += 1
    assert checked >= count


@pytest.mark.parametrize("kernel,count", [("attn_bwd_dq_wide_kernel", 2), ("attn_bwd_dkdv_wide_kernel", 4)])
def test_backward_wide_loops_keep_their_accumulators_in_place(kernel, count):
    """Every basic block of these kernels that holds MFMAs of the main loop (more than 32 of them) is free of
    scratch-memory traffic and of copies between ordinary and accumulation registers."""
    text = _isa("cca_attention_bwd.hip")
    bodies = re.findall(r"^_ZN3cca\S*" + kernel + r"\S*:.*?s_endpgm", text, flags=re.S | re.M)
    assert len(bodies) >= count
    for body in bodies:
        blocks = re.split(r"^\.LBB\d+_\d+:.*$", body, flags=re.M)
        hot = [b for b in blocks if b.count("v_mfma") > 32]
        assert hot
        for b in hot:
            assert "scratch_" not in b and "v_accvgpr" not in b
