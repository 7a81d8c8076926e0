"""The d_h = 256 attention kernel issues its score MFMAs as inline assembly (so that their accumulators stay in
ordinary vector registers), and the compiler does not track matrix-core hazards through inline assembly: the result
of an 8-pass MFMA must not be touched by a vector-ALU instruction for 11 issue slots after it (12 for a write).
This test compiles the attention source to ISA and measures, for every such MFMA, the number of instructions
issued before the first other instruction that touches its destination registers; the kernel's schedule is
required to keep at least 16."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NEED = 16


def _regs(tok):
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", tok)
    return {int(m.group(1))} if m else set()


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
    there).  s_nop N counts N + 1."""
    worst, where = None, None
    for i, (op, toks, in_asm, text) in enumerate(ins):
        if not (in_asm and op.startswith("v_mfma")):
            continue
        dst, dist = _regs(toks[0]), 0
        for op2, toks2, _, text2 in ins[i + 1:i + 400]:
            touched = set().union(*[_regs(x) for x in toks2]) if toks2 else set()
            if touched & dst:
                if not op2.startswith("v_mfma") and (worst is None or dist < worst):
                    worst, where = dist, (text, text2)
                break
            dist += int(toks2[0]) + 1 if op2 == "s_nop" else 1
    return worst, where


def test_inline_mfma_results_are_not_read_too_early():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    src = os.path.join(ROOT, "paper_2510_04476_amd", "csrc", "cca_attention.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attn.s")
        subprocess.run([hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only", "-S", "-Xclang",
                        "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I",
                        os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2510_04476_amd", "csrc"), src,
                        "-o", out], check=True, stderr=subprocess.DEVNULL)
        text = open(out).read()
    kernels = re.findall(r"^(_ZN3cca\S*attn_fwd_wide_kernel\S*):.*?s_endpgm", text, flags=re.S | re.M)
    bodies = re.findall(r"^_ZN3cca\S*attn_fwd_wide_kernel\S*:.*?s_endpgm", text, flags=re.S | re.M)
    assert len(bodies) >= 4, kernels
    checked = 0
    for name, body in zip(kernels, bodies):
        ins = _parse(body.splitlines())
        n_inline = sum(1 for op, _, a, _ in ins if a and op.startswith("v_mfma"))
        assert n_inline > 0, name
        loops = [i for i, ln in enumerate(body.splitlines()) if "Inner Loop Header" in ln]
        worst, where = _min_distance(ins)
        assert worst is not None and worst >= NEED, (name, worst, where)
        # the steady-state loop wraps around: scan it twice
        lines = body.splitlines()
        for start in loops[:1]:
            end = next(i for i in range(start, len(lines)) if "s_cbranch_execnz" in lines[i])
            loop = _parse(lines[start:end + 1])
            w2, wh2 = _min_distance(loop + loop)
            assert w2 is None or w2 >= NEED, (name, w2, wh2)
        checked += 1
    assert checked >= 4
