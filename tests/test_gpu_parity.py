"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the
same seeded inputs.  Tolerances are the spec ones: bf16 rel-L2 <= 1e-2
and max-abs <= 2e-2 on `out`; fp32 <= 1e-5."""
import sys

import numpy as np
import pytest
import torch

import paper_2510_04476_amd as P
from paper_2510_04476_amd import binding as B
from oracle import cca_oracle as O
from synth_inputs import WORKLOADS, make_inputs, round_to_bf16, sample_rows
from util import check_out, check_tap, errors, oracle_forward, to_np

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def run_gpu(w, inp, **override):
    cfg = P.config_from_workload(w, **override)
    x, wt = P.weights_to_device(cfg, inp)
    saved = P.CCASaved.allocate(cfg, x.device)
    out = P.cca_forward(cfg, wt, x, saved=saved)
    torch.cuda.synchronize()
    return cfg, out, saved


def compare_all(w, inp, ref, out, saved, rows=None):
    dt = w["dtype"]
    sel = (lambda a: a) if rows is None else (lambda a: a[:, rows])
    res = {}
    B_, T = w["B"], w["T"]
    lat_ref = np.concatenate([ref["q0"].reshape(B_, T, -1), ref["k0"].reshape(B_, T, -1), ref["vc"], ref["vp"]], -1)
    res["lat"] = check_tap(to_np(saved.lat), lat_ref, dt, "lat")
    res["q"] = check_tap(to_np(saved.q), ref["q"], dt, "q")
    res["k"] = check_tap(to_np(saved.k), ref["k"], dt, "k")
    res["v"] = check_tap(to_np(saved.v), ref["v"], dt, "v")
    res["o"] = check_tap(sel(to_np(saved.o)), ref["o"].reshape(B_, -1, w["Hq"] * w["dh"]), dt, "o")
    lse = to_np(saved.lse)
    lse = lse if rows is None else lse[:, :, rows]
    res["lse"] = check_tap(lse, ref["lse"], dt, "lse")
    res["out"] = check_out(sel(to_np(out)), ref["out"], dt)
    # factor applied by the norm step: |y| / |x| per head vector (1 when the norm is off)
    rn_ref = np.concatenate([np.linalg.norm(ref["q"], axis=-1) / np.linalg.norm(ref["q3"], axis=-1),
                             np.linalg.norm(ref["k"], axis=-1) / np.linalg.norm(ref["k3"], axis=-1)], axis=-1)
    rel, _ = errors(to_np(saved.rnorm), rn_ref)
    assert rel <= (1e-2 if dt == "bf16" else 1e-5), ("rnorm", rel)
    if saved.o_lo is not None:
        # o + o_lo carries the attention output to ~16 mantissa bits; what is left is the kernel's own error
        # (bf16 probabilities), far below the rounding of o alone at every element
        o_ref = ref["o"].reshape(B_, -1, w["Hq"] * w["dh"])
        rel_hi, _ = errors(sel(to_np(saved.o)), o_ref)
        rel_sum, _ = errors(sel(to_np(saved.o) + to_np(saved.o_lo)), o_ref)
        assert rel_sum <= rel_hi, ("o + o_lo", rel_sum, rel_hi)
        assert float(np.abs(sel(to_np(saved.o_lo))).max()) <= 2.0 ** -8 * max(1.0, float(np.abs(o_ref).max()))
        res["o+o_lo"] = (rel_sum, rel_hi)
    return res


# ---- config 1: tiny fp32, literal ------------------------------------------
def test_tiny_fp32():
    w = WORKLOADS["tiny_fp32"]
    say("case tiny_fp32", w)
    inp = make_inputs(w, seed=0)
    _, out, saved = run_gpu(w, inp)
    res = compare_all(w, inp, oracle_forward(w, inp), out, saved)
    say(res)


SMALL = [
    # ragged T, several tiles, GQA, both dtypes, head widths on and off the MFMA path
    dict(B=2, T=333, E=256, Hq=4, Hk=2, dh=32, k_seq=2, k_ch=2, dtype="f32", paper_flags=True),
    dict(B=2, T=333, E=512, Hq=4, Hk=2, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=2, T=777, E=1024, Hq=4, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=1, T=515, E=1024, Hq=8, Hk=2, dh=128, k_seq=3, k_ch=4, dtype="bf16", paper_flags=True),
    dict(B=1, T=300, E=512, Hq=2, Hk=1, dh=256, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=3, T=130, E=384, Hq=3, Hk=3, dh=128, k_seq=4, k_ch=1, dtype="bf16", paper_flags=True),
    dict(B=1, T=1, E=256, Hq=2, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=2, T=2, E=256, Hq=2, Hk=1, dh=64, k_seq=2, k_ch=2, dtype="f32", paper_flags=True),
    # d_h = 64 on the fused prologue: three taps, R = 4, several 256-token tiles with a ragged tail, T past 128 * 8
    dict(B=2, T=1100, E=512, Hq=8, Hk=2, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=1, T=260, E=512, Hq=3, Hk=3, dh=64, k_seq=1, k_ch=3, dtype="bf16", paper_flags=True),
    # group sizes that are not a power of two (R = 3, R = 6) on the fused prologue and the matrix-core attention
    dict(B=2, T=400, E=1536, Hq=6, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=1, T=300, E=768, Hq=6, Hk=1, dh=128, k_seq=2, k_ch=1, dtype="bf16", paper_flags=True),
    dict(B=2, T=520, E=768, Hq=6, Hk=2, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=1, T=270, E=768, Hq=12, Hk=2, dh=64, k_seq=1, k_ch=2, dtype="bf16", paper_flags=True),
    # d_h = 256 on the matrix-core attention kernel (one wavefront per SIMD, 128-row query blocks): several query
    # blocks with a ragged tail, R = 2; the prologue of this width streams its folded filter through LDS
    dict(B=2, T=700, E=2048, Hq=4, Hk=2, dh=256, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    # d_h = 256 with two taps, R = 3, a token count that leaves the last 256-token block of the streamed prologue ragged
    dict(B=1, T=530, E=1536, Hq=3, Hk=1, dh=256, k_seq=1, k_ch=2, dtype="bf16", paper_flags=True),
]


@pytest.mark.parametrize("i", range(len(SMALL)))
@pytest.mark.parametrize("conv_visible", [False, True])
def test_small_shapes(i, conv_visible):
    w = SMALL[i]
    say("case small", i, "conv_visible", conv_visible, w)
    inp = make_inputs(w, seed=10 + i, conv_visible=conv_visible)
    _, out, saved = run_gpu(w, inp)
    res = compare_all(w, inp, oracle_forward(w, inp), out, saved)
    say(res)


@pytest.mark.parametrize("i", [1, 2, 3, 4, 5, 6, 8, 10, 13, 14])
@pytest.mark.parametrize("causal", [True, False])
def test_small_shapes_inference_path(i, causal):
    """Without saved tensors the attention kernel takes its inference form (row sums of the unrounded
    probabilities): `out` must meet the same bar, and agree with the training form to bf16 rounding."""
    w = SMALL[i]
    say("case small, no saved tensors", i, "causal", causal, w)
    inp = make_inputs(w, seed=10 + i, conv_visible=True)
    flags = B.CCA_FLAGS_PAPER if causal else B.CCA_FLAGS_PAPER & ~B.CCA_CAUSAL
    cfg = P.config_from_workload(w, flags=flags)
    x, wt = P.weights_to_device(cfg, inp)
    out = P.cca_forward(cfg, wt, x)
    saved = P.CCASaved.allocate(cfg, x.device)
    out_t = P.cca_forward(cfg, wt, x, saved=saved)
    torch.cuda.synchronize()
    ref = oracle_forward(w, inp, causal=causal)
    say(check_out(to_np(out), ref["out"], w["dtype"]))
    scale = float(np.abs(ref["out"]).max())
    assert float(np.abs(to_np(out) - to_np(out_t)).max()) <= 2.0 ** -6 * scale


FLAG_CASES = {
    "no_qk_mean": (B.CCA_FLAGS_PAPER & ~B.CCA_QK_MEAN, dict(use_qk_mean=False)),
    "no_conv_seq": (B.CCA_FLAGS_PAPER & ~B.CCA_CONV_SEQ, dict(use_conv_seq=False)),
    "no_conv_ch": (B.CCA_FLAGS_PAPER & ~B.CCA_CONV_CH, dict(use_conv_ch=False)),
    "no_v_shift": (B.CCA_FLAGS_PAPER & ~B.CCA_V_SHIFT, dict(use_v_shift=False)),
    "no_norm": (B.CCA_FLAGS_PAPER & ~(B.CCA_QK_NORM | B.CCA_KEY_TEMP), dict(use_qk_norm=False, use_key_temp=False)),
    "no_temp": (B.CCA_FLAGS_PAPER & ~B.CCA_KEY_TEMP, dict(use_key_temp=False)),
    "no_rope": (B.CCA_FLAGS_PAPER & ~B.CCA_ROPE, dict(use_rope=False)),
    "rope_interleaved": (B.CCA_FLAGS_PAPER | B.CCA_ROPE_INTERLEAVED, dict(rope_interleaved=True)),
    "non_causal": (B.CCA_FLAGS_PAPER & ~B.CCA_CAUSAL, dict(causal=False)),
}


@pytest.mark.parametrize("name", sorted(FLAG_CASES))
@pytest.mark.parametrize("dtype,dh", [("f32", 32), ("bf16", 128), ("bf16", 64)])
def test_each_flag(name, dtype, dh):
    flags, okw = FLAG_CASES[name]
    w = dict(B=2, T=200, E=4 * dh * 2, Hq=4, Hk=2, dh=dh, k_seq=2, k_ch=2, dtype=dtype, paper_flags=True)
    say("case flag", name, w)
    # without the norm the logits are small unless the weights are scaled up
    inp = make_inputs(w, seed=21, conv_visible=True)
    _, out, saved = run_gpu(w, inp, flags=flags)
    res = compare_all(w, inp, oracle_forward(w, inp, **okw), out, saved)
    say(res)


@pytest.mark.parametrize("Hq,Hk", [(4, 4), (8, 2), (4, 1)])
def test_mha_gqa_flags(Hq, Hk):
    """Compression 1, no transforms: plain MHA / GQA through the same kernels."""
    w = dict(B=2, T=300, E=Hq * 128, Hq=Hq, Hk=Hk, dh=128, k_seq=1, k_ch=1, dtype="bf16", paper_flags=False)
    say("case mha", w)
    inp = make_inputs(w, seed=5)
    _, out, saved = run_gpu(w, inp)
    res = compare_all(w, inp, oracle_forward(w, inp), out, saved)
    say(res)


# ---- stage level: attention on oracle-made latents --------------------------
@pytest.mark.parametrize("mode", ["normed", "normed_hot", "free"])
@pytest.mark.parametrize("T,Hq,Hk,dh,causal", [(1000, 8, 2, 128, True), (640, 4, 4, 128, False),
                                                (257, 2, 1, 64, True), (513, 4, 2, 128, True),
                                                (700, 6, 2, 128, True), (330, 6, 1, 64, True), (450, 12, 2, 64, False),
                                                (900, 4, 2, 256, True), (390, 3, 1, 256, False), (129, 2, 2, 256, True)])
def test_attention_stage(T, Hq, Hk, dh, causal, mode):
    """normed: q, k on the spheres the prologue produces (bounded-score path of the kernel);
    normed_hot: same with a temperature large enough that the kernel must fall back to the running max;
    free: arbitrary q, k with QK_NORM cleared, one planted large key late in the sequence (late rescale)."""
    say("case attention stage", T, Hq, Hk, dh, causal, mode)
    rng = np.random.default_rng(T)
    Bn = 2
    q = rng.standard_normal((Bn, T, Hq, dh))
    k = rng.standard_normal((Bn, T, Hk, dh))
    flags = B.CCA_FLAGS_PAPER if causal else B.CCA_FLAGS_PAPER & ~B.CCA_CAUSAL
    temp = np.zeros(Hk, np.float32)
    if mode == "free":
        flags &= ~(B.CCA_QK_NORM | B.CCA_KEY_TEMP)
        q *= 1.5
        k *= 1.5
        k[:, (2 * T) // 3] *= 3.0
    else:
        if mode == "normed_hot":
            temp = np.full(Hk, 1.6, np.float32)  # beta ~ 5: bound on the scores beyond the kernel's limit
        else:
            temp = np.linspace(-0.3, 0.4, Hk).astype(np.float32)
        q *= np.sqrt(dh) / np.linalg.norm(q, axis=-1, keepdims=True)
        k *= np.sqrt(dh) / np.linalg.norm(k, axis=-1, keepdims=True) * np.exp(temp)[None, None, :, None]
    v = rng.standard_normal((Bn, T, Hk, dh))
    q, k, v = (round_to_bf16(a.astype(np.float32)) for a in (q, k, v))
    cfg = P.CCAConfig(B=Bn, T=T, d_model=Hq * dh, n_q_heads=Hq, n_kv_heads=Hk, head_dim=dh, flags=flags)
    dev = lambda a: torch.from_numpy(a).to("cuda", torch.bfloat16)
    o, lse = P.cca_attention(cfg, dev(q), dev(k), dev(v), want_lse=True, temp=torch.from_numpy(temp).cuda())
    torch.cuda.synchronize()
    o_ref, lse_ref = O.attention(q, k, v, 1.0 / np.sqrt(dh), causal=causal)
    say("o", check_tap(to_np(o).reshape(o_ref.shape), o_ref, "bf16", "o"))
    rel, mx = errors(to_np(lse), lse_ref)
    lim, worst = lse_bounds(q, k, dh)
    say("lse", dict(max_abs=mx, asserted=lim, worst_case=worst, measured_over_asserted=mx / lim))
    assert mx <= lim, ("lse", rel, mx, lim)


def lse_bounds(q, k, dh):
    """Error model of lse (natural-log units).  The kernel multiplies each q component by c = scale * log2(e)
    and rounds it to bf16 again: q'_i = q_i c (1 + d_i), |d_i| <= 2^-8 (bf16 keeps 8 significant bits: half a
    unit in the last place is 2^-8 of a number just above a power of two), so a logit s = scale * <q, k> is off
    by sum_i scale q_i k_i d_i, at most 2^-8 * scale * sum_i |q_i k_i| <= 2^-8 s_max with s_max = scale |q| |k|
    (every d_i at its limit with the sign of q_i k_i: test_lse_error_worst_case constructs that input), and lse
    is a soft maximum of the logits (its gradient is a probability vector), so its error is bounded by the same
    number.  On top: the row sum adds probabilities rounded to bf16 (relative 2^-8 each at worst, so 2^-8 on lse)
    and fp32 arithmetic.  Worst case: 2^-8 (s_max + 1) + 1e-3.  For inputs whose d_i are not aligned the d_i
    average out over the d_h terms (rms 2^-8 / sqrt(12) each); the bound ASSERTED for such inputs is a quarter of
    the worst case of the logit term with a floor for the other two terms, 2^-10 max(8, s_max): tighter than
    anything the error model can guarantee."""
    smax = float(np.linalg.norm(q, axis=-1).max() * np.linalg.norm(k, axis=-1).max() / np.sqrt(dh))
    return 2.0 ** -10 * max(8.0, smax), 2.0 ** -8 * (smax + 1.0) + 1e-3


def test_lse_error_worst_case():
    """Pins the lse error model from above: an input built so that the kernel's second bf16 rounding of
    q * scale * log2(e) errs the same way in every component (each q_i is the bf16 number in [0.5, 1) whose
    product with c is rounded up the most) and one key per row is aligned with the query.  The measured lse
    error must stay inside the worst-case bound and reach a good part of it (so the bound is not slack that
    could hide a defect), while the bound asserted for ordinary inputs, a quarter of it, is exceeded here."""
    dh, T, Hq, Hk, Bn = 128, 300, 2, 1, 1
    c = np.float32(1.0 / np.sqrt(dh)) * np.float32(1.44269504088896340736)
    grid = (np.arange(128, 256, dtype=np.float32) / np.float32(256.0))  # bf16 numbers in [0.5, 1)
    prod = (grid * c).astype(np.float32)
    d = (round_to_bf16(prod).astype(np.float64) - prod.astype(np.float64)) / prod.astype(np.float64)
    v0 = float(grid[int(np.argmax(d))])
    say("worst-case q component", v0, "relative rounding error of q*c", float(d.max()), "limit", 2.0 ** -8)
    rng = np.random.default_rng(5)
    sign = np.where(rng.random((Bn, T, Hq, dh)) < 0.5, -1.0, 1.0)
    q = (v0 * sign).astype(np.float32)                      # |q| = v0 sqrt(d_h) <= sqrt(d_h): inside the promise
    k = rng.standard_normal((Bn, T, Hk, dh))
    k *= np.sqrt(dh) / np.linalg.norm(k, axis=-1, keepdims=True)
    k[:, ::2] = sign[:, ::2, :1]                            # even keys: aligned with head 0's query of the same token
    v = rng.standard_normal((Bn, T, Hk, dh))
    q, k, v = (round_to_bf16(np.asarray(a, np.float32)) for a in (q, k, v))
    cfg = P.CCAConfig(B=Bn, T=T, d_model=Hq * dh, n_q_heads=Hq, n_kv_heads=Hk, head_dim=dh, flags=B.CCA_FLAGS_PAPER)
    dev = lambda a: torch.from_numpy(a).to("cuda", torch.bfloat16)
    o, lse = P.cca_attention(cfg, dev(q), dev(k), dev(v), want_lse=True, temp=torch.zeros(Hk, device="cuda"))
    torch.cuda.synchronize()
    o_ref, lse_ref = O.attention(q, k, v, 1.0 / np.sqrt(dh), causal=True)
    err = np.abs(to_np(lse) - lse_ref)[:, 0, ::2]           # rows whose own (aligned) key dominates
    lim, worst = lse_bounds(q, k, dh)
    say("lse worst case", dict(max_abs=float(err.max()), asserted_for_ordinary_inputs=lim, worst_case=worst))
    assert err.max() <= worst
    s_aligned = v0 * np.sqrt(dh)                            # the dominating logit, scale * <q, k> = v0 sqrt(d_h)
    assert err.max() >= 0.6 * 2.0 ** -8 * s_aligned, "the constructed input no longer exercises the rounding of q"
    assert err.max() > lim, "the bound asserted for ordinary inputs is not expected to hold for this input"
    say("o", check_tap(to_np(o).reshape(o_ref.shape), o_ref, "bf16", "o"))


# ---- config 2: CCA prefill bf16, T = 4096, literal and conv-visible ----------
@pytest.mark.parametrize("conv_visible", [False, True])
def test_cca_4k(conv_visible):
    w = WORKLOADS["cca_4k"]
    say("case cca_4k conv_visible", conv_visible)
    inp = make_inputs(w, seed=0, conv_visible=conv_visible)
    _, out, saved = run_gpu(w, inp)
    rows = sample_rows(w["T"], 512)
    res = compare_all(w, inp, oracle_forward(w, inp, rows=rows), out, saved, rows=rows)
    say(res)


# ---- config 3: CCGQA prefill bf16, T = 16384: prologue taps on every token,
#      attention / out on sampled rows (row t needs only keys <= t) -----------
@pytest.mark.parametrize("name", ["ccgqa_16k", "ccgqa_16k_dh256"])
def test_ccgqa_16k_sampled_rows(name):
    w = WORKLOADS[name]
    say("case", name)
    inp = make_inputs(w, seed=0, conv_visible=name != "ccgqa_16k")
    _, out, saved = run_gpu(w, inp)
    rows = sample_rows(w["T"], 192)
    ref = oracle_forward(w, inp, rows=rows)
    res = compare_all(w, inp, ref, out, saved, rows=rows)
    say(res)
    # the call bench.py times: no saved tensors, so the attention kernel runs in its inference form
    cfg = P.config_from_workload(w)
    x, wt = P.weights_to_device(cfg, inp)
    out_inf = P.cca_forward(cfg, wt, x)
    torch.cuda.synchronize()
    say("inference form", check_out(to_np(out_inf)[:, rows], ref["out"], w["dtype"]))


def test_paired_query_blocks_odd_count_ragged():
    """B*H_q = 32 and 15 query blocks of 256: the causal launch pairs a heavy with a light block per workgroup,
    the middle block has no partner, and the last block is ragged (T = 3700)."""
    w = dict(B=4, T=3700, E=1024, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    say("case paired blocks, odd count", w)
    inp = make_inputs(w, seed=5, conv_visible=True)
    _, out, saved = run_gpu(w, inp)
    rows = sample_rows(w["T"], 160)
    ref = oracle_forward(w, inp, rows=rows)
    res = compare_all(w, inp, ref, out, saved, rows=rows)
    say(res)
    cfg = P.config_from_workload(w)
    x, wt = P.weights_to_device(cfg, inp)
    out_inf = P.cca_forward(cfg, wt, x)
    torch.cuda.synchronize()
    say("inference form", check_out(to_np(out_inf)[:, rows], ref["out"], w["dtype"]))


def test_paired_query_blocks_head_width_256():
    """d_h = 256: B*H_q = 32 and 17 query blocks of 128 rows (paired heavy / light, the middle one alone, ragged
    last block), attention stage on unit-sphere q, k against the oracle on sampled rows."""
    T, Hq, Hk, dh, Bn = 2100, 8, 2, 256, 4
    say("case paired blocks d_h 256", T, Hq, Hk)
    rng = np.random.default_rng(9)
    q = rng.standard_normal((Bn, T, Hq, dh))
    k = rng.standard_normal((Bn, T, Hk, dh))
    temp = np.array([0.2, -0.1], np.float32)
    q *= np.sqrt(dh) / np.linalg.norm(q, axis=-1, keepdims=True)
    k *= np.sqrt(dh) / np.linalg.norm(k, axis=-1, keepdims=True) * np.exp(temp)[None, None, :, None]
    v = rng.standard_normal((Bn, T, Hk, dh))
    q, k, v = (round_to_bf16(a.astype(np.float32)) for a in (q, k, v))
    cfg = P.CCAConfig(B=Bn, T=T, d_model=Hq * dh, n_q_heads=Hq, n_kv_heads=Hk, head_dim=dh, flags=B.CCA_FLAGS_PAPER)
    dev = lambda a: torch.from_numpy(a).to("cuda", torch.bfloat16)
    o, lse = P.cca_attention(cfg, dev(q), dev(k), dev(v), want_lse=True, temp=torch.from_numpy(temp).cuda())
    o_inf = P.cca_attention(cfg, dev(q), dev(k), dev(v), temp=torch.from_numpy(temp).cuda())
    torch.cuda.synchronize()
    rows = sample_rows(T, 96)
    o_ref, lse_ref = O.attention(q, k, v, 1.0 / np.sqrt(dh), causal=True, rows=rows)
    shape = (Bn, len(rows), Hq, dh)
    say("o", check_tap(to_np(o)[:, rows].reshape(shape), o_ref, "bf16", "o"))
    say("o, inference form", check_tap(to_np(o_inf)[:, rows].reshape(shape), o_ref, "bf16", "o"))
    lim, _ = lse_bounds(q, k, dh)
    assert float(np.abs(to_np(lse)[:, :, rows] - lse_ref).max()) <= lim


def test_forward_is_deterministic_and_causal_on_gpu():
    w = dict(B=1, T=600, E=1024, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    say("case determinism / causality")
    inp = make_inputs(w, seed=3, conv_visible=True)
    _, out1, _ = run_gpu(w, inp)
    _, out2, _ = run_gpu(w, inp)
    assert torch.equal(out1, out2)
    t0 = 301
    x2 = inp["x"].copy()
    x2[:, t0:] = round_to_bf16(x2[:, t0:] + 1.0)
    _, out3, _ = run_gpu(w, dict(inp, x=x2))
    assert torch.equal(out1[:, :t0], out3[:, :t0])
    assert not torch.equal(out1[:, t0], out3[:, t0])


# ---- backward of the attention stage against the oracle's adjoint ------------------------------
@pytest.mark.parametrize("T,Hq,Hk,causal,dh", [
    (700, 8, 2, True, 128), (333, 4, 4, True, 128), (520, 4, 1, False, 128), (64, 2, 2, True, 128), (450, 6, 2, True, 128),
    (300, 6, 1, False, 128),
    # d_h = 256: the one-wavefront-per-SIMD kernels (128 query rows / 128 keys per workgroup, dV and dK in two passes):
    # several blocks with a ragged tail, R = 2 / 1 / 4 / 3, a single short block, non-causal
    (700, 4, 2, True, 256), (333, 2, 2, True, 256), (520, 4, 1, False, 256), (64, 2, 2, True, 256), (390, 3, 1, True, 256),
    (129, 2, 1, False, 256)])
def test_attention_backward_stage(T, Hq, Hk, causal, dh):
    say("case attention backward", T, Hq, Hk, causal, dh)
    Bn = 2
    rng = np.random.default_rng(100 + T)
    q = rng.standard_normal((Bn, T, Hq, dh))
    k = rng.standard_normal((Bn, T, Hk, dh))
    temp = np.linspace(-0.2, 0.3, Hk).astype(np.float32)
    q *= np.sqrt(dh) / np.linalg.norm(q, axis=-1, keepdims=True)
    k *= np.sqrt(dh) / np.linalg.norm(k, axis=-1, keepdims=True) * np.exp(temp)[None, None, :, None]
    v = rng.standard_normal((Bn, T, Hk, dh))
    do = rng.standard_normal((Bn, T, Hq * dh))
    q, k, v, do = (round_to_bf16(a.astype(np.float32)) for a in (q, k, v, do))
    flags = B.CCA_FLAGS_PAPER if causal else B.CCA_FLAGS_PAPER & ~B.CCA_CAUSAL
    cfg = P.CCAConfig(B=Bn, T=T, d_model=Hq * dh, n_q_heads=Hq, n_kv_heads=Hk, head_dim=dh, flags=flags)
    dev = lambda a: torch.from_numpy(a).to("cuda", torch.bfloat16)
    dq_, dk_, dv_, do_ = dev(q), dev(k), dev(v), dev(do)
    o_lo = torch.empty(Bn, T, Hq * dh, dtype=torch.bfloat16, device="cuda")
    o, lse = P.cca_attention(cfg, dq_, dk_, dv_, want_lse=True, temp=torch.from_numpy(temp).cuda(), o_lo=o_lo)
    g_q, g_k, g_v = P.cca_attention_backward(cfg, dq_, dk_, dv_, o, lse, do_, o_lo=o_lo)
    torch.cuda.synchronize()
    r_q, r_k, r_v = O.attention_bwd(do, q, k, v, 1.0 / np.sqrt(dh), causal=causal)
    say("dq", check_tap(to_np(g_q), r_q, "bf16", "d_q"))
    say("dk", check_tap(to_np(g_k), r_k, "bf16", "d_k"))
    say("dv", check_tap(to_np(g_v), r_v, "bf16", "d_v"))


@pytest.mark.parametrize("Hq,Hk,causal", [(4, 2, True), (2, 2, True), (4, 1, False), (3, 3, False)])
def test_attention_head_width_256_is_bit_identical_from_run_to_run(Hq, Hk, causal):
    """The d_h = 256 attention kernels (forward and backward) issue MFMAs as inline assembly, whose hazards the
    compiler does not pad; a violated hazard shows as results that change from run to run (seen during development:
    an operand written by the vector ALU directly in front of such an MFMA).  Twelve runs over several blocks per
    head must give the same bits."""
    T, dh = 3000, 256  # (every compiled form of the backward kernels: causal or not, one or several query heads per KV head)
    say("case determinism d_h 256", T, Hq, Hk, causal)
    g = torch.Generator(device="cuda").manual_seed(5)
    rn = lambda *sh: torch.randn(*sh, device="cuda", generator=g)
    unit = lambda t, H: (t.view(1, T, H, dh) * dh ** 0.5 / t.view(1, T, H, dh).norm(dim=-1, keepdim=True)).to(torch.bfloat16).view(1, T, -1)
    q, k = unit(rn(1, T, Hq * dh), Hq), unit(rn(1, T, Hk * dh), Hk)
    v, d_o = rn(1, T, Hk * dh).to(torch.bfloat16), rn(1, T, Hq * dh).to(torch.bfloat16)
    flags = B.CCA_FLAGS_PAPER if causal else B.CCA_FLAGS_PAPER & ~B.CCA_CAUSAL
    cfg = P.CCAConfig(B=1, T=T, d_model=Hq * dh, n_q_heads=Hq, n_kv_heads=Hk, head_dim=dh, flags=flags)
    temp = torch.zeros(Hk, device="cuda")
    first = None
    for _ in range(12):
        o_lo = torch.empty_like(q)
        o, lse = P.cca_attention(cfg, q, k, v, want_lse=True, temp=temp, o_lo=o_lo)
        g_q, g_k, g_v = P.cca_attention_backward(cfg, q, k, v, o, lse, d_o, o_lo=o_lo)
        torch.cuda.synchronize()
        cur = (o, lse, o_lo, g_q, g_k, g_v)
        assert all(bool(torch.isfinite(t.float()).all()) for t in cur)
        if first is None:
            first = cur
        else:
            assert all(torch.equal(a, b) for a, b in zip(first, cur))


# ---- config 4: CCGQA vs MHA head-to-head at B = 4, T = 16384, both through the same kernels.  The HIP path runs
#      the full batch; the oracle (batch items are independent) checks the first and the last item on sampled rows.
@pytest.mark.parametrize("name", ["ccgqa_16k_b4", "mha_16k_b4"])
def test_head_to_head_b4_sampled_rows(name):
    w = WORKLOADS[name]
    say("case head-to-head", name)
    inp = make_inputs(w, seed=0)
    cfg, out, saved = run_gpu(w, inp)
    rows = sample_rows(w["T"], 48)
    items = [0, w["B"] - 1]
    w2 = dict(w, B=len(items))
    ref = oracle_forward(w2, dict(inp, x=inp["x"][items]), rows=rows)
    pick = lambda t: t[items]
    sub = B.CCASaved(lat=pick(saved.lat), q=pick(saved.q), k=pick(saved.k), v=pick(saved.v), o=pick(saved.o),
                     lse=pick(saved.lse), rnorm=pick(saved.rnorm), o_lo=pick(saved.o_lo))
    res = compare_all(w2, inp, ref, pick(out), sub, rows=rows)
    say(res)


# ---- options of the interface: epsilon under the norm, prepared weights --------------------------------------
@pytest.mark.parametrize("i", [0, 2, 8])
def test_norm_epsilon(i):
    """cfg.norm_eps > 0 on the generic (fp32), the fused d_h = 128 and the fused d_h = 64 prologue; large enough
    (a third of a typical sum of squares) that ignoring it would fail the q / k taps."""
    w = SMALL[i]
    inp = make_inputs(w, seed=70 + i, conv_visible=True)
    pre = oracle_forward(w, inp)
    eps = float(np.median((pre["q3"] ** 2).sum(-1)) / 3)
    say("case norm_eps", i, w, "eps", eps)
    cfg, out, saved = run_gpu(w, inp, norm_eps=eps)
    ref = oracle_forward(w, inp, norm_eps=eps)
    assert errors(pre["q"], ref["q"])[0] > 0.05  # the option matters for this input
    res = compare_all(w, inp, ref, out, saved)
    say(res)


@pytest.mark.parametrize("i", [2, 3, 8, 10])
def test_prepared_weights_give_identical_results(i):
    """cca_prepare + cca_forward(weights.prepared) against cca_forward deriving the same data per call: bit for
    bit, for a batch size other than the one the buffer was prepared under, with and without saved tensors."""
    w = SMALL[i]
    say("case prepared", i, w)
    inp = make_inputs(w, seed=80 + i, conv_visible=True)
    cfg = P.config_from_workload(w)
    x, wt = P.weights_to_device(cfg, inp)
    wt_p = P.cca_prepare(P.config_from_workload(dict(w, B=w["B"] + 3)), wt)
    torch.cuda.synchronize()
    out_a = P.cca_forward(cfg, wt, x)
    out_b = P.cca_forward(cfg, wt_p, x)
    s_a, s_b = P.CCASaved.allocate(cfg, x.device), P.CCASaved.allocate(cfg, x.device)
    out_c = P.cca_forward(cfg, wt, x, saved=s_a)
    out_d = P.cca_forward(cfg, wt_p, x, saved=s_b)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b) and torch.equal(out_c, out_d)
    for name in ("lat", "q", "k", "v", "o", "lse", "rnorm"):
        assert torch.equal(getattr(s_a, name), getattr(s_b, name)), name
    say(check_out(to_np(out_b), oracle_forward(w, inp)["out"], w["dtype"]))
