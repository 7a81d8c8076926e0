"""GPU parity of the decode step: by causality, the output for the token at position t equals row t of the whole
block applied to tokens 0..t, so the oracle is the forward oracle (fp64) on the same seeded inputs."""
import sys

import numpy as np
import pytest
import torch

import paper_2510_04476_amd as P
from paper_2510_04476_amd import binding as B
from synth_inputs import make_inputs
from util import check_out, check_tap, oracle_forward, to_np

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def decode_all(w, inp, start=0, flags=None, **cfg_kw):
    """Prefill tokens [0, start) with cca_forward, then decode tokens start..T-1 one by one.  Returns out
    (B, T - start, E) and the final state."""
    kw = dict(cfg_kw) if flags is None else dict(cfg_kw, flags=flags)
    cfg = P.config_from_workload(w, **kw)
    x, wt = P.weights_to_device(cfg, inp)
    state = P.CCADecodeState.allocate(cfg, x.device)
    if start > 0:
        wp = dict(w, T=start)
        cfgp = P.config_from_workload(wp, **kw)
        saved = P.CCASaved.allocate(cfgp, x.device)
        P.cca_forward(cfgp, wt, x[:, :start].contiguous(), saved=saved)
        state.load_prefill(saved, start)
    outs = []
    for t in range(start, w["T"]):
        outs.append(P.cca_decode_step(cfg, wt, x[:, t].contiguous(), state, t))
    torch.cuda.synchronize()
    return torch.stack(outs, dim=1), state


CASES = [
    dict(B=2, T=37, E=256, Hq=4, Hk=2, dh=32, k_seq=2, k_ch=2, dtype="f32", paper_flags=True),
    dict(B=1, T=70, E=256, Hq=2, Hk=1, dh=64, k_seq=3, k_ch=2, dtype="f32", paper_flags=True),
    dict(B=2, T=90, E=1024, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=3, T=40, E=384, Hq=3, Hk=3, dh=128, k_seq=4, k_ch=1, dtype="bf16", paper_flags=True),
    dict(B=1, T=33, E=512, Hq=2, Hk=1, dh=256, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=1, T=20, E=2048, Hq=16, Hk=1, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),  # R = 16 > 8
    # batch above 32 rows (two row blocks in the projections), R = 3, projection widths that are not multiples of
    # 128 and a contraction length that is not a multiple of 16
    dict(B=40, T=6, E=264, Hq=3, Hk=1, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),
    dict(B=20, T=5, E=256, Hq=4, Hk=2, dh=32, k_seq=2, k_ch=2, dtype="f32", paper_flags=True),   # fp32, 17..32 rows
    dict(B=33, T=4, E=248, Hq=2, Hk=2, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True),  # 33 rows, widths 8 * odd
]


@pytest.mark.parametrize("i", range(len(CASES)))
def test_decode_from_scratch_matches_forward_oracle(i):
    w = CASES[i]
    say("case decode from scratch", i, w)
    inp = make_inputs(w, seed=70 + i, conv_visible=True)
    out, state = decode_all(w, inp)
    ref = oracle_forward(w, inp)
    say(check_out(to_np(out), ref["out"], w["dtype"]))
    # the cache holds what the prefill prologue would have written
    say(check_tap(to_np(state.k_cache), ref["k"], w["dtype"], "k_cache"))
    say(check_tap(to_np(state.v_cache), ref["v"], w["dtype"], "v_cache"))


@pytest.mark.parametrize("i", [0, 2, 3])
@pytest.mark.parametrize("start", [1, 17])
def test_decode_after_prefill(i, start):
    w = CASES[i]
    say("case decode after prefill", i, "start", start, w)
    inp = make_inputs(w, seed=80 + i, conv_visible=True)
    out, _ = decode_all(w, inp, start=start)
    ref = oracle_forward(w, inp)
    say(check_out(to_np(out), ref["out"][:, start:], w["dtype"]))


@pytest.mark.parametrize("name", ["no_conv", "no_v_shift", "no_norm", "rope_interleaved", "mha"])
def test_decode_flags(name):
    F = B.CCA_FLAGS_PAPER
    flags, okw = {
        "no_conv": (F & ~(B.CCA_CONV_SEQ | B.CCA_CONV_CH), dict(use_conv_seq=False, use_conv_ch=False)),
        "no_v_shift": (F & ~B.CCA_V_SHIFT, dict(use_v_shift=False)),
        "no_norm": (F & ~(B.CCA_QK_NORM | B.CCA_KEY_TEMP), dict(use_qk_norm=False, use_key_temp=False)),
        "rope_interleaved": (F | B.CCA_ROPE_INTERLEAVED, dict(rope_interleaved=True)),
        "mha": (B.CCA_FLAGS_MHA, dict(use_conv_seq=False, use_conv_ch=False, use_qk_mean=False, use_v_shift=False,
                                       use_qk_norm=False, use_key_temp=False, use_rope=False)),
    }[name]
    w = dict(B=2, T=45, E=512, Hq=4, Hk=2, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    say("case decode flags", name, w)
    inp = make_inputs(w, seed=91, conv_visible=True)
    out, _ = decode_all(w, inp, flags=flags)
    ref = oracle_forward(w, inp, **okw)
    say(check_out(to_np(out), ref["out"], w["dtype"]))


def test_decode_norm_epsilon():
    """cfg.norm_eps reaches the decode prologue (prefill of 9 tokens by the fused kernel, then token by token)."""
    w = dict(B=2, T=30, E=512, Hq=4, Hk=2, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    inp = make_inputs(w, seed=92, conv_visible=True)
    eps = float(np.median((oracle_forward(w, inp)["q3"] ** 2).sum(-1)) / 3)
    say("case decode norm_eps", w, eps)
    out, _ = decode_all(w, inp, start=9, norm_eps=eps)
    ref = oracle_forward(w, inp, norm_eps=eps)
    say(check_out(to_np(out), ref["out"][:, 9:], w["dtype"]))


def test_decode_long_cache_split_over_workgroups():
    """A long cache (several splits of the key range, ragged last split), decoded after a prefill."""
    w = dict(B=2, T=3000, E=1024, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    start = 2990
    say("case decode long cache", w)
    inp = make_inputs(w, seed=95)
    out, _ = decode_all(w, inp, start=start)
    rows = np.arange(start, w["T"])
    ref = oracle_forward(w, inp, rows=rows)
    say(check_out(to_np(out), ref["out"], w["dtype"]))


def test_decode_bench_configuration_sampled():
    """The configuration bench.py times (32 sequences, a 16k cache, the headline layer): two distinct sequences
    alternate over the batch; the oracle computes the last row of each."""
    from synth_inputs import WORKLOADS
    w0 = WORKLOADS["ccgqa_16k"]
    w2 = dict(w0, B=2)
    T, Bd = w0["T"], 32
    say("case decode at the benchmark configuration", w2, "batch", Bd)
    inp = make_inputs(w2, seed=7)
    cfg2 = P.config_from_workload(dict(w2, T=T - 1))
    x, wt = P.weights_to_device(P.config_from_workload(w2), inp)
    saved = P.CCASaved.allocate(cfg2, x.device)
    P.cca_forward(cfg2, wt, x[:, :T - 1].contiguous(), saved=saved)
    cfg = P.config_from_workload(dict(w0, B=Bd))
    state = P.CCADecodeState.allocate(cfg, x.device)
    two = P.CCADecodeState.allocate(P.config_from_workload(w2), x.device)
    two.load_prefill(saved, T - 1)
    for b in range(Bd):
        state.k_cache[b].copy_(two.k_cache[b % 2])
        state.v_cache[b].copy_(two.v_cache[b % 2])
        state.lat_ring[b].copy_(two.lat_ring[b % 2])
    del two, saved
    x_new = x[:, T - 1].repeat(Bd // 2, 1).contiguous()  # rows b -> sequence b % 2
    out = P.cca_decode_step(cfg, wt, x_new, state, T - 1)
    torch.cuda.synchronize()
    ref = oracle_forward(w2, inp, rows=np.array([T - 1]))["out"][:, 0]  # (2, E)
    got = to_np(out)
    say(check_out(got, np.tile(ref, (Bd // 2, 1)), "bf16"))
    assert np.array_equal(got[0], got[2]) and np.array_equal(got[1], got[31]), "same sequence, different result"


@pytest.mark.parametrize("i", [0, 2, 3, 6])
def test_decode_ragged_batch_matches_forward_oracle(i):
    """Sequences of one batch at different positions (cca_decode_step_ragged).  Sequence b starts delay[b] calls
    late - until then it decodes its token 0 at position 0 again, which rewrites the same cache row and ring slot -
    and after its last token it repeats that one, so from the second call on every call carries a different
    position, ring slot and cache length per sequence.  Every row of every sequence is compared with the oracle."""
    w = CASES[i]
    say("case ragged decode", i, w)
    inp = make_inputs(w, seed=110 + i, conv_visible=True)
    cfg = P.config_from_workload(w)
    x, wt = P.weights_to_device(cfg, inp)
    state = P.CCADecodeState.allocate(cfg, x.device)
    Bn, T = w["B"], w["T"]
    delay = np.array([(5 * b + 3 * (b % 2)) % 9 for b in range(Bn)])
    got = torch.empty(Bn, T, w["E"], dtype=x.dtype, device=x.device)
    seen = np.zeros((Bn, T), bool)
    rows = torch.arange(Bn, device=x.device)
    for s in range(T + int(delay.max())):
        pos = np.clip(s - delay, 0, T - 1)
        pos_d = torch.tensor(pos, dtype=torch.int32, device=x.device)
        out = P.cca_decode_step_ragged(cfg, wt, x[rows, pos_d.long()].contiguous(), state, pos_d, int(pos.max()))
        got[rows, pos_d.long()] = out
        seen[np.arange(Bn), pos] = True
    torch.cuda.synchronize()
    assert seen.all()
    ref = oracle_forward(w, inp)
    say(check_out(to_np(got), ref["out"], w["dtype"]))
    say(check_tap(to_np(state.k_cache), ref["k"], w["dtype"], "k_cache"))
    say(check_tap(to_np(state.v_cache), ref["v"], w["dtype"], "v_cache"))


def test_decode_ragged_long_and_short_sequence_share_a_call():
    """One sequence near the end of a 3000-token cache (several splits of the key range) and one 40 tokens long
    (all but the first split empty) in the same call; positions beyond the host's bound are clamped to it."""
    w = dict(B=2, T=3000, E=1024, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    say("case ragged decode, long and short", w)
    inp = make_inputs(w, seed=97)
    cfg = P.config_from_workload(w)
    x, wt = P.weights_to_device(cfg, inp)
    saved = P.CCASaved.allocate(cfg, x.device)
    P.cca_forward(cfg, wt, x, saved=saved)
    state = P.CCADecodeState.allocate(cfg, x.device)
    state.k_cache.copy_(saved.k)   # rows at and beyond a sequence's position are rewritten or never read
    state.v_cache.copy_(saved.v)
    ring = state.lat_ring.shape[1]
    start = np.array([2990, 40])
    for b in range(2):
        for t in range(start[b] - ring, start[b]):
            state.lat_ring[b, t % ring].copy_(saved.lat[b, t])
    outs, n_steps = [], 4
    for s in range(n_steps):
        pos = start + s
        pos_d = torch.tensor(pos, dtype=torch.int32, device=x.device)
        x_new = torch.stack([x[b, pos[b]] for b in range(2)]).contiguous()
        outs.append(P.cca_decode_step_ragged(cfg, wt, x_new, state, pos_d, int(pos.max())))
    # an entry above max_pos is clamped to max_pos: the same call as the last one, the short sequence's entry too large
    pos = start + n_steps - 1
    bad = torch.tensor([pos[0], 10 ** 6], dtype=torch.int32, device=x.device)
    x_new = torch.stack([x[0, pos[0]], x[1, pos[0]]]).contiguous()
    clamped = P.cca_decode_step_ragged(cfg, wt, x_new, state, bad, int(pos[0]))
    torch.cuda.synchronize()
    want = np.concatenate([start[0] + np.arange(n_steps), start[1] + np.arange(n_steps)])
    ref = oracle_forward(w, inp, rows=want)["out"]   # (2, 2 * n_steps, E)
    got = to_np(torch.stack(outs, dim=1))            # (2, n_steps, E)
    say(check_out(got[0], ref[0, :n_steps], "bf16"))
    say(check_out(got[1], ref[1, n_steps:], "bf16"))
    say(check_out(to_np(clamped)[0], ref[0, n_steps - 1], "bf16"))
    assert torch.isfinite(clamped.float()).all()


def test_decode_step_and_prefill_replay_in_a_hip_graph():
    """The library allocates nothing, never synchronises and enqueues only kernels on the caller's stream, so a call
    can be captured into a HIP graph: every replay, with eager calls in between, gives the eager result bit for bit."""
    w = CASES[2]
    inp = make_inputs(w, seed=72, conv_visible=True)
    cfg = P.config_from_workload(w)
    x, wt = P.weights_to_device(cfg, inp)
    saved = P.CCASaved.allocate(cfg, x.device)
    P.cca_forward(cfg, wt, x, saved=saved)
    state = P.CCADecodeState.allocate(cfg, x.device)
    pos = w["T"] - 1
    state.load_prefill(saved, pos)
    x_new = x[:, pos].contiguous()
    ws = P.new_workspace(cfg, x.device)
    out_e, out_g = torch.empty_like(x_new), torch.empty_like(x_new)
    full_e, full_g = torch.empty_like(x), torch.empty_like(x)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):  # warm-up on the capture stream
        P.cca_decode_step(cfg, wt, x_new, state, pos, out=out_g)
        P.cca_forward(cfg, wt, x, out=full_g, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        P.cca_decode_step(cfg, wt, x_new, state, pos, out=out_g)
        P.cca_forward(cfg, wt, x, out=full_g, workspace=ws)
    torch.cuda.synchronize()
    for rep in range(3):
        out_g.zero_()
        full_g.zero_()
        graph.replay()
        torch.cuda.synchronize()
        P.cca_decode_step(cfg, wt, x_new, state, pos, out=out_e)
        P.cca_forward(cfg, wt, x, out=full_e, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e) and torch.equal(full_g, full_e), f"replay {rep} differs from the eager call"
    ref = oracle_forward(w, inp)
    say(check_out(to_np(full_g), ref["out"], w["dtype"]))
    say(check_out(to_np(out_g), ref["out"][:, pos], w["dtype"]))


def test_decode_rejects_bad_arguments():
    w = CASES[2]
    cfg = P.config_from_workload(w)
    inp = make_inputs(w, seed=1)
    x, wt = P.weights_to_device(cfg, inp)
    state = P.CCADecodeState.allocate(cfg, x.device)
    with pytest.raises(P.CCAError):
        P.cca_decode_step(cfg, wt, x[:, 0].contiguous(), state, w["T"])  # position outside the cache
    with pytest.raises(P.CCAError):
        P.cca_decode_step(cfg, wt, x[:, 0].contiguous(), state, -1)
    small = P.CCADecodeState(state.k_cache, state.v_cache, state.lat_ring, state.workspace[:16])
    with pytest.raises(P.CCAError):
        P.cca_decode_step(cfg, wt, x[:, 0].contiguous(), small, 0)
    pos_d = torch.zeros(w["B"], dtype=torch.int32, device=x.device)
    with pytest.raises(P.CCAError):
        P.cca_decode_step_ragged(cfg, wt, x[:, 0].contiguous(), state, pos_d, w["T"])  # bound outside the cache
    with pytest.raises(P.CCAError):
        P.cca_decode_step_ragged(cfg, wt, x[:, 0].contiguous(), small, pos_d, 0)
