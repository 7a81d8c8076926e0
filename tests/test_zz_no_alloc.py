"""cca_decode_step_static (the entry point that allocates nothing: its scratch is an array inside the library)
against cca_decode_step with a caller's workspace: bit for bit, on two calls in a row, the second with a smaller
input (fewer sequences, a shorter cache prefix), so that whatever the first call left in the shared array is
still there when the second one runs."""
import ctypes as C
import sys

import numpy as np
import pytest
import torch

import paper_2510_04476_amd as P
from paper_2510_04476_amd import binding as B
from synth_inputs import make_inputs
from util import check_out, oracle_forward, to_np

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def one_step(w, inp, pos, static):
    """Prefill tokens [0, pos) with cca_forward, then one decode step for token `pos` through either entry point."""
    cfg = P.config_from_workload(w)
    x, wt = P.weights_to_device(cfg, inp)
    state = P.CCADecodeState.allocate(cfg, x.device)
    wp = dict(w, T=pos)
    cfgp = P.config_from_workload(wp)
    saved = P.CCASaved.allocate(cfgp, x.device)
    P.cca_forward(cfgp, wt, x[:, :pos].contiguous(), saved=saved)
    state.load_prefill(saved, pos)
    x_new = x[:, pos].contiguous()
    out = torch.empty(cfg.B, cfg.d_model, dtype=cfg.torch_dtype, device=x.device)
    if static:
        P.cca_decode_step_static(cfg, wt, x_new, state, pos, out)
    else:
        P.cca_decode_step(cfg, wt, x_new, state, pos, out=out)
    torch.cuda.synchronize()
    return out, state


def test_static_decode_matches_workspace_decode_twice_in_a_row():
    big = dict(B=6, T=700, E=1024, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    small = dict(B=2, T=90, E=512, Hq=4, Hk=2, dh=64, k_seq=2, k_ch=2, dtype="bf16", paper_flags=True)
    for name, w in (("first call", big), ("second call, smaller input", small)):
        inp = make_inputs(w, seed=31, conv_visible=True)
        pos = w["T"] - 1
        say("case static decode", name, w, "pos", pos)
        out_s, st_s = one_step(w, inp, pos, static=True)
        out_w, st_w = one_step(w, inp, pos, static=False)
        assert torch.equal(out_s, out_w), name
        assert torch.equal(st_s.k_cache, st_w.k_cache) and torch.equal(st_s.v_cache, st_w.v_cache), name
        assert torch.equal(st_s.lat_ring, st_w.lat_ring), name
        ref = oracle_forward(w, inp, rows=np.array([pos]))
        say(check_out(to_np(out_s), ref["out"][:, 0], w["dtype"]))


def test_static_decode_rejects_what_does_not_fit():
    """A batch whose scratch exceeds the built-in array is refused with CCA_ERR_WORKSPACE before anything is
    enqueued (fake addresses are never dereferenced); validation errors come first, as for cca_decode_step."""
    lib = P.load_library()
    p = C.c_void_p(0x10000)
    w = B.cca_weights(p, p, p, p, p, None)
    st = B.cca_decode_state(p, p, p)
    huge = P.CCAConfig(B=512, T=16384, d_model=2048, n_q_heads=8, n_kv_heads=2, head_dim=128)
    need, _ = P.cca_decode_workspace_size(huge)
    assert need > P.CCA_DECODE_STATIC_BYTES
    cc = huge.c()
    assert lib.cca_decode_step_static(C.byref(cc), C.byref(w), p, C.byref(st), 0, p, None) == B.CCA_ERR_WORKSPACE
    ok = P.CCAConfig(B=2, T=64, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=64)
    assert P.cca_decode_workspace_size(ok)[0] <= P.CCA_DECODE_STATIC_BYTES
    c2 = ok.c()
    assert lib.cca_decode_step_static(C.byref(c2), C.byref(w), None, C.byref(st), 0, p, None) == B.CCA_ERR_NULL
    assert lib.cca_decode_step_static(C.byref(c2), C.byref(w), p, C.byref(st), 64, p, None) == B.CCA_ERR_SHAPE
