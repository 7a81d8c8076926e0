"""Pins of the oracle's backward pass: the paper gives no backward equations, so
the hand-derived adjoint is checked against the numerical definition (central
finite differences of the fp64 forward oracle) for every gradient, and with the
<dOut, J delta> = <J^T dOut, delta> identity at a larger size."""
import numpy as np
import pytest

from oracle import cca_oracle as O
from synth_inputs import make_inputs

W = dict(B=2, T=7, E=24, Hq=4, Hk=2, dh=4, k_seq=2, k_ch=2, dtype="f32")
KEYS = ("x", "w_down", "w_conv_seq", "w_conv_ch", "temp", "w_out")
GRAD = dict(x="d_x", w_down="d_w_down", w_conv_seq="d_w_conv_seq", w_conv_ch="d_w_conv_ch", temp="d_temp",
            w_out="d_w_out")


def fwd(inp, w, **kw):
    return O.cca_forward(*(inp[k] for k in KEYS), n_q_heads=w["Hq"], n_kv_heads=w["Hk"], head_dim=w["dh"], **kw)["out"]


def bwd(inp, w, d_out, **kw):
    return O.cca_backward(*(inp[k] for k in KEYS), d_out, n_q_heads=w["Hq"], n_kv_heads=w["Hk"], head_dim=w["dh"],
                          **kw)


def make(w, seed):
    inp = make_inputs(w, seed=seed, w_scale=0.4, conv_visible=True)
    return {k: np.asarray(v, np.float64) for k, v in inp.items()}


FLAGSETS = [
    {},
    dict(use_qk_mean=False),
    dict(use_conv_seq=False, use_v_shift=False),
    dict(use_conv_ch=False, use_rope=False),
    dict(use_qk_norm=False, use_key_temp=False),
    dict(use_key_temp=False, rope_interleaved=True),
    dict(causal=False),
    dict(norm_eps=0.7),
]


@pytest.mark.parametrize("flags", FLAGSETS)
def test_backward_matches_finite_differences(flags):
    w = W
    inp = make(w, seed=3)
    rng = np.random.default_rng(1)
    d_out = rng.standard_normal((w["B"], w["T"], w["E"]))
    g = bwd(inp, w, d_out, **flags)
    eps = 1e-6
    for key in KEYS:
        a = inp[key]
        got = g[GRAD[key]]
        idx = [tuple(rng.integers(0, s) for s in a.shape) for _ in range(12)]
        for i in idx:
            ap, am = a.copy(), a.copy()
            ap[i] += eps
            am[i] -= eps
            num = ((fwd(dict(inp, **{key: ap}), w, **flags) - fwd(dict(inp, **{key: am}), w, **flags)) * d_out).sum() / (2 * eps)
            assert abs(num - got[i]) <= 2e-6 * max(1.0, abs(num)), (key, i, num, got[i])


def test_backward_dot_product_identity():
    w = dict(B=2, T=40, E=64, Hq=4, Hk=2, dh=8, k_seq=3, k_ch=2, dtype="f32")
    inp = make(w, seed=5)
    rng = np.random.default_rng(2)
    d_out = rng.standard_normal((w["B"], w["T"], w["E"]))
    g = bwd(inp, w, d_out)
    # directional derivative along a random direction in all inputs at once
    delta = {k: rng.standard_normal(inp[k].shape) for k in KEYS}
    eps = 1e-6
    plus = {k: inp[k] + eps * delta[k] for k in KEYS}
    minus = {k: inp[k] - eps * delta[k] for k in KEYS}
    lhs = ((fwd(plus, w) - fwd(minus, w)) * d_out).sum() / (2 * eps)
    rhs = sum((g[GRAD[k]] * delta[k]).sum() for k in KEYS)
    assert abs(lhs - rhs) <= 1e-6 * abs(lhs)


def test_attention_backward_against_autograd():
    """The attention adjoint alone against reverse-mode differentiation of the library softmax attention."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(0)
    B, T, Hq, Hk, d = 2, 13, 4, 2, 8
    q, k, v, do = (rng.standard_normal(s) for s in [(B, T, Hq, d), (B, T, Hk, d), (B, T, Hk, d), (B, T, Hq, d)])
    dq, dk, dv = O.attention_bwd(do, q, k, v, 0.3, causal=True)
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (q, k, v))
    o = F.scaled_dot_product_attention(tq.transpose(1, 2), tk.transpose(1, 2).repeat_interleave(2, 1),
                                       tv.transpose(1, 2).repeat_interleave(2, 1), is_causal=True, scale=0.3)
    (o.transpose(1, 2) * torch.tensor(do)).sum().backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_backward_restricted_to_rows_equals_full_backward(causal):
    """With d_out zero outside a set of rows, the rows= shortcut (skip the other query rows) must give the same
    gradients as the full adjoint: it is what the full-size GPU parity test relies on."""
    w = dict(B=2, T=300, E=64, Hq=4, Hk=2, dh=8, k_seq=2, k_ch=2, dtype="f32")
    inp = make(w, seed=8)
    rng = np.random.default_rng(4)
    rows = np.array(sorted(rng.choice(w["T"], size=37, replace=False)))
    d_out = np.zeros((w["B"], w["T"], w["E"]))
    d_out[:, rows] = rng.standard_normal((w["B"], len(rows), w["E"]))
    full = bwd(inp, w, d_out, causal=causal)
    part = bwd(inp, w, d_out, causal=causal, rows=rows)
    for key in ("d_x", "d_w_down", "d_w_conv_seq", "d_w_conv_ch", "d_temp", "d_w_out", "d_q", "d_k", "d_v", "d_lat"):
        np.testing.assert_allclose(part[key], full[key], rtol=1e-11, atol=1e-13, err_msg=key)
