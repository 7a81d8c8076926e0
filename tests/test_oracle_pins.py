"""Pins of the fp64 oracle to things other than itself (CPU only).

Each test names the statement of the paper (or of the mathematics) it rests on.
"""
import math

import numpy as np
import pytest
import scipy.linalg
import torch
import torch.nn.functional as F

from oracle import cca_oracle as O
from synth_inputs import make_inputs, latent_dims

TINY = dict(B=2, T=24, E=48, Hq=4, Hk=2, dh=8, k_seq=2, k_ch=2, dtype="f32", paper_flags=True)


def heads(w):
    return dict(n_q_heads=w["Hq"], n_kv_heads=w["Hk"], head_dim=w["dh"])


def run(w, inp, **kw):
    return O.cca_forward(inp["x"], inp["w_down"], inp["w_conv_seq"], inp["w_conv_ch"],
                         inp["temp"], inp["w_out"], **heads(w), **kw)


ALL_OFF = dict(use_conv_seq=False, use_conv_ch=False, use_qk_mean=False, use_v_shift=False,
               use_qk_norm=False, use_key_temp=False, use_rope=False)


# --- P1: with compression 1, no convs and no extra transforms the block is
#     textbook MHA / GQA (Sec. 2.1 MHA equations; GQA paragraph) -------------
def dense_mha(x, wq, wk, wv, wo, Hq, Hk, dh, causal=True):
    """softmax(Q K^T / sqrt(d) + mask) V with the T x T matrix written out."""
    B, T, _ = x.shape
    q = (x @ wq).reshape(B, T, Hq, dh)
    k = (x @ wk).reshape(B, T, Hk, dh)
    v = (x @ wv).reshape(B, T, Hk, dh)
    out = np.zeros((B, T, Hq * dh))
    for b in range(B):
        for h in range(Hq):
            g = h // (Hq // Hk)
            s = q[b, :, h] @ k[b, :, g].T / math.sqrt(dh)
            if causal:
                s = s + np.triu(np.full((T, T), -np.inf), 1)
            p = np.exp(s - s.max(1, keepdims=True))
            p /= p.sum(1, keepdims=True)
            out[b, :, h * dh:(h + 1) * dh] = p @ v[b, :, g]
    return out @ wo


@pytest.mark.parametrize("Hq,Hk", [(4, 4), (4, 2), (4, 1)])
@pytest.mark.parametrize("causal", [True, False])
def test_reduces_to_mha_gqa(Hq, Hk, causal):
    dh, E = 8, 32                       # compression 1: Hq*dh == E
    w = dict(B=2, T=19, E=E, Hq=Hq, Hk=Hk, dh=dh, k_seq=1, k_ch=1, dtype="f32")
    inp = make_inputs(w, seed=3, w_scale=0.3)
    res = run(w, inp, causal=causal, **ALL_OFF)
    d = latent_dims(w)
    wd = inp["w_down"].astype(np.float64)
    wq, wk, wv = wd[:, :d["e_q"]], wd[:, d["e_q"]:d["e_q"] + d["e_kv"]], wd[:, d["e_q"] + d["e_kv"]:]
    ref = dense_mha(inp["x"].astype(np.float64), wq, wk, wv, inp["w_out"].astype(np.float64), Hq, Hk, dh, causal)
    np.testing.assert_allclose(res["out"], ref, rtol=1e-11, atol=1e-12)
    # the same through the library attention routine
    x = torch.from_numpy(inp["x"]).double()
    q = (x @ torch.from_numpy(wq)).view(2, 19, Hq, dh).transpose(1, 2)
    k = (x @ torch.from_numpy(wk)).view(2, 19, Hk, dh).transpose(1, 2).repeat_interleave(Hq // Hk, dim=1)
    v = (x @ torch.from_numpy(wv)).view(2, 19, Hk, dh).transpose(1, 2).repeat_interleave(Hq // Hk, dim=1)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=causal).transpose(1, 2).reshape(2, 19, -1)
    lib = (o @ torch.from_numpy(inp["w_out"]).double()).numpy()
    np.testing.assert_allclose(res["out"], lib, rtol=1e-10, atol=1e-12)


# --- P2: identity filters (last tap = 1 / identity matrix) are a no-op ------
def test_identity_convs_are_noop():
    w = TINY
    inp = make_inputs(w, seed=1, w_scale=0.2)
    e = latent_dims(w)
    w0 = np.zeros((e["e_q"] + e["e_kv"], w["k_seq"]), np.float32)
    w0[:, -1] = 1
    w1 = np.zeros((w["Hq"] + w["Hk"], w["dh"], w["dh"], w["k_ch"]), np.float32)
    w1[..., -1] = np.eye(w["dh"])
    inp_id = dict(inp, w_conv_seq=w0, w_conv_ch=w1)
    a = run(w, inp_id)
    b = run(w, inp, use_conv_seq=False, use_conv_ch=False)
    for key in ("q", "k", "v", "out"):
        assert np.array_equal(a[key], b[key]), key


def test_single_tap_conv_is_a_delay():
    """A filter with only tap 0 set delays by k-1 tokens (tap order)."""
    u = np.random.default_rng(0).standard_normal((2, 9, 6))
    w0 = np.zeros((6, 3))
    w0[:, 0] = 1.0
    y = O.conv_seq(u, w0)
    assert np.array_equal(y[:, 2:], u[:, :-2]) and not y[:, :2].any()
    u4 = u.reshape(2, 9, 2, 3)
    w1 = np.zeros((2, 3, 3, 2))
    w1[..., 0] = np.eye(3)
    y4 = O.conv_ch(u4, w1)
    assert np.array_equal(y4[:, 1:], u4[:, :-1]) and not y4[:, 0].any()


# --- P3: causality ("depth-wise causal" convs, previous-token value stream,
#     causal mask) -----------------------------------------------------------
@pytest.mark.parametrize("t0", [1, 7, 23])
def test_causality(t0):
    w = TINY
    inp = make_inputs(w, seed=2, w_scale=0.2, conv_visible=True)
    base = run(w, inp)["out"]
    x2 = inp["x"].copy()
    x2[:, t0:] += np.random.default_rng(5).standard_normal(x2[:, t0:].shape).astype(np.float32)
    pert = run(w, dict(inp, x=x2))["out"]
    assert np.array_equal(base[:, :t0], pert[:, :t0])
    # and the perturbed token itself does move (no global one-token delay)
    assert np.abs(base[:, t0] - pert[:, t0]).max() > 1e-3


def test_batch_items_do_not_leak():
    w = TINY
    inp = make_inputs(w, seed=2, w_scale=0.2, conv_visible=True)
    both = run(w, inp)["out"]
    w1 = dict(w, B=1)
    for b in range(2):
        one = run(w1, dict(inp, x=inp["x"][b:b + 1]))["out"]
        np.testing.assert_allclose(one[0], both[b], rtol=0, atol=1e-13)


# --- P4: brute-force softmax, plain Python loops ----------------------------
def test_attention_brute_force():
    rng = np.random.default_rng(0)
    B, T, Hq, Hk, d = 1, 11, 4, 2, 5
    q, k, v = (rng.standard_normal(s) * 2 for s in [(B, T, Hq, d), (B, T, Hk, d), (B, T, Hk, d)])
    scale = 0.37
    o, lse = O.attention(q, k, v, scale, causal=True)
    for h in range(Hq):
        g = h // 2
        for t in range(T):
            e = [math.exp(scale * sum(q[0, t, h, i] * k[0, s, g, i] for i in range(d))) for s in range(t + 1)]
            z = sum(e)
            for i in range(d):
                ref = sum(e[s] / z * v[0, s, g, i] for s in range(t + 1))
                assert abs(o[0, t, h, i] - ref) < 1e-12
            assert abs(lse[0, h, t] - math.log(z)) < 1e-12


def test_equal_logits_give_running_mean():
    rng = np.random.default_rng(0)
    T = 9
    q = np.zeros((1, T, 2, 4))
    k = rng.standard_normal((1, T, 2, 4))
    v = rng.standard_normal((1, T, 2, 4))
    o, _ = O.attention(q, k, v, 1.0, causal=True)
    ref = np.cumsum(v, axis=1) / np.arange(1, T + 1)[None, :, None, None]
    np.testing.assert_allclose(o, ref, atol=1e-14)


def test_row_subset_matches_full():
    rng = np.random.default_rng(0)
    q, k, v = (rng.standard_normal(s) for s in [(1, 40, 4, 8), (1, 40, 2, 8), (1, 40, 2, 8)])
    o, lse = O.attention(q, k, v, 0.3)
    rows = np.array([0, 3, 17, 39])
    o2, lse2 = O.attention(q, k, v, 0.3, rows=rows)
    np.testing.assert_allclose(o2, o[:, rows], atol=1e-15)
    np.testing.assert_allclose(lse2, lse[:, :, rows], atol=1e-15)


# --- P5: closed forms of the norm / temperature / RoPE / qk-mean steps ------
def test_norm_temperature_rope_closed_forms():
    w = TINY
    inp = make_inputs(w, seed=4, w_scale=0.2, conv_visible=True)
    r = run(w, inp)
    dh = w["dh"]
    np.testing.assert_allclose(np.linalg.norm(r["q"], axis=-1), math.sqrt(dh), rtol=1e-12)
    beta = np.exp(inp["temp"].astype(np.float64))
    np.testing.assert_allclose(np.linalg.norm(r["k"], axis=-1),
                               math.sqrt(dh) * beta[None, None, :] * np.ones(r["k"].shape[:3]), rtol=1e-12)
    # |logit| <= sqrt(d_h) * beta with scale 1/sqrt(d_h)
    s = np.einsum("bthd,bshd->bhts", r["q"], np.repeat(r["k"], 2, axis=2)) / math.sqrt(dh)
    assert (np.abs(s) <= (math.sqrt(dh) * np.repeat(beta, 2))[None, :, None, None] * (1 + 1e-12)).all()
    # m_k = (mean_{h in g} q0 + k0) / 2 since mean(broadcast(k0)) = k0
    q2 = np.zeros_like(r["q0"])
    k2 = np.zeros_like(r["k0"])
    _, mk = O.qk_mean(q2, k2, r["q0"], r["k0"])
    ref = 0.5 * (r["q0"].reshape(2, 24, 2, 2, 8).mean(3) + r["k0"])
    np.testing.assert_allclose(mk, ref, atol=1e-15)


# --- P6: at t = 0 attention has one term, so out[0] is a closed form of the
#     current-token value stream alone ("half of the heads") -----------------
def test_first_token_closed_form():
    w = TINY
    inp = make_inputs(w, seed=6, w_scale=0.2, conv_visible=True)
    r = run(w, inp)
    e = latent_dims(w)
    x0 = inp["x"][:, 0].astype(np.float64)
    wd = inp["w_down"].astype(np.float64)
    wv = wd[:, e["e_q"] + e["e_kv"]: e["e_q"] + e["e_kv"] + e["e_kv"] // 2]
    vc0 = x0 @ wv                                   # (B, e_kv/2) = KV head 0 only (Hk = 2)
    o0 = np.zeros((2, w["Hq"], w["dh"]))
    o0[:, 0], o0[:, 1] = vc0, vc0                   # q heads 0,1 share KV head 0; heads 2,3 see v[0] = 0
    ref = o0.reshape(2, -1) @ inp["w_out"].astype(np.float64)
    np.testing.assert_allclose(r["out"][:, 0], ref, atol=1e-13)



# --- P7: the two convolutions written as matrices (Sec. 2.2 convolution equation): a causal convolution along time
#     is a lower-triangular Toeplitz operator, the grouped one a block-Toeplitz operator with a dense d x d block
#     per tap; qk-mean and value-shift written index by index (qk-mean and value-shift equations) -----------------
def seq_operator(w0c, T):
    """(T, T) matrix of one channel's causal filter: entry (t, s) is the tap that reaches t - s steps back."""
    ks = len(w0c)
    col = np.zeros(T)
    col[:min(ks, T)] = w0c[::-1][:T]          # 0 steps back = last tap
    return scipy.linalg.toeplitz(col, np.zeros(T))


def ch_operator(w1h, T):
    """(T*d_out, T*d_in) matrix of one head's filter (d_out, d_in, k_ch): block (t, t - s) is the tap for s steps back."""
    kc = w1h.shape[2]
    return sum(np.kron(np.eye(T, k=-s), w1h[:, :, kc - 1 - s]) for s in range(min(kc, T)))


def test_conv_seq_is_a_lower_triangular_toeplitz_product():
    rng = np.random.default_rng(21)
    B, T, C, ks = 2, 9, 5, 3
    u, w0 = rng.standard_normal((B, T, C)), rng.standard_normal((C, ks))
    y = O.conv_seq(u, w0)
    for c in range(C):
        L = seq_operator(w0[c], T)
        assert np.array_equal(np.triu(L, 1), np.zeros((T, T)))          # causal
        np.testing.assert_allclose(y[:, :, c], u[:, :, c] @ L.T, rtol=1e-12, atol=1e-14)


def test_conv_ch_is_a_block_toeplitz_product():
    rng = np.random.default_rng(22)
    B, T, H, d, kc = 2, 7, 3, 4, 2
    u, w1 = rng.standard_normal((B, T, H, d)), rng.standard_normal((H, d, d, kc))
    y = O.conv_ch(u, w1)
    for h in range(H):
        M = ch_operator(w1[h], T)
        for b in range(B):
            np.testing.assert_allclose(y[b, :, h].ravel(), M @ u[b, :, h].ravel(), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("which", ["seq", "ch"])
def test_each_convolution_against_the_library_grouped_conv1d(which):
    """One step at a time against the library routine: a left-padded grouped cross-correlation."""
    rng = np.random.default_rng(24)
    B, T, H, d, k = 2, 13, 3, 4, 3
    u = rng.standard_normal((B, T, H, d))
    ut = F.pad(torch.from_numpy(u.reshape(B, T, H * d)).transpose(1, 2), (k - 1, 0))
    if which == "seq":
        w0 = rng.standard_normal((H * d, k))
        got = O.conv_seq(u.reshape(B, T, H * d), w0)
        want = F.conv1d(ut, torch.from_numpy(w0)[:, None, :], groups=H * d)
    else:
        w1 = rng.standard_normal((H, d, d, k))
        got = O.conv_ch(u, w1).reshape(B, T, H * d)
        want = F.conv1d(ut, torch.from_numpy(w1.reshape(H * d, d, k)), groups=H)
    np.testing.assert_allclose(got, want.transpose(1, 2).numpy(), rtol=1e-12, atol=1e-14)


def test_qk_mean_and_value_shift_index_by_index():
    rng = np.random.default_rng(23)
    B, T, Hq, Hk, d = 2, 5, 6, 2, 4
    R = Hq // Hk
    q0, k0 = rng.standard_normal((B, T, Hq, d)), rng.standard_normal((B, T, Hk, d))
    q2, k2 = rng.standard_normal((B, T, Hq, d)), rng.standard_normal((B, T, Hk, d))
    q3, k3 = O.qk_mean(q2, k2, q0, k0)
    for h in range(Hq):
        np.testing.assert_allclose(q3[:, :, h], q2[:, :, h] + (q0[:, :, h] + k0[:, :, h // R]) / 2, rtol=1e-14)
    for g in range(Hk):
        mean_of_group = sum((q0[:, :, h] + k0[:, :, g]) / 2 for h in range(g * R, (g + 1) * R)) / R
        np.testing.assert_allclose(k3[:, :, g], k2[:, :, g] + mean_of_group, rtol=1e-14)
    e_kv = Hk * d
    vc, vp = rng.standard_normal((B, T, e_kv // 2)), rng.standard_normal((B, T, e_kv // 2))
    v = O.value_shift(vc, vp, Hk, d).reshape(B, T, e_kv)
    for t in range(T):
        assert np.array_equal(v[:, t, :e_kv // 2], vc[:, t])
        assert np.array_equal(v[:, t, e_kv // 2:], vp[:, t - 1] if t else np.zeros_like(vp[:, 0]))


def test_prologue_composition_with_matrix_operators():
    """What enters the norm is conv2(conv1(latent)) plus the means of the latents BEFORE the convolutions, and the
    value stream bypasses both (Sec. 2.2): rebuilt from the matrix operators above, no step function involved."""
    w = dict(B=2, T=11, E=40, Hq=4, Hk=2, dh=6, k_seq=3, k_ch=2, dtype="f32")
    inp = make_inputs(w, seed=8, w_scale=0.3, conv_visible=True)
    r = run(w, inp, use_rope=False)
    Hq, Hk, dh, T = w["Hq"], w["Hk"], w["dh"], w["T"]
    R, e_q, e_kv = Hq // Hk, Hq * dh, Hk * dh
    lat = inp["x"].astype(np.float64) @ inp["w_down"].astype(np.float64)
    w0, w1 = inp["w_conv_seq"].astype(np.float64), inp["w_conv_ch"].astype(np.float64)
    for b in range(w["B"]):
        pre = [lat[b, :, h * dh:(h + 1) * dh] for h in range(Hq + Hk)]               # (T, dh) per latent head
        conv = []
        for h in range(Hq + Hk):
            after_seq = np.stack([seq_operator(w0[h * dh + i], T) @ pre[h][:, i] for i in range(dh)], axis=1)
            conv.append((ch_operator(w1[h], T) @ after_seq.ravel()).reshape(T, dh))
        for h in range(Hq):
            want = conv[h] + (pre[h] + pre[Hq + h // R]) / 2
            np.testing.assert_allclose(r["q3"][b, :, h], want, rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(r["q"][b, :, h], want * math.sqrt(dh) / np.linalg.norm(want, axis=1, keepdims=True),
                                       rtol=1e-11, atol=1e-13)
        for g in range(Hk):
            want = conv[Hq + g] + pre[Hq + g] / 2 + sum(pre[g * R:(g + 1) * R]) / (2 * R)
            np.testing.assert_allclose(r["k3"][b, :, g], want, rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(r["k"][b, :, g], want * math.sqrt(dh) * math.exp(inp["temp"][g])
                                       / np.linalg.norm(want, axis=1, keepdims=True), rtol=1e-11, atol=1e-13)
        v = r["v"][b].reshape(T, e_kv)
        np.testing.assert_allclose(v[:, :e_kv // 2], lat[b, :, e_q + e_kv:e_q + e_kv + e_kv // 2], rtol=1e-12)
        np.testing.assert_allclose(v[1:, e_kv // 2:], lat[b, :-1, e_q + e_kv + e_kv // 2:], rtol=1e-12)
        assert np.array_equal(v[0, e_kv // 2:], np.zeros(e_kv // 2))


# --- P8: RoPE = multiplication of (u_i + i u_{i+d/2}) by exp(i t theta_i);
#     relative-position property; position 0 is the identity ----------------
@pytest.mark.parametrize("interleaved", [False, True])
def test_rope_complex_form_and_relative_property(interleaved):
    rng = np.random.default_rng(0)
    B, T, H, d = 1, 33, 2, 8
    u = rng.standard_normal((B, T, H, d))
    r = O.rope(u, 10000.0, interleaved)
    theta = 10000.0 ** (-2.0 * np.arange(d // 2) / d)
    z = (u[..., 0::2] + 1j * u[..., 1::2]) if interleaved else (u[..., :d // 2] + 1j * u[..., d // 2:])
    zr = z * np.exp(1j * np.arange(T)[None, :, None, None] * theta)
    got = (r[..., 0::2] + 1j * r[..., 1::2]) if interleaved else (r[..., :d // 2] + 1j * r[..., d // 2:])
    np.testing.assert_allclose(got, zr, atol=1e-13)
    assert np.array_equal(r[:, 0], u[:, 0])
    a, b = rng.standard_normal((1, 1, 1, d)), rng.standard_normal((1, 1, 1, d))
    ra = O.rope(np.repeat(a, T, 1), 10000.0, interleaved)
    rb = O.rope(np.repeat(b, T, 1), 10000.0, interleaved)
    dots = np.einsum("btd,bsd->ts", ra[:, :, 0], rb[:, :, 0])
    for off in (0, 1, 5):
        diag = np.diagonal(dots, -off)
        np.testing.assert_allclose(diag, diag[0], atol=1e-12)


def test_rope_large_position_angle():
    """Angles are formed in fp64 from t * theta_i (t up to 16383)."""
    u = np.zeros((1, 16384, 1, 4))
    u[..., 0] = 1.0
    r = O.rope(u, 10000.0)
    t = 16383
    assert abs(r[0, t, 0, 0] - math.cos(t * 1.0)) < 1e-12
    assert abs(r[0, t, 0, 2] - math.sin(t * 1.0)) < 1e-12
    assert abs(r[0, t, 0, 1]) < 1e-15 and abs(r[0, t, 0, 3]) < 1e-15


# --- every optional transform really changes the result ----------------------
@pytest.mark.parametrize("flag", ["use_conv_seq", "use_conv_ch", "use_qk_mean", "use_v_shift",
                                  "use_qk_norm", "use_key_temp", "use_rope"])
def test_each_flag_matters(flag):
    w = TINY
    inp = make_inputs(w, seed=9, w_scale=0.2, conv_visible=True)
    a = run(w, inp)["out"]
    b = run(w, inp, **{flag: False})["out"]
    assert np.abs(a - b).max() > 1e-4


def test_planted_mistakes_are_caught(monkeypatch):
    """Mistakes planted in the oracle make the library cross-check fail."""
    def bad_conv_ch(u, w1):               # transposed filter
        return O.__dict__["_conv_ch_orig"](u, np.swapaxes(w1, 1, 2))
    monkeypatch.setitem(O.__dict__, "_conv_ch_orig", O.conv_ch)
    monkeypatch.setattr(O, "conv_ch", bad_conv_ch)
    with pytest.raises(AssertionError):
        test_prologue_composition_with_matrix_operators()
    monkeypatch.setattr(O, "conv_ch", O.__dict__["_conv_ch_orig"])

    def bad_shift(vc, vp, Hk, dh, shift=True):   # shifts the wrong half
        return O.__dict__["_vs_orig"](vp, vc, Hk, dh, shift)
    monkeypatch.setitem(O.__dict__, "_vs_orig", O.value_shift)
    monkeypatch.setattr(O, "value_shift", bad_shift)
    with pytest.raises(AssertionError):
        test_first_token_closed_form()


def test_norm_epsilon_option_closed_form():
    """The library's optional epsilon under the L2 norm (not in the paper: eps = 0 is the paper's norm and must
    leave every result bit for bit as it was): |q4| = sqrt(d) |q3| / sqrt(|q3|^2 + eps), direction unchanged."""
    rng = np.random.default_rng(11)
    q3 = rng.standard_normal((2, 5, 4, 8))
    k3 = rng.standard_normal((2, 5, 2, 8))
    temp = np.array([0.3, -0.2])
    q_a, k_a = O.qk_norm_temp(q3, k3, temp)
    q_b, k_b = O.qk_norm_temp(q3, k3, temp, eps=0.0)
    assert np.array_equal(q_a, q_b) and np.array_equal(k_a, k_b)
    eps = 2.5
    q_e, k_e = O.qk_norm_temp(q3, k3, temp, eps=eps)
    n2q, n2k = (q3 * q3).sum(-1), (k3 * k3).sum(-1)
    np.testing.assert_allclose(np.linalg.norm(q_e, axis=-1), np.sqrt(8 * n2q / (n2q + eps)), rtol=1e-14)
    np.testing.assert_allclose(np.linalg.norm(k_e, axis=-1), np.sqrt(8 * n2k / (n2k + eps)) * np.exp(temp), rtol=1e-14)
    np.testing.assert_allclose(q_e / np.linalg.norm(q_e, axis=-1, keepdims=True),
                               q3 / np.linalg.norm(q3, axis=-1, keepdims=True), rtol=1e-13)
    # an all-zero head vector stays finite (zero) once eps > 0
    z, _ = O.qk_norm_temp(np.zeros((1, 1, 1, 8)), np.ones((1, 1, 1, 8)), None, eps=1e-6)
    assert np.array_equal(z, np.zeros((1, 1, 1, 8)))
