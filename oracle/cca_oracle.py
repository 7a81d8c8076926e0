"""CPU oracle (fp64, NumPy) for the CCA / CCGQA prefill block.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
path is checked against.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import it; the product path never
does.  It shares no code with the HIP path and imports nothing from it.

CCA is its own function (not an approximation of MHA), so the oracle takes the
method's steps in the paper's order, each by its plain definition:

  1. down-projection of x to latent q, k and the two value streams
     (Sec. 2.2, first CCA equation and the value-shift equation);
  2. depth-wise causal sequence convolution on q and k (conv1_seq);
  3. head-wise grouped causal convolution mixing the channels of one head
     across k_ch time steps (conv2_seq+ch);
  4. qk-mean: add the mean of the *pre-convolution* q and (group-broadcast) k;
  5. value-shift: half of the value channels come from the previous token;
  6. L2 normalisation of q, k over the head width, scaled by sqrt(d_h); the
     key additionally by beta = exp(temp) per KV head;
  7. RoPE on q and k in the latent space;
  8. causal softmax attention per latent head, KV heads shared by groups of
     consecutive query heads (CCGQA);
  9. up-projection to d_model.

All arithmetic is fp64.  Inputs are whatever the caller hands over (already
rounded to the storage type), upcast to fp64; nothing is rounded in between.

Pins (tests/test_oracle_pins.py): reduction to textbook MHA / GQA; identity
convolutions; causality; brute-force softmax on tiny inputs; norm / RoPE
closed forms; the first-token closed form; a cross-check of steps 1-6 against
library convolution / normalisation routines; RoPE as complex multiplication.
Readings that no printed value can pin (k_ch = 2, softmax scale 1/sqrt(d_h)
when d_h != E/16, rotate-half RoPE pairing with base 10000) are "parity
unpinned": the HIP path is checked against this oracle's reading of them.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "down_project", "conv_seq", "conv_ch", "qk_mean", "value_shift",
    "qk_norm_temp", "rope", "attention", "up_project", "cca_forward", "cca_backward",
]


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _shift_time(a, s):
    """a[:, t] -> a[:, t - s] along axis 1 with zeros entering at the start of
    every sequence (axis 0 is the batch, so sequences never leak into each
    other)."""
    if s == 0:
        return a
    out = np.zeros_like(a)
    if s < a.shape[1]:
        out[:, s:] = a[:, : a.shape[1] - s]
    return out


# -- step 1 -----------------------------------------------------------------
def down_project(x, w_down, n_q_heads, n_kv_heads, head_dim):
    """q0 = x W_Q, k0 = x W_K, vc = x W_V, vp = x W_Vbar (Sec. 2.2: the
    down-projection equation and the value-shift equation).  ``w_down`` packs
    the four matrices column-wise as [W_Q | W_K | W_V | W_Vbar]."""
    x, w_down = _f64(x), _f64(w_down)
    B, T, E = x.shape
    e_q, e_kv = n_q_heads * head_dim, n_kv_heads * head_dim
    half = e_kv // 2
    assert w_down.shape == (E, e_q + 2 * e_kv)
    lat = x @ w_down
    q0 = lat[..., :e_q].reshape(B, T, n_q_heads, head_dim)
    k0 = lat[..., e_q:e_q + e_kv].reshape(B, T, n_kv_heads, head_dim)
    vc = lat[..., e_q + e_kv:e_q + e_kv + half]
    vp = lat[..., e_q + e_kv + half:]
    return q0, k0, vc, vp


# -- step 2 -----------------------------------------------------------------
def conv_seq(u, w0):
    """Depth-wise causal convolution along time (conv1_seq in the conv
    equation of Sec. 2.2).  u: (B,T,C), w0: (C,k_seq).  Tap k_seq-1 multiplies
    the current token, tap j the token k_seq-1-j steps back."""
    u, w0 = _f64(u), _f64(w0)
    k = w0.shape[1]
    y = np.zeros_like(u)
    for j in range(k):
        y += w0[:, j] * _shift_time(u, k - 1 - j)
    return y


# -- step 3 -----------------------------------------------------------------
def conv_ch(u, w1):
    """Grouped causal convolution, one group per head (conv2_seq+ch).
    u: (B,T,H,d), w1: (H, d_out, d_in, k_ch).  Each head has a dense d x d
    filter per tap; tap k_ch-1 multiplies the current token."""
    u, w1 = _f64(u), _f64(w1)
    H, d_out, d_in, k = w1.shape
    y = np.zeros(u.shape[:3] + (d_out,))
    for j in range(k):
        us = _shift_time(u, k - 1 - j)
        for h in range(H):
            # y[b,t,h,o] += sum_i w1[h,o,i,j] * us[b,t,h,i]
            y[:, :, h, :] += us[:, :, h, :] @ w1[h, :, :, j].T
    return y


# -- step 4 -----------------------------------------------------------------
def qk_mean(q2, k2, q0, k0):
    """qk-mean equation of Sec. 2.2.  m_q = (q_pre + B_group(k_pre)) / 2 per
    query head; m_k = E_group(m_q) = mean of m_q over the query heads that
    share a KV head.  q_pre, k_pre are the step-1 latents."""
    Hq, Hk = q0.shape[2], k0.shape[2]
    R = Hq // Hk
    k_b = np.repeat(k0, R, axis=2)                     # q head h <- kv head h // R
    m_q = 0.5 * (q0 + k_b)
    m_k = m_q.reshape(m_q.shape[0], m_q.shape[1], Hk, R, -1).mean(axis=3)
    return q2 + m_q, k2 + m_k


# -- step 5 -----------------------------------------------------------------
def value_shift(vc, vp, n_kv_heads, head_dim, shift=True):
    """Value-shift equation: v_t = [W_V x_t , W_Vbar x_{t-1}], zero for the
    first token of each sequence.  First half of the value channels is the
    current-token stream, second half the previous-token stream."""
    vc, vp = _f64(vc), _f64(vp)
    if shift:
        vp = _shift_time(vp, 1)
    v = np.concatenate([vc, vp], axis=-1)
    return v.reshape(v.shape[0], v.shape[1], n_kv_heads, head_dim)


# -- step 6 -----------------------------------------------------------------
def qk_norm_temp(q3, k3, temp=None, eps=0.0):
    """q <- q sqrt(d_h) / ||q||_2, k <- k sqrt(d_h) / ||k||_2 * exp(temp_g)
    (first two lines of the final equation block of Sec. 2.2).  The paper's
    norm has no epsilon (eps = 0, the default); a caller-chosen eps > 0 is
    added to the sum of squares under the root, an option of the library's
    interface, not of the paper."""
    d = q3.shape[-1]
    q4 = q3 * np.sqrt(d) / np.sqrt((q3 * q3).sum(-1, keepdims=True) + eps)
    k4 = k3 * np.sqrt(d) / np.sqrt((k3 * k3).sum(-1, keepdims=True) + eps)
    if temp is not None:
        k4 = k4 * np.exp(_f64(temp))[None, None, :, None]
    return q4, k4


# -- step 7 -----------------------------------------------------------------
def rope(u, base=10000.0, interleaved=False, positions=None):
    """Rotary position embedding on the full head width.  u: (B,T,H,d).
    Pair i rotates by angle t * base^(-2i/d); pairs are (i, i + d/2)
    (rotate-half) or (2i, 2i+1) when ``interleaved``."""
    u = _f64(u)
    B, T, H, d = u.shape
    half = d // 2
    t = np.arange(T, dtype=np.float64) if positions is None else _f64(positions)
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = t[:, None] * theta[None, :]                   # (T, d/2)
    c, s = np.cos(ang)[None, :, None, :], np.sin(ang)[None, :, None, :]
    out = np.empty_like(u)
    if interleaved:
        a, b = u[..., 0::2], u[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = b * c + a * s
    else:
        a, b = u[..., :half], u[..., half:]
        out[..., :half] = a * c - b * s
        out[..., half:] = b * c + a * s
    return out


# -- step 8 -----------------------------------------------------------------
def attention(q, k, v, scale, causal=True, rows=None):
    """o[t,h] = sum_s softmax_s(scale <q[t,h], k[s,h//R]>) v[s,h//R]; with
    ``causal`` only s <= t (attention line of the final equation block;
    KV-head sharing as in the CCGQA paragraph).

    q: (B,T,Hq,d); k, v: (B,T,Hk,d).  Each query row is handled on its own by
    the two-pass definition (max, exp, normalise); the T x T matrix is never
    held for more than a chunk of rows.  ``rows`` (1-D int array) restricts
    the computation to those query positions.  Returns o (B,n_rows,Hq,d) and
    the natural-log sum-exp of the scaled logits, lse (B,Hq,n_rows).
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, T, Hq, d = q.shape
    Hk = k.shape[2]
    R = Hq // Hk
    rows = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    n = len(rows)
    o = np.zeros((B, n, Hq, v.shape[-1]))
    lse = np.zeros((B, Hq, n))
    chunk = 256
    for b in range(B):
        for h in range(Hq):
            g = h // R
            kh, vh = k[b, :, g, :], v[b, :, g, :]
            for c0 in range(0, n, chunk):
                r = rows[c0:c0 + chunk]
                s_max = int(r.max()) + 1 if causal else T
                s = scale * (q[b, r, h, :] @ kh[:s_max].T)          # (len(r), s_max)
                if causal:
                    s = np.where(np.arange(s_max)[None, :] <= r[:, None], s, -np.inf)
                m = s.max(axis=1, keepdims=True)
                p = np.exp(s - m)
                z = p.sum(axis=1, keepdims=True)
                o[b, c0:c0 + len(r), h, :] = (p / z) @ vh[:s_max]
                lse[b, h, c0:c0 + len(r)] = (m + np.log(z))[:, 0]
    return o, lse


# -- step 9 -----------------------------------------------------------------
def up_project(o, w_out):
    """out = [o_1 .. o_{n_h}] W_O (last line of the final equation block)."""
    o, w_out = _f64(o), _f64(w_out)
    B, n = o.shape[:2]
    return o.reshape(B, n, -1) @ w_out


def cca_forward(x, w_down, w_conv_seq, w_conv_ch, temp, w_out, *,
                n_q_heads, n_kv_heads, head_dim,
                causal=True, use_conv_seq=True, use_conv_ch=True,
                use_qk_mean=True, use_v_shift=True, use_qk_norm=True,
                use_key_temp=True, use_rope=True, rope_interleaved=False,
                rope_base=10000.0, softmax_scale=None, rows=None, norm_eps=0.0):
    """Whole block, steps 1-9.  Returns a dict with ``out`` (B,n_rows,E) and
    every intermediate (q0, k0 pre-conv latents; q, k, v as they enter
    attention; o; lse)."""
    Hq, Hk, dh = n_q_heads, n_kv_heads, head_dim
    e_q = Hq * dh
    x = _f64(x)
    B, T, _ = x.shape
    q0, k0, vc, vp = down_project(x, w_down, Hq, Hk, dh)
    q, k = q0, k0
    if use_conv_seq:
        w0 = _f64(w_conv_seq)
        q = conv_seq(q.reshape(B, T, -1), w0[:e_q]).reshape(q0.shape)
        k = conv_seq(k.reshape(B, T, -1), w0[e_q:]).reshape(k0.shape)
    if use_conv_ch:
        w1 = _f64(w_conv_ch)
        q = conv_ch(q, w1[:Hq])
        k = conv_ch(k, w1[Hq:])
    if use_qk_mean:
        q, k = qk_mean(q, k, q0, k0)
    q3, k3 = q, k                                      # as they enter the norm step
    v = value_shift(vc, vp, Hk, dh, shift=use_v_shift)
    if use_qk_norm:
        q, k = qk_norm_temp(q, k, temp if use_key_temp else None, norm_eps)
    if use_rope:
        q = rope(q, rope_base, rope_interleaved)
        k = rope(k, rope_base, rope_interleaved)
    scale = 1.0 / np.sqrt(dh) if not softmax_scale else float(softmax_scale)
    o, lse = attention(q, k, v, scale, causal=causal, rows=rows)
    out = up_project(o, w_out)
    return dict(out=out, q0=q0, k0=k0, vc=vc, vp=vp, q3=q3, k3=k3, q=q, k=k, v=v, o=o, lse=lse)


# ===========================================================================
# Backward (adjoint) of steps 9 -> 1.  The paper gives no backward equations;
# each function below is the hand-derived transpose of the forward step of the
# same name, in fp64.  Pinned by central finite differences of cca_forward and
# by the <dOut, J d> = <J^T dOut, d> identity (tests/test_oracle_backward.py).
# ===========================================================================
def _unshift_time(a, s):
    """Adjoint of _shift_time: out[:, t] = a[:, t + s], zeros entering at the end."""
    if s == 0:
        return a
    out = np.zeros_like(a)
    if s < a.shape[1]:
        out[:, : a.shape[1] - s] = a[:, s:]
    return out


def conv_seq_bwd(dy, u, w0):
    """y[t,c] = sum_j w0[c,j] u[t-(k-1-j), c]  ->  du, dw0."""
    dy, u, w0 = _f64(dy), _f64(u), _f64(w0)
    k = w0.shape[1]
    du = np.zeros_like(u)
    dw0 = np.zeros_like(w0)
    for j in range(k):
        s = k - 1 - j
        du += w0[:, j] * _unshift_time(dy, s)
        dw0[:, j] = (dy * _shift_time(u, s)).sum(axis=(0, 1))
    return du, dw0


def conv_ch_bwd(dy, u, w1):
    """y[t,h,o] = sum_j sum_i w1[h,o,i,j] u[t-(k-1-j), h, i]  ->  du, dw1."""
    dy, u, w1 = _f64(dy), _f64(u), _f64(w1)
    H, d_out, d_in, k = w1.shape
    du = np.zeros_like(u)
    dw1 = np.zeros_like(w1)
    for j in range(k):
        s = k - 1 - j
        dys = _unshift_time(dy, s)         # dy[t + s]
        us = _shift_time(u, s)             # u[t - s]
        for h in range(H):
            du[:, :, h, :] += dys[:, :, h, :] @ w1[h, :, :, j]
            dw1[h, :, :, j] = np.einsum("bto,bti->oi", dy[:, :, h, :], us[:, :, h, :])
    return du, dw1


def qk_mean_bwd(dq3, dk3):
    """q3 = q2 + m_q, k3 = k2 + m_k with m_q = (q0 + rep(k0))/2, m_k = mean_r m_q.
    Returns (dq2, dk2, dq0_part, dk0_part)."""
    Hq, Hk = dq3.shape[2], dk3.shape[2]
    R = Hq // Hk
    dm_q = dq3 + np.repeat(dk3, R, axis=2) / R
    dq0 = 0.5 * dm_q
    dk0 = 0.5 * dm_q.reshape(dm_q.shape[0], dm_q.shape[1], Hk, R, -1).sum(axis=3)
    return dq3, dk3, dq0, dk0


def value_shift_bwd(dv, shift=True):
    """v = [vc | shift(vp)]  ->  dvc, dvp."""
    B, T = dv.shape[:2]
    dv = dv.reshape(B, T, -1)
    half = dv.shape[-1] // 2
    dvc, dvp = dv[..., :half], dv[..., half:]
    if shift:
        dvp = _unshift_time(dvp, 1)
    return dvc, dvp


def qk_norm_temp_bwd(dq4, dk4, q3, k3, temp=None, eps=0.0):
    """y = x sqrt(d) / |x| (* exp(temp_g) for keys)  ->  dx, dtemp and sum_t |<dk4_t, k4_t>| (the magnitude
    the signed sum dtemp cancels down from: the natural error scale for a reduced-precision dtemp)."""
    d = q3.shape[-1]

    def one(dy, x, mul):
        n = np.sqrt((x * x).sum(-1, keepdims=True) + eps)   # y = mul sqrt(d) x / n; dn/dx = x / n
        xh = x / n
        return mul * np.sqrt(d) / n * (dy - xh * (xh * dy).sum(-1, keepdims=True))

    dq3 = one(dq4, q3, 1.0)
    if temp is None:
        return dq3, one(dk4, k3, 1.0), None, None
    beta = np.exp(_f64(temp))[None, None, :, None]
    dk3 = one(dk4, k3, beta)
    k4 = k3 * np.sqrt(d) / np.sqrt((k3 * k3).sum(-1, keepdims=True) + eps) * beta
    per_token = (dk4 * k4).sum(axis=3)                 # (B,T,Hk): d temp_g is the sum of these signed terms
    return dq3, dk3, per_token.sum(axis=(0, 1)), np.abs(per_token).sum(axis=(0, 1))


def rope_bwd(dy, base=10000.0, interleaved=False):
    """RoPE is a rotation: its adjoint rotates by the opposite angle."""
    dy = _f64(dy)
    B, T, H, d = dy.shape
    half = d // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.arange(T, dtype=np.float64)[:, None] * theta[None, :]
    c, s = np.cos(ang)[None, :, None, :], np.sin(ang)[None, :, None, :]
    out = np.empty_like(dy)
    if interleaved:
        a, b = dy[..., 0::2], dy[..., 1::2]
        out[..., 0::2] = a * c + b * s
        out[..., 1::2] = b * c - a * s
    else:
        a, b = dy[..., :half], dy[..., half:]
        out[..., :half] = a * c + b * s
        out[..., half:] = b * c - a * s
    return out


def attention_bwd(do, q, k, v, scale, causal=True, rows=None):
    """Adjoint of attention(): with P = softmax(scale q k^T) row-wise,
    dV = P^T dO, dP = dO V^T, dS = P * (dP - rowsum(dP * P)),
    dQ = scale dS K, dK = scale dS^T Q; dK, dV summed over the query heads of a group.

    ``rows`` (1-D int array): the caller states that ``do`` is zero at every
    other query position; those rows have dS = 0 and add nothing to dV, so
    they are skipped (their dQ stays zero)."""
    do, q, k, v = _f64(do), _f64(q), _f64(k), _f64(v)
    B, T, Hq, d = q.shape
    Hk = k.shape[2]
    R = Hq // Hk
    do = do.reshape(B, T, Hq, -1)
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    rows = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    chunk = 256
    for b in range(B):
        for h in range(Hq):
            g = h // R
            for c0 in range(0, len(rows), chunk):
                r = rows[c0:c0 + chunk]
                s_max = int(r.max()) + 1 if causal else T
                s = scale * (q[b, r, h, :] @ k[b, :s_max, g, :].T)
                if causal:
                    s = np.where(np.arange(s_max)[None, :] <= r[:, None], s, -np.inf)
                p = np.exp(s - s.max(axis=1, keepdims=True))
                p /= p.sum(axis=1, keepdims=True)
                dp = do[b, r, h, :] @ v[b, :s_max, g, :].T
                ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
                dv[b, :s_max, g, :] += p.T @ do[b, r, h, :]
                dq[b, r, h, :] = scale * (ds @ k[b, :s_max, g, :])
                dk[b, :s_max, g, :] += scale * (ds.T @ q[b, r, h, :])
    return dq, dk, dv


def cca_backward(x, w_down, w_conv_seq, w_conv_ch, temp, w_out, d_out, *,
                 n_q_heads, n_kv_heads, head_dim,
                 causal=True, use_conv_seq=True, use_conv_ch=True,
                 use_qk_mean=True, use_v_shift=True, use_qk_norm=True,
                 use_key_temp=True, use_rope=True, rope_interleaved=False,
                 rope_base=10000.0, softmax_scale=None, rows=None, norm_eps=0.0):
    """Gradients of sum(out * d_out) with respect to x and every weight.
    Recomputes the forward intermediates it needs.  Returns a dict:
    d_x, d_w_down, d_w_conv_seq, d_w_conv_ch, d_temp, d_w_out plus the
    intermediate gradients d_o, d_q, d_k, d_v (as they leave attention) and d_lat.

    ``rows`` (1-D int array): the caller states that ``d_out`` is zero at
    every other position; the attention forward / backward then visit only
    those query rows (everything is linear in d_out, so the result is the
    same as with rows=None)."""
    Hq, Hk, dh = n_q_heads, n_kv_heads, head_dim
    e_q, e_kv = Hq * dh, Hk * dh
    x, d_out = _f64(x), _f64(d_out)
    B, T, _ = x.shape
    w_down, w_out = _f64(w_down), _f64(w_out)
    # ---- forward, keeping what the adjoint needs
    q0, k0, vc, vp = down_project(x, w_down, Hq, Hk, dh)
    q1, k1 = q0, k0
    if use_conv_seq:
        w0 = _f64(w_conv_seq)
        q1 = conv_seq(q0.reshape(B, T, -1), w0[:e_q]).reshape(q0.shape)
        k1 = conv_seq(k0.reshape(B, T, -1), w0[e_q:]).reshape(k0.shape)
    q2, k2 = q1, k1
    if use_conv_ch:
        w1 = _f64(w_conv_ch)
        q2, k2 = conv_ch(q1, w1[:Hq]), conv_ch(k1, w1[Hq:])
    q3, k3 = qk_mean(q2, k2, q0, k0) if use_qk_mean else (q2, k2)
    v = value_shift(vc, vp, Hk, dh, shift=use_v_shift)
    q4, k4 = qk_norm_temp(q3, k3, temp if use_key_temp else None, norm_eps) if use_qk_norm else (q3, k3)
    q5, k5 = (rope(q4, rope_base, rope_interleaved), rope(k4, rope_base, rope_interleaved)) if use_rope else (q4, k4)
    scale = 1.0 / np.sqrt(dh) if not softmax_scale else float(softmax_scale)
    ridx = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    o, _ = attention(q5, k5, v, scale, causal=causal, rows=rows)       # (B, len(ridx), Hq, dh)
    # ---- adjoint, last step first
    o_flat = o.reshape(B, len(ridx), -1)
    d_w_out = np.einsum("bte,btf->ef", o_flat, d_out[:, ridx])
    d_o = np.zeros((B, T, e_q))
    d_o[:, ridx] = d_out[:, ridx] @ w_out.T
    d_q5, d_k5, d_v = attention_bwd(d_o, q5, k5, v, scale, causal=causal, rows=rows)
    d_q4, d_k4 = (rope_bwd(d_q5, rope_base, rope_interleaved), rope_bwd(d_k5, rope_base, rope_interleaved)) \
        if use_rope else (d_q5, d_k5)
    d_temp, d_temp_abs = np.zeros(Hk), np.zeros(Hk)
    if use_qk_norm:
        d_q3, d_k3, dt, dt_abs = qk_norm_temp_bwd(d_q4, d_k4, q3, k3, temp if use_key_temp else None, norm_eps)
        if dt is not None:
            d_temp, d_temp_abs = dt, dt_abs
    else:
        d_q3, d_k3 = d_q4, d_k4
    d_q0 = np.zeros_like(q0)
    d_k0 = np.zeros_like(k0)
    if use_qk_mean:
        d_q2, d_k2, dq0m, dk0m = qk_mean_bwd(d_q3, d_k3)
        d_q0 += dq0m
        d_k0 += dk0m
    else:
        d_q2, d_k2 = d_q3, d_k3
    d_w1 = np.zeros_like(_f64(w_conv_ch)) if w_conv_ch is not None else None
    if use_conv_ch:
        d_q1, dw1q = conv_ch_bwd(d_q2, q1, w1[:Hq])
        d_k1, dw1k = conv_ch_bwd(d_k2, k1, w1[Hq:])
        d_w1 = np.concatenate([dw1q, dw1k], axis=0)
    else:
        d_q1, d_k1 = d_q2, d_k2
    d_w0 = np.zeros_like(_f64(w_conv_seq)) if w_conv_seq is not None else None
    if use_conv_seq:
        dq, dw0q = conv_seq_bwd(d_q1.reshape(B, T, -1), q0.reshape(B, T, -1), w0[:e_q])
        dk, dw0k = conv_seq_bwd(d_k1.reshape(B, T, -1), k0.reshape(B, T, -1), w0[e_q:])
        d_q0 += dq.reshape(q0.shape)
        d_k0 += dk.reshape(k0.shape)
        d_w0 = np.concatenate([dw0q, dw0k], axis=0)
    else:
        d_q0 += d_q1
        d_k0 += d_k1
    d_vc, d_vp = value_shift_bwd(d_v, shift=use_v_shift)
    d_lat = np.concatenate([d_q0.reshape(B, T, -1), d_k0.reshape(B, T, -1), d_vc, d_vp], axis=-1)
    d_x = d_lat @ w_down.T
    d_w_down = np.einsum("bte,btf->ef", x, d_lat)
    return dict(d_x=d_x, d_w_down=d_w_down, d_w_conv_seq=d_w0, d_w_conv_ch=d_w1, d_temp=d_temp, d_w_out=d_w_out,
                d_temp_abs=d_temp_abs, d_o=d_o, d_q=d_q5, d_k=d_k5, d_v=d_v, d_lat=d_lat)
