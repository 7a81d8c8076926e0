"""Seeded synthetic inputs for the CCA / CCGQA prefill block.

This module only *draws numbers and names shapes*.  It holds none of the
method's arithmetic (no projection, convolution, norm, RoPE or attention), so
both the CPU oracle's tests and the HIP path's tests may import it without the
two implementations sharing code.

The kernel measurements in the paper use random tensors of a given shape
(App. D.1: E = 2048, BF16, head_dim 128, S up to 16384), so synthetic tensors
*are* the paper's workload for this path.

Draw order (fixed, one PCG64 stream per seed): x, W_Q, W_K, W_V, W_Vbar,
w_conv_seq, w_conv_ch, temp, W_O.  x has unit scale, everything else is scaled
by ``w_scale`` (0.02).  The "conv-visible" variant rescales the two conv
filters and temp so that a wrong conv / temperature is not hidden under the
qk-mean skip branch.
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------
# Named workloads.  Plain dicts of integers / booleans: shapes only.
#   E = d_model, Hq / Hk = latent query / KV heads, dh = latent head width.
# ---------------------------------------------------------------------------
WORKLOADS = {
    # Tiny CCA forward, fp32, compression 4 -> 2 heads x 32
    "tiny_fp32": dict(B=1, T=256, E=256, Hq=2, Hk=2, dh=32, k_seq=2, k_ch=2,
                      dtype="f32", paper_flags=True),
    # CCA prefill bf16, compression 4 -> 4 heads x 128
    "cca_4k": dict(B=1, T=4096, E=2048, Hq=4, Hk=4, dh=128, k_seq=2, k_ch=2,
                   dtype="bf16", paper_flags=True),
    # CCGQA prefill bf16, C1 = 2, C2 = 8 -> 8 q heads / 2 kv heads x 128
    "ccgqa_16k": dict(B=1, T=16384, E=2048, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2,
                      dtype="bf16", paper_flags=True),
    # head-to-head, B = 4
    "ccgqa_16k_b4": dict(B=4, T=16384, E=2048, Hq=8, Hk=2, dh=128, k_seq=2, k_ch=2,
                         dtype="bf16", paper_flags=True),
    "mha_16k_b4": dict(B=4, T=16384, E=2048, Hq=16, Hk=16, dh=128, k_seq=1, k_ch=1,
                       dtype="bf16", paper_flags=False),
    "mha_16k": dict(B=1, T=16384, E=2048, Hq=16, Hk=16, dh=128, k_seq=1, k_ch=1,
                    dtype="bf16", paper_flags=False),
    # the CCGQA layout at the widest head of the paper's kernel figures: same latent widths, 4 / 1 heads x 256
    "ccgqa_16k_dh256": dict(B=1, T=16384, E=2048, Hq=4, Hk=1, dh=256, k_seq=2, k_ch=2,
                            dtype="bf16", paper_flags=True),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32.

    Pure storage-format rounding of *inputs*; not part of the method.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def latent_dims(w: dict) -> dict:
    """Widths implied by a workload dict (names follow the paper's symbols)."""
    e_q = w["Hq"] * w["dh"]          # E / C1
    e_kv = w["Hk"] * w["dh"]         # E / C2
    return dict(e_q=e_q, e_kv=e_kv, n_lat=e_q + 2 * e_kv,
                group=w["Hq"] // w["Hk"])


def make_inputs(w: dict, seed: int = 0, w_scale: float = 0.02,
                conv_visible: bool = False, temp_scale: float | None = None) -> dict:
    """Draw x and all weights for workload dict ``w``.

    Returns fp32 numpy arrays; when ``w['dtype'] == 'bf16'`` every array except
    ``temp`` is rounded once to bf16-representable values so that the oracle
    and the GPU consume identical numbers.
    """
    B, T, E = w["B"], w["T"], w["E"]
    Hq, Hk, dh = w["Hq"], w["Hk"], w["dh"]
    k_seq, k_ch = w["k_seq"], w["k_ch"]
    d = latent_dims(w)
    e_q, e_kv = d["e_q"], d["e_kv"]
    rng = np.random.Generator(np.random.PCG64(seed))

    def draw(*shape):
        return rng.standard_normal(shape, dtype=np.float32)

    x = draw(B, T, E)
    w_q = draw(E, e_q) * w_scale
    w_k = draw(E, e_kv) * w_scale
    w_v = draw(E, e_kv // 2) * w_scale
    w_vbar = draw(E, e_kv - e_kv // 2) * w_scale
    w_conv_seq = draw(e_q + e_kv, k_seq)
    w_conv_ch = draw(Hq + Hk, dh, dh, k_ch)
    temp = draw(Hk)
    w_o = draw(e_q, E) * w_scale
    if conv_visible:
        w_conv_seq = w_conv_seq * np.float32(1.0 / np.sqrt(k_seq))
        w_conv_ch = w_conv_ch * np.float32(1.0 / np.sqrt(dh * k_ch))
        temp = temp * np.float32(0.5 if temp_scale is None else temp_scale)
    else:
        w_conv_seq = w_conv_seq * w_scale
        w_conv_ch = w_conv_ch * w_scale
        temp = temp * np.float32(w_scale if temp_scale is None else temp_scale)

    out = dict(
        x=x,
        w_down=np.concatenate([w_q, w_k, w_v, w_vbar], axis=1),
        w_conv_seq=w_conv_seq.astype(np.float32),
        w_conv_ch=w_conv_ch.astype(np.float32),
        temp=temp.astype(np.float32),
        w_out=w_o,
    )
    if w["dtype"] == "bf16":
        for k in ("x", "w_down", "w_conv_seq", "w_conv_ch", "w_out"):
            out[k] = round_to_bf16(out[k])
    return out


def make_upstream_grad(w: dict, seed: int = 1) -> np.ndarray:
    """d_out ~ N(0,1), shape (B, T, E); bf16-rounded for bf16 workloads."""
    rng = np.random.Generator(np.random.PCG64(seed))
    g = rng.standard_normal((w["B"], w["T"], w["E"]), dtype=np.float32)
    return round_to_bf16(g) if w["dtype"] == "bf16" else g


def sample_rows(T: int, n: int, seed: int = 7) -> np.ndarray:
    """Sorted sample of n query positions in [0, T) that always contains the
    first row, the last row and a row just after a 256-token tile edge."""
    rng = np.random.Generator(np.random.PCG64(seed))
    fixed = {0, T - 1, min(T - 1, 256), min(T - 1, 255)}
    extra = rng.choice(T, size=max(0, n - len(fixed)), replace=False)
    return np.array(sorted(fixed | set(int(t) for t in extra)), dtype=np.int64)
