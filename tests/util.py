"""Shared helpers of the GPU parity tests (marshalling and error metrics only)."""
import numpy as np
import torch

from oracle import cca_oracle as O


def oracle_forward(w, inp, rows=None, **kw):
    """fp64 oracle on the same (already rounded) inputs.  w: workload dict."""
    flags = {}
    if not w.get("paper_flags", True):
        flags = dict(use_conv_seq=False, use_conv_ch=False, use_qk_mean=False, use_v_shift=False,
                     use_qk_norm=False, use_key_temp=False, use_rope=False)
    flags.update(kw)
    return O.cca_forward(inp["x"], inp["w_down"], inp["w_conv_seq"], inp["w_conv_ch"], inp["temp"], inp["w_out"],
                         n_q_heads=w["Hq"], n_kv_heads=w["Hk"], head_dim=w["dh"], rows=rows, **flags)


def to_np(t):
    return t.detach().to(torch.float64).cpu().numpy()


def errors(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in GPU result"
    rel_l2 = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
    max_abs = float(np.abs(got - ref).max()) if got.size else 0.0
    return rel_l2, max_abs


# spec tolerances: bf16 rel-L2 <= 1e-2 and max-abs <= 2e-2; fp32 <= 1e-5 both
TOL = {"bf16": (1e-2, 2e-2), "f32": (1e-5, 1e-5)}


def check_out(got, ref, dtype, what="out"):
    rel, mx = errors(got, ref)
    rtol, atol = TOL[dtype]
    assert rel <= rtol and mx <= atol, f"{what}: rel_l2={rel:.3e} (<= {rtol}), max_abs={mx:.3e} (<= {atol})"
    return rel, mx


def check_tap(got, ref, dtype, what):
    """Intermediates can be O(10) in magnitude (q, k have norm sqrt(d_h)), so
    the absolute bound scales with the largest reference magnitude."""
    rel, mx = errors(got, ref)
    rtol, atol = TOL[dtype]
    lim = atol * max(1.0, float(np.abs(ref).max()))
    assert rel <= rtol and mx <= lim, f"{what}: rel_l2={rel:.3e} (<= {rtol}), max_abs={mx:.3e} (<= {lim:.3e})"
    return rel, mx
