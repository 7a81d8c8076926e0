"""Host-side helpers around the binding: workload dict -> config, numpy inputs
-> device tensors, and the FLOP count used to turn a latency into TFLOP/s."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as b


def config_from_workload(w: dict, **override) -> b.CCAConfig:
    """w: dict with B, T, E, Hq, Hk, dh, k_seq, k_ch, dtype ('bf16' | 'f32'),
    paper_flags (True: all transforms of Sec. 2.2 on; False: plain MHA/GQA)."""
    cfg = b.CCAConfig(B=w["B"], T=w["T"], d_model=w["E"], n_q_heads=w["Hq"], n_kv_heads=w["Hk"],
                      head_dim=w["dh"], k_seq=w["k_seq"], k_ch=w["k_ch"],
                      dtype=b.CCA_BF16 if w["dtype"] == "bf16" else b.CCA_F32,
                      flags=b.CCA_FLAGS_PAPER if w.get("paper_flags", True) else b.CCA_FLAGS_MHA)
    for k, v in override.items():
        setattr(cfg, k, v)
    return cfg


def weights_to_device(cfg: b.CCAConfig, inp: dict, device="cuda"):
    """numpy inputs (see synth_inputs.make_inputs) -> (x, CCAWeights) on device in cfg's storage type."""
    dt = cfg.torch_dtype

    def dev(a, dtype=dt):
        return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype).contiguous()

    w = b.CCAWeights(w_down=dev(inp["w_down"]), w_out=dev(inp["w_out"]), w_conv_seq=dev(inp["w_conv_seq"]),
                     w_conv_ch=dev(inp["w_conv_ch"]), temp=dev(inp["temp"], torch.float32))
    return dev(inp["x"]), w


def forward_flops(cfg: b.CCAConfig) -> dict:
    """Multiply-add work of one forward pass, counted as 2 FLOP per MAC.
    Causal attention is counted at half the dense T^2 term (only s <= t is
    needed), the usual convention for causal attention kernels; the cost table
    of the paper counts the dense 4*B*E*S^2/C1."""
    B, T, E = cfg.B, cfg.T, cfg.d_model
    e_q, e_kv = cfg.e_q, cfg.e_kv
    proj = 2.0 * B * T * E * (e_q + 2 * e_kv) + 2.0 * B * T * e_q * E
    conv = 0.0
    if cfg.flags & b.CCA_CONV_SEQ:
        conv += 2.0 * B * T * (e_q + e_kv) * cfg.k_seq
    if cfg.flags & b.CCA_CONV_CH:
        conv += 2.0 * B * T * (cfg.n_q_heads + cfg.n_kv_heads) * cfg.head_dim ** 2 * cfg.k_ch
    attn_dense = 4.0 * B * T * T * e_q
    attn = attn_dense / 2 if (cfg.flags & b.CCA_CAUSAL) else attn_dense
    return dict(proj=proj, conv=conv, attn=attn, attn_dense=attn_dense, total=proj + conv + attn)
