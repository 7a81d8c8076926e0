#!/usr/bin/env python3
"""Benchmark of the CCA / CCGQA prefill block on one MI355X.

A step is one pass of the whole hot path (down-projection, prologue, latent
attention, up-projection = one `cca_forward` call) over one batch of synthetic
input that is already resident in HBM.  The workload is the CCGQA prefill
configuration the headline metric is quoted on: B=1, T=16384, d_model=2048,
8 query heads / 2 KV heads x 128 (C1=2, C2=8), causal, bf16.

Prints ONE JSON line.  `value` is whole-block TFLOP/s with causal attention
counted at half the dense T^2 term; `roofline` is for the dominant kernel (the
latent attention kernel, MFMA-bound) and is measured with HIP events around
that kernel's launches on the stream it runs on; `cpu_baseline` is the fp64
oracle timed on the host cores on a causal prefix of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
# HBM bytes per attn_fwd_kernel launch on the ccgqa_16k workload, from two rocprofv3 --pmc runs (FETCH_SIZE
# 146.10 MiB after scaling by 2.000, WRITE_SIZE 32.05 MiB after scaling by 1.000, the factors a 256 MiB
# device-to-device copy gives for the same counters); summary in profiles/ccgqa_16k_hbm_traffic_pmc.txt.
# Algorithmic bytes of the kernel: 80 MiB (Q 32 + K,V 16 read, O 32 written).
ATTN_TRAFFIC_BYTES = {"ccgqa_16k": int((146.10 + 32.05) * 2 ** 20)}


# Layouts of the grid, all at E = 2048 through the same entry points, head counts for d_h = 128 (at d_h = 64 there
# are twice as many heads, so the latent widths stay the same).  "gqa8" reads the paper's GQA-8 as 8x fewer KV heads
# than MHA (16 query heads, 2 KV heads: the KV-cache size of the C2 = 8 layouts).
GRID_LAYOUTS = {
    "mha": dict(Hq=16, Hk=16, paper_flags=False),
    "gqa8": dict(Hq=16, Hk=2, paper_flags=False),
    "cca4x": dict(Hq=4, Hk=4, paper_flags=True),
    "ccgqa": dict(Hq=8, Hk=2, paper_flags=True),
}


def run_grid(P, torch, dh=128) -> int:
    from paper_2510_04476_amd import binding as b
    dev = "cuda"
    rows = []
    with_bwd = True
    for causal in (True, False):
        for S in (512, 1024, 2048, 4096, 8192, 16384):
            base = {}
            for name, lay in GRID_LAYOUTS.items():
                w = dict(B=1, T=S, E=2048, dh=dh, k_seq=2, k_ch=2, dtype="bf16", paper_flags=lay["paper_flags"],
                         Hq=lay["Hq"] * 128 // dh, Hk=lay["Hk"] * 128 // dh)
                cfg = P.config_from_workload(w)
                if not causal:
                    cfg.flags &= ~b.CCA_CAUSAL
                g = torch.Generator(device=dev).manual_seed(0)
                rn = lambda *sh, sc=1.0: (torch.randn(*sh, device=dev, generator=g) * sc).to(cfg.torch_dtype)
                x = rn(cfg.B, cfg.T, cfg.d_model)
                wt = P.CCAWeights(w_down=rn(cfg.d_model, cfg.n_lat, sc=0.02), w_out=rn(cfg.e_q, cfg.d_model, sc=0.02),
                                  w_conv_seq=rn(cfg.e_q + cfg.e_kv, cfg.k_seq, sc=0.02),
                                  w_conv_ch=rn(cfg.n_q_heads + cfg.n_kv_heads, cfg.head_dim, cfg.head_dim, cfg.k_ch, sc=0.02),
                                  temp=torch.randn(cfg.n_kv_heads, device=dev, generator=g) * 0.02)
                wt_p = P.cca_prepare(cfg, wt)  # forward timing: weights prepared once, as a deployment would
                d_out = rn(cfg.B, cfg.T, cfg.d_model)
                out, d_x = torch.empty_like(x), torch.empty_like(x)
                saved = P.CCASaved.allocate(cfg, dev)
                grads = P.CCAGrads.allocate_like(wt)
                ws, wsb = P.new_workspace(cfg, dev), P.new_backward_workspace(cfg, dev)
                fwd = lambda: P.cca_forward(cfg, wt_p, x, out=out, saved=None, workspace=ws)

                def fwd_bwd():
                    P.cca_forward(cfg, wt, x, out=out, saved=saved, workspace=ws)
                    P.cca_backward(cfg, wt, x, saved, d_out, d_x=d_x, grads=grads, workspace=wsb)

                def timeit(fn, n):
                    t0 = time.perf_counter()       # enter the timed loop from ~60 ms of sustained work, never from
                    while time.perf_counter() - t0 < 0.06:  # idle clocks (see prewarm() in main)
                        fn()
                        fn()
                        torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(n):
                        fn()
                    torch.cuda.synchronize()
                    return (time.perf_counter() - t0) * 1e3 / n

                n = 30 if S <= 4096 else 10
                f_ms = timeit(fwd, n)
                fb_ms = timeit(fwd_bwd, max(3, n // 3)) if with_bwd else float("nan")
                base.setdefault("f", f_ms if name == "mha" else None)
                base.setdefault("fb", fb_ms if name == "mha" else None)
                r = {"layout": name, "d_h": dh, "S": S, "causal": causal, "fwd_ms": round(f_ms, 4),
                     "fwd_bwd_ms": round(fb_ms, 4) if with_bwd else None,
                     "bwd_ms": round(fb_ms - f_ms, 4) if with_bwd else None,
                     "fwd_speedup_vs_mha": round(base["f"] / f_ms, 3),
                     "bwd_speedup_vs_mha": round((base["fb"] - base["f"]) / (fb_ms - f_ms), 3) if with_bwd else None}
                rows.append(r)
                print(json.dumps(r), flush=True)
                del x, wt, d_out, out, d_x, saved, grads, ws, wsb
    print(f"{'layout':8s} {'S':>6s} {'causal':>6s} {'fwd ms':>9s} {'bwd ms':>9s} {'fwd x MHA':>10s} {'bwd x MHA':>10s}")
    for r in rows:
        nb = lambda v, f: format(v, f) if v is not None else format("-", ">" + f.split(".")[0])
        print(f"{r['layout']:8s} {r['S']:6d} {str(r['causal']):>6s} {r['fwd_ms']:9.4f} {nb(r['bwd_ms'], '9.4f')} "
              f"{r['fwd_speedup_vs_mha']:10.3f} {nb(r['bwd_speedup_vs_mha'], '10.3f')}")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="ccgqa_16k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mha", action="store_true", help="skip the same-kernel MHA comparison run")
    ap.add_argument("--no-backward", action="store_true", help="skip the forward+backward measurement")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-step measurement")
    ap.add_argument("--only", choices=["forward", "attention", "prologue", "down_project", "up_project", "backward",
                                       "attention_backward", "prologue_backward", "decode"],
                    help="profiling aid: launch just this stage --steps times (after one full forward) and exit")
    ap.add_argument("--grid-dh", type=int, default=128, choices=[64, 128, 256],
                    help="head width of the --grid run")
    ap.add_argument("--grid", action="store_true",
                    help="latency grid on the axes of the paper's kernel figures (App. D.1: E = 2048, bf16, S = 512..16384, "
                         "causal and non-causal, forward and forward+backward) for four layouts at d_h = --grid-dh, instead "
                         "of the one-line benchmark; prints one JSON line per point and a table")
    ap.add_argument("--cpu-prefix", type=int, default=16384, help="tokens of the causal prefix the oracle is timed on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (a second GPU would take a KV group or a batch item; not built)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2510_04476_amd as P
    from synth_inputs import WORKLOADS, make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    P.load_library()  # raises if the HIP library is not built: there is no fallback
    if args.grid:
        return run_grid(P, torch, args.grid_dh)
    w = WORKLOADS[args.workload]
    cfg = P.config_from_workload(w)
    inp = make_inputs(w, seed=0)
    x, wt = P.weights_to_device(cfg, inp)
    ws = P.new_workspace(cfg, x.device)
    out = torch.empty_like(x)
    saved = P.CCASaved.allocate(cfg, x.device)
    fl = P.forward_flops(cfg)
    # One-time set-up per set of weights (transposed projection weights, folded conv filters, RoPE tables): what a
    # deployment does when it loads the layer.  The timed step reads the prepared buffer; the cost of deriving the
    # same data on every call instead is reported as ms_per_step_unprepared.
    wt_raw = wt
    wt = P.cca_prepare(cfg, wt_raw)
    torch.cuda.synchronize()

    def step():
        P.cca_forward(cfg, wt, x, out=out, saved=None, workspace=ws)

    def step_unprepared():
        P.cca_forward(cfg, wt_raw, x, out=out, saved=None, workspace=ws)

    def backward_buffers():
        from synth_inputs import make_upstream_grad
        g = torch.from_numpy(make_upstream_grad(w, seed=1)).to(x.device, cfg.torch_dtype)
        return dict(d_out=g, d_x=torch.empty_like(x), grads=P.CCAGrads.allocate_like(wt),
                    ws=P.new_backward_workspace(cfg, x.device),
                    d_o=torch.randn_like(saved.o), d_q=torch.empty_like(saved.q), d_k=torch.empty_like(saved.k),
                    d_v=torch.empty_like(saved.v), d_lat=torch.empty_like(saved.lat))

    def decode_setup(Bd):
        """State of Bd sequences with a full cache of random contents (timing only)."""
        cd = P.config_from_workload(dict(w, B=Bd))
        g = torch.Generator(device=x.device).manual_seed(1)
        st = P.CCADecodeState.allocate(cd, x.device)
        for t_ in (st.k_cache, st.v_cache, st.lat_ring):
            t_.copy_(torch.randn(t_.shape, device=x.device, generator=g).to(t_.dtype))
        xd = torch.randn(Bd, cd.d_model, device=x.device, generator=g).to(cd.torch_dtype)
        od = torch.empty_like(xd)
        return cd, st, (lambda: P.cca_decode_step(cd, wt, xd, st, cd.T - 1, out=od))

    if args.only == "decode":
        cd, st, dstep = decode_setup(32)
        for _ in range(args.steps):
            dstep()
        torch.cuda.synchronize()
        print(json.dumps({"only": "decode", "launches": args.steps, "workload": args.workload, "batch": 32,
                          "cache_len": cd.T}))
        return 0
    if args.only:
        P.cca_forward(cfg, wt, x, out=out, saved=saved, workspace=ws)
        bb = backward_buffers() if "backward" in args.only else None
        if bb is not None:  # d_q, d_k, d_v of a real attention backward as inputs of the prologue stage call
            P.cca_attention_backward(cfg, saved.q, saved.k, saved.v, saved.o, saved.lse, bb["d_o"], bb["d_q"],
                                     bb["d_k"], bb["d_v"], workspace=bb["ws"], o_lo=saved.o_lo)
        stage = {
            "forward": lambda: P.cca_forward(cfg, wt, x, out=out, saved=None, workspace=ws),
            "backward": lambda: P.cca_backward(cfg, wt, x, saved, bb["d_out"], d_x=bb["d_x"], grads=bb["grads"],
                                               workspace=bb["ws"]),
            "attention_backward": lambda: P.cca_attention_backward(cfg, saved.q, saved.k, saved.v, saved.o, saved.lse,
                                                                   bb["d_o"], bb["d_q"], bb["d_k"], bb["d_v"],
                                                                   workspace=bb["ws"], o_lo=saved.o_lo),
            "prologue_backward": lambda: P.cca_prologue_backward(cfg, wt, saved.lat, saved.q, saved.k, saved.rnorm,
                                                                 bb["d_q"], bb["d_k"], bb["d_v"], d_lat=bb["d_lat"],
                                                                 grads=bb["grads"], workspace=bb["ws"]),
            "attention": lambda: P.cca_attention(cfg, saved.q, saved.k, saved.v, o=saved.o, lse=None, temp=wt.temp),
            "prologue": lambda: P.cca_prologue(cfg, wt, saved.lat, saved.q, saved.k, saved.v, workspace=ws),
            "down_project": lambda: P.cca_down_project(cfg, x, wt.w_down, lat=saved.lat, workspace=ws),
            "up_project": lambda: P.cca_up_project(cfg, saved.o, wt.w_out, out=out, workspace=ws),
        }[args.only]
        for _ in range(args.steps):
            stage()
        torch.cuda.synchronize()
        # calibration for hardware byte counters: a plain device-to-device copy of known size
        # (reads 256 MiB, writes 256 MiB per launch), three launches
        src = torch.empty(256 << 20, dtype=torch.uint8, device=x.device).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "launches": args.steps, "workload": args.workload,
                          "calibration_copy_bytes_each_way": 256 << 20}))
        return 0

    def prewarm(fn, seconds):
        """Untimed calls of fn for `seconds` of wall-clock.  After an idle gap as short as 0.1 s the chip needs some
        50 ms of work to return to the clocks it sustains (measured: the same 20 steps take 0.735 ms each from cold and
        0.668 ms once warm), so every timed region is entered from sustained work, never from idle."""
        t0, n = time.perf_counter(), 0
        while time.perf_counter() - t0 < seconds:
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            n += 5
        return n

    def timed(fn, n):
        """Average duration of n back-to-back launches of fn: one HIP event before the first and one after the
        last, both on the stream the launches go to (torch's current stream, the one the binding passes)."""
        prewarm(fn, 0.05)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    # ---- measured ceilings beside the nominal peaks: matrix-core rate of an MFMA-only kernel (the clock the chip
    #      holds under that load sets it), and the device-to-device copy rate of a 1 GiB buffer (read + write).
    #      Taken first, outside every timed region. ------------------------------------------------------------
    mfma_meas = P.cca_probe_mfma_rate()
    mfma_meas_random = P.cca_probe_mfma_rate(random_operands=True)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=x.device).fill_(1)
    dst = torch.empty_like(src)
    copy_ms = timed(lambda: dst.copy_(src), 5)
    hbm_meas = 2.0 * src.numel() / copy_ms / 1e6
    del src, dst

    n_prewarm = prewarm(step, 0.25)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # full-size parity is taken on exactly what was timed: the output of the last timed call (inference form of
    # the attention kernel, prepared weights), copied out before anything else writes `out`
    out_timed = out.clone()
    n_u = max(5, args.steps // 2)
    prewarm(step_unprepared, 0.05)
    t0 = time.perf_counter()
    for _ in range(n_u):
        step_unprepared()
    torch.cuda.synchronize()
    ms_unprepared = (time.perf_counter() - t0) * 1e3 / n_u

    # ---- per-stage kernels on their own, HIP events on the launch stream --------------------
    P.cca_forward(cfg, wt, x, out=out, saved=saved, workspace=ws)

    n_ev = max(10, min(args.steps, 50))
    attn_ms = timed(lambda: P.cca_attention(cfg, saved.q, saved.k, saved.v, o=saved.o, lse=None, temp=wt.temp), n_ev)
    down_ms = timed(lambda: P.cca_down_project(cfg, x, wt.w_down, lat=saved.lat, workspace=ws), n_ev)
    pro_ms = timed(lambda: P.cca_prologue(cfg, wt, saved.lat, saved.q, saved.k, saved.v, workspace=ws), n_ev)
    up_ms = timed(lambda: P.cca_up_project(cfg, saved.o, wt.w_out, out=out, workspace=ws), n_ev)
    attn_tflops = fl["attn"] / attn_ms / 1e9
    # the same kernel, same launch, on all-zero q, k, v: identical instruction stream, constant operands.  What it
    # gains over the run above is what the chip's power management takes on real data (diagnostic, not the roofline).
    zq, zk, zo = torch.zeros_like(saved.q), torch.zeros_like(saved.k), torch.empty_like(saved.o)
    attn_zero_ms = timed(lambda: P.cca_attention(cfg, zq, zk, zk, o=zo, lse=None, temp=wt.temp), n_ev)
    del zq, zk, zo

    # ---- forward + backward (training step of the block): cca_forward saving intermediates, then cca_backward ----
    bwd = None
    if not args.no_backward:
        bb = backward_buffers()

        def train_step():
            P.cca_forward(cfg, wt, x, out=out, saved=saved, workspace=ws)
            P.cca_backward(cfg, wt, x, saved, bb["d_out"], d_x=bb["d_x"], grads=bb["grads"], workspace=bb["ws"])

        n_b = max(5, args.steps // 2)
        prewarm(train_step, 0.1)
        t0 = time.perf_counter()
        for _ in range(n_b):
            train_step()
        torch.cuda.synchronize()
        fb_ms = (time.perf_counter() - t0) * 1e3 / n_b
        b_ms = timed(lambda: P.cca_backward(cfg, wt, x, saved, bb["d_out"], d_x=bb["d_x"], grads=bb["grads"],
                                            workspace=bb["ws"]), n_ev)
        ab_ms = timed(lambda: P.cca_attention_backward(cfg, saved.q, saved.k, saved.v, saved.o, saved.lse, bb["d_o"],
                                                       bb["d_q"], bb["d_k"], bb["d_v"], workspace=bb["ws"],
                                                       o_lo=saved.o_lo), n_ev)
        pb_ms = timed(lambda: P.cca_prologue_backward(cfg, wt, saved.lat, saved.q, saved.k, saved.rnorm, bb["d_q"],
                                                      bb["d_k"], bb["d_v"], d_lat=bb["d_lat"], grads=bb["grads"],
                                                      workspace=bb["ws"]), n_ev)
        # adjoint work: every projection twice (input and weight gradient), the convolutions twice, attention
        # five contractions instead of two (recomputed scores are extra work and not counted)
        bwd_flops = 2.0 * fl["proj"] + 2.0 * fl["conv"] + 2.5 * fl["attn"]
        bwd = {"fwd_bwd_ms": round(fb_ms, 4), "backward_ms": round(b_ms, 4),
               "fwd_bwd_tflops": round((fl["total"] + bwd_flops) / fb_ms / 1e9, 1),
               "backward_tflops": round(bwd_flops / b_ms / 1e9, 1), "backward_flops": bwd_flops,
               "attention_backward_ms": round(ab_ms, 4),
               "attention_backward_tflops": round(2.5 * fl["attn"] / ab_ms / 1e9, 1),
               "prologue_backward_ms": round(pb_ms, 4)}
        del bb

    # ---- same-kernel MHA baseline (compression 1, 16 x 128 heads, no transforms) ------------
    mha = None
    if args.workload == "ccgqa_16k" and not args.no_mha:
        wm = WORKLOADS["mha_16k"]
        cm = P.config_from_workload(wm)
        im = make_inputs(wm, seed=0)
        xm, wtm = P.weights_to_device(cm, im)
        wtm = P.cca_prepare(cm, wtm)  # prepared like the CCGQA weights it is compared with
        wsm = P.new_workspace(cm, xm.device)
        outm = torch.empty_like(xm)
        prewarm(lambda: P.cca_forward(cm, wtm, xm, out=outm, workspace=wsm), 0.1)
        t0 = time.perf_counter()
        n_m = max(5, args.steps // 2)
        for _ in range(n_m):
            P.cca_forward(cm, wtm, xm, out=outm, workspace=wsm)
        torch.cuda.synchronize()
        mha_ms = (time.perf_counter() - t0) * 1e3 / n_m
        flm = P.forward_flops(cm)
        mha = {"ms_per_step": round(mha_ms, 4), "tflops": round(flm["total"] / mha_ms / 1e9, 1),
               "speedup_ccgqa_vs_mha": round(mha_ms / ms, 3), "flop_ratio": round(flm["total"] / fl["total"], 3)}
        del xm, wtm, wsm, outm

    # ---- head-to-head at B = 4 (timing only: tensors of the same distributions drawn on the device) ----------
    h2h = None
    if args.workload == "ccgqa_16k" and not args.no_mha:
        def time_b4(name):
            wb = WORKLOADS[name]
            cb = P.config_from_workload(wb)
            g = torch.Generator(device=x.device).manual_seed(0)
            rn = lambda *sh, sc=1.0: (torch.randn(*sh, device=x.device, generator=g) * sc).to(cb.torch_dtype)
            xb = rn(cb.B, cb.T, cb.d_model)
            wtb = P.CCAWeights(w_down=rn(cb.d_model, cb.n_lat, sc=0.02), w_out=rn(cb.e_q, cb.d_model, sc=0.02),
                               w_conv_seq=rn(cb.e_q + cb.e_kv, cb.k_seq, sc=0.02),
                               w_conv_ch=rn(cb.n_q_heads + cb.n_kv_heads, cb.head_dim, cb.head_dim, cb.k_ch, sc=0.02),
                               temp=torch.randn(cb.n_kv_heads, device=x.device, generator=g) * 0.02)
            wtb = P.cca_prepare(cb, wtb)
            wsb = P.new_workspace(cb, x.device)
            ob = torch.empty_like(xb)
            prewarm(lambda: P.cca_forward(cb, wtb, xb, out=ob, workspace=wsb), 0.1)
            t0 = time.perf_counter()
            for _ in range(5):
                P.cca_forward(cb, wtb, xb, out=ob, workspace=wsb)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / 5, P.forward_flops(cb)["total"]
        c_ms, c_fl = time_b4("ccgqa_16k_b4")
        m_ms, m_fl = time_b4("mha_16k_b4")
        h2h = {"ccgqa_ms": round(c_ms, 4), "ccgqa_tflops": round(c_fl / c_ms / 1e9, 1), "mha_ms": round(m_ms, 4),
               "mha_tflops": round(m_fl / m_ms / 1e9, 1), "speedup_ccgqa_vs_mha": round(m_ms / c_ms, 3),
               "flop_ratio": round(m_fl / c_fl, 3)}

    # ---- decode step against a full latent KV cache (timing only; parity is tests/test_gpu_decode.py) ----------
    dec = None
    if args.workload == "ccgqa_16k" and not args.no_decode:
        Bd = 32
        cd, st, dstep = decode_setup(Bd)
        d_ms = timed(dstep, 20)
        cache_b = 2.0 * Bd * cd.T * cd.e_kv * 2
        weight_b = (cd.d_model * cd.n_lat + cd.e_q * cd.d_model) * 2.0
        dec = {"batch": Bd, "cache_len": cd.T, "ms_per_step": round(d_ms, 4),
               "tokens_per_s": round(Bd / d_ms * 1e3, 1),
               "hbm_bytes_per_step": int(cache_b + weight_b),
               "achieved_gbps": round((cache_b + weight_b) / d_ms / 1e6, 1), "peak_gbps": 8000.0,
               "frac": round((cache_b + weight_b) / d_ms / 1e6 / 8000.0, 4),
               "kv_cache_bytes_per_token": int(2 * cd.e_kv * 2),
               "mha_kv_cache_bytes_per_token": int(2 * cd.d_model * 2)}
        del st

    # ---- CPU oracle on a causal prefix of the same inputs -----------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import cca_oracle as O
        Tp = min(args.cpu_prefix, w["T"])
        flags = {} if w.get("paper_flags", True) else dict(
            use_conv_seq=False, use_conv_ch=False, use_qk_mean=False, use_v_shift=False, use_qk_norm=False,
            use_key_temp=False, use_rope=False)
        t0 = time.perf_counter()
        ref = O.cca_forward(inp["x"][:, :Tp], inp["w_down"], inp["w_conv_seq"], inp["w_conv_ch"], inp["temp"],
                            inp["w_out"], n_q_heads=w["Hq"], n_kv_heads=w["Hk"], head_dim=w["dh"], **flags)
        cpu_s = time.perf_counter() - t0
        cfg_p = P.config_from_workload(dict(w, T=Tp))
        cpu_tflops = P.forward_flops(cfg_p)["total"] / cpu_s / 1e12
        def parity(t):
            got = t[:, :Tp].float().cpu().numpy().astype(np.float64)
            return (float(np.linalg.norm(got - ref["out"]) / np.linalg.norm(ref["out"])),
                    float(np.abs(got - ref["out"]).max()))
        rel, mx = parity(out_timed)  # the timed call's own output
        P.cca_forward(cfg, wt_raw, x, out=out, saved=saved, workspace=ws)  # the form a training step runs
        torch.cuda.synchronize()
        rel_s, mx_s = parity(out)
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count()
        threads = int(os.environ.get("OMP_NUM_THREADS", cores))
        cpu = {"value": round(cpu_tflops, 4), "unit": "TFLOP/s", "cores": min(cores, threads), "kind": "oracle",
               "sample": f"causal prefix: first {Tp} of {w['T']} tokens of the same inputs, fp64 NumPy, {cpu_s:.1f} s",
               "parity_rel_l2": rel, "parity_max_abs": mx, "parity_of": "output of the timed inference call",
               "parity_saving_form_rel_l2": rel_s, "parity_saving_form_max_abs": mx_s}

    ceilings = {"mfma_bf16_tflops_measured": round(mfma_meas, 1),
                "mfma_bf16_tflops_measured_random_operands": round(mfma_meas_random, 1),
                "mfma_bf16_tflops_nominal": PEAK_BF16_TFLOPS,
                "hbm_copy_gbps_measured": round(hbm_meas, 1), "hbm_gbps_nominal": 8000.0,
                "attention_frac_of_measured_mfma": round(attn_tflops / mfma_meas, 4),
                "attention_frac_of_measured_mfma_random_operands": round(attn_tflops / mfma_meas_random, 4),
                "attention_tflops_same_kernel_zero_inputs": round(fl["attn"] / attn_zero_ms / 1e9, 1)}

    res = {
        "metric": "CCGQA prefill TFLOP/s (causal attention counted at half the dense T^2 term) at T=16k, 1 MI355X",
        "value": round(fl["total"] / ms / 1e9, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "prewarm_steps": n_prewarm,
        "ms_per_step": round(ms, 4),
        "ms_per_step_unprepared": round(ms_unprepared, 4),
        "pct_bf16_mfma_peak": round(fl["total"] / ms / 1e9 / PEAK_BF16_TFLOPS * 100, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={w['B']} T={w['T']} d_model={w['E']} Hq={w['Hq']} Hk={w['Hk']} "
                               f"d_h={w['dh']} k_seq={w['k_seq']} k_ch={w['k_ch']} causal",
                   "flops_per_step": fl["total"]},
        "stages_ms": {"down_project": round(down_ms, 4), "prologue": round(pro_ms, 4),
                      "attention": round(attn_ms, 4), "up_project": round(up_ms, 4)},
        "stages_tflops": {"down_project": round(2.0 * cfg.B * cfg.T * cfg.d_model * cfg.n_lat / down_ms / 1e9, 1),
                          "attention": round(attn_tflops, 1),
                          "up_project": round(2.0 * cfg.B * cfg.T * cfg.e_q * cfg.d_model / up_ms / 1e9, 1)},
        "prologue_gbps": round((cfg.B * cfg.T * (cfg.n_lat + cfg.e_q + 2 * cfg.e_kv) * 2) / pro_ms / 1e6, 1),
        "backward": bwd,
        "mha_same_kernel": mha,
        "head_to_head_b4": h2h,
        "decode": dec,
        "roofline": {"kernel": "attn_fwd_kernel (latent attention)", "bound": "mfma",
                     "achieved": round(attn_tflops, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": ATTN_TRAFFIC_BYTES.get(args.workload),
                     "flops_per_launch": fl["attn"], "avg_launch_ms": round(attn_ms, 4)},
        "measured_ceilings": ceilings,
        "cpu_baseline": cpu,
        "paper_context": "H100 bf16, S=16k: fused CCA kernel ~1.7x prefill vs MHA (CCA-4x); decoupled C1=2/C2=8 layout 1.3-1.4x",
    }
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
