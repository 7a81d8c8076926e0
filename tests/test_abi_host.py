"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2510_04476_amd as P
from paper_2510_04476_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "cca.h")).read()
    declared = set(re.findall(r"\b(cca_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = P.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert P.cca_version() >= 100
    for s in range(-8, 1):
        assert P.cca_strerror(s) and "unknown" not in P.cca_strerror(s)
    assert "unknown" in P.cca_strerror(-99)


def good():
    return P.CCAConfig(B=1, T=64, d_model=256, n_q_heads=2, n_kv_heads=2, head_dim=32, dtype=B.CCA_F32)


def ws(cfg):
    n = C.c_size_t(0)
    cc = cfg.c()
    return P.load_library().cca_workspace_size(C.byref(cc), C.byref(n), None), n.value


def test_workspace_size_ok_and_null():
    lib = P.load_library()
    st, n = ws(good())
    assert st == B.CCA_OK and n > 0
    cc = good().c()
    assert lib.cca_workspace_size(C.byref(cc), None, None) == B.CCA_ERR_NULL
    assert lib.cca_workspace_size(None, C.byref(C.c_size_t()), None) == B.CCA_ERR_NULL
    # both figures from one call; the backward one agrees with its own entry point
    f, b_, b2 = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    assert lib.cca_workspace_size(C.byref(cc), C.byref(f), C.byref(b_)) == B.CCA_OK
    assert lib.cca_backward_workspace_size(C.byref(cc), C.byref(b2)) == B.CCA_OK
    assert f.value == n and b_.value == b2.value > 0
    only_b = C.c_size_t(0)
    assert lib.cca_workspace_size(C.byref(cc), None, C.byref(only_b)) == B.CCA_OK and only_b.value == b2.value


def test_workspace_sizes_of_a_very_large_shape_do_not_wrap():
    """B * T = 2^23 rows: every per-row buffer is beyond 2^32 bytes, so a 32-bit product anywhere in the size
    arithmetic would show as far too few bytes per token row.  (The small shape carries a larger share of
    buffers that do not grow with the tokens, so its bytes per row bound the large shape's from above.)"""
    small = P.CCAConfig(B=1, T=16384, d_model=2048, n_q_heads=8, n_kv_heads=2, head_dim=128)
    big = P.CCAConfig(B=64, T=131072, d_model=2048, n_q_heads=8, n_kv_heads=2, head_dim=128)
    rows_small, rows_big = 16384, 64 * 131072
    for size in (P.cca_workspace_size, P.cca_backward_workspace_size):
        per_row_small, per_row_big = size(small) / rows_small, size(big) / rows_big
        assert size(big) > 1 << 33
        assert 0.7 * per_row_small <= per_row_big <= per_row_small, (per_row_small, per_row_big)
    assert per_row_big >= 2 * (1536 + 1024 + 2 * 256) * 2  # at least lat, q, k, v and their gradients in bf16
    fixed = P.cca_prepared_size(small)
    assert fixed <= P.cca_prepared_size(big) < 2 * fixed  # RoPE table rows grow with T, nothing else


def test_compression_factors_are_checked_against_the_head_layout():
    """Sec. 2.2: latent widths E/C1 (queries) and E/C2 (keys, values).  0 = derive; otherwise exact."""
    cfg = P.CCAConfig(B=1, T=64, d_model=2048, n_q_heads=8, n_kv_heads=2, head_dim=128)   # C1 = 2, C2 = 8
    assert ws(cfg)[0] == B.CCA_OK
    for cq, ckv, status in [(2, 8, B.CCA_OK), (2, 0, B.CCA_OK), (0, 8, B.CCA_OK), (4, 8, B.CCA_ERR_SHAPE),
                            (2, 4, B.CCA_ERR_SHAPE), (-1, 0, B.CCA_ERR_SHAPE), (0, -2, B.CCA_ERR_SHAPE),
                            (1, 1, B.CCA_ERR_SHAPE)]:
        cfg.compress_q, cfg.compress_kv = cq, ckv
        assert ws(cfg)[0] == status, (cq, ckv)
    mha = P.CCAConfig(B=1, T=64, d_model=2048, n_q_heads=16, n_kv_heads=16, head_dim=128, flags=B.CCA_FLAGS_MHA,
                      compress_q=1, compress_kv=1)
    assert ws(mha)[0] == B.CCA_OK
    # a latent that is not an integer fraction of d_model is accepted only with the factor left at 0
    odd = P.CCAConfig(B=1, T=64, d_model=512, n_q_heads=3, n_kv_heads=3, head_dim=128)
    assert ws(odd)[0] == B.CCA_OK
    odd.compress_q = 1
    assert ws(odd)[0] == B.CCA_ERR_SHAPE


def test_prepare_validation_and_size():
    lib = P.load_library()
    big = P.CCAConfig(B=1, T=4096, d_model=2048, n_q_heads=8, n_kv_heads=2, head_dim=128)
    cc = big.c()
    n = C.c_size_t(0)
    assert lib.cca_prepared_size(C.byref(cc), C.byref(n)) == B.CCA_OK
    # transposed weights (E x N_lat and e_q x E, bf16) + folded 3-tap filters of 10 heads + RoPE tables
    assert n.value >= 2048 * 1536 * 2 + 1024 * 2048 * 2 + 10 * 128 * 3 * 128 * 2
    assert lib.cca_prepared_size(C.byref(cc), None) == B.CCA_ERR_NULL
    other_b = P.CCAConfig(B=7, T=4096, d_model=2048, n_q_heads=8, n_kv_heads=2, head_dim=128).c()
    m = C.c_size_t(0)
    assert lib.cca_prepared_size(C.byref(other_b), C.byref(m)) == B.CCA_OK and m.value == n.value  # independent of B
    p = C.c_void_p(0x10000)
    w = B.cca_weights(p, p, p, p, p, None)
    assert lib.cca_prepare(C.byref(cc), C.byref(w), p, n.value - 1, None) == B.CCA_ERR_WORKSPACE
    assert lib.cca_prepare(C.byref(cc), C.byref(w), None, n.value, None) == B.CCA_ERR_WORKSPACE
    assert lib.cca_prepare(C.byref(cc), C.byref(w), C.c_void_p(0x10008), n.value, None) == B.CCA_ERR_ALIGN
    assert lib.cca_prepare(C.byref(cc), None, p, n.value, None) == B.CCA_ERR_NULL
    assert lib.cca_prepare(C.byref(cc), C.byref(B.cca_weights(None, p, p, p, p, None)), p, n.value, None) == B.CCA_ERR_NULL
    # fp32 storage has nothing to prepare: size 0 and the call is a no-op that needs no buffer
    f32 = good().c()
    assert lib.cca_prepared_size(C.byref(f32), C.byref(m)) == B.CCA_OK and m.value == 0
    assert lib.cca_prepare(C.byref(f32), C.byref(w), None, 0, None) == B.CCA_OK
    # a misaligned prepared buffer is refused by cca_forward before anything is enqueued
    wbad = B.cca_weights(p, p, p, p, p, C.c_void_p(0x10004))
    need = ws(big)[1]
    assert lib.cca_forward(C.byref(cc), C.byref(wbad), p, p, None, p, need, None) == B.CCA_ERR_ALIGN


@pytest.mark.parametrize("field,value,status", [
    ("dtype", 7, B.CCA_ERR_DTYPE),
    ("T", 0, B.CCA_ERR_SHAPE),
    ("B", -1, B.CCA_ERR_SHAPE),
    ("n_kv_heads", 3, B.CCA_ERR_LAYOUT),          # H_q % H_k != 0
    ("n_q_heads", 16, B.CCA_ERR_SHAPE),           # latent wider than d_model
    ("k_seq", 9, B.CCA_ERR_UNSUPPORTED),
    ("k_ch", 0, B.CCA_ERR_UNSUPPORTED),
    ("head_dim", 30, B.CCA_ERR_UNSUPPORTED),      # rows would lose 16-byte alignment
    ("flags", 1 << 20, B.CCA_ERR_UNSUPPORTED),
    ("flags", B.CCA_CAUSAL | B.CCA_KEY_TEMP, B.CCA_ERR_UNSUPPORTED),
    ("rope_base", 0.0, B.CCA_ERR_SHAPE),
    ("softmax_scale", -1.0, B.CCA_ERR_SHAPE),
    ("norm_eps", -1e-6, B.CCA_ERR_SHAPE),
    ("norm_eps", float("nan"), B.CCA_ERR_SHAPE),
    ("norm_eps", float("inf"), B.CCA_ERR_SHAPE),
    ("compress_q", 3, B.CCA_ERR_SHAPE),           # 256 != 3 * 2 * 32
    ("compress_kv", 8, B.CCA_ERR_SHAPE),
])
def test_config_validation(field, value, status):
    cfg = good()
    setattr(cfg, field, value)
    assert ws(cfg)[0] == status


def test_forward_rejects_null_misaligned_and_small_workspace():
    lib = P.load_library()
    cfg = good()
    cc = cfg.c()
    # fake but never dereferenced device addresses: validation fails first
    p = C.c_void_p(0x10000)
    w = B.cca_weights(p, p, p, p, p, None)
    need = ws(cfg)[1]
    call = lambda w_, x, out, wsp, n: lib.cca_forward(C.byref(cc), C.byref(w_), x, out, None, wsp, n, None)
    assert call(w, None, p, p, need) == B.CCA_ERR_NULL
    assert call(B.cca_weights(None, p, p, p, p, None), p, p, p, need) == B.CCA_ERR_NULL
    assert call(B.cca_weights(p, None, p, p, p, None), p, p, p, need) == B.CCA_ERR_NULL   # conv flag on, weight missing
    assert call(w, C.c_void_p(0x10008), p, p, need) == B.CCA_ERR_ALIGN
    assert call(w, p, p, p, need - 1) == B.CCA_ERR_WORKSPACE
    assert call(w, p, p, None, need) == B.CCA_ERR_WORKSPACE
    assert lib.cca_attention(C.byref(cc), p, p, None, p, None, None, p, None) == B.CCA_ERR_NULL
    assert lib.cca_prologue(C.byref(cc), None, p, p, p, p, None, p, 0, None) == B.CCA_ERR_NULL
    assert lib.cca_down_project(C.byref(cc), p, None, p, p, 0, None) == B.CCA_ERR_NULL
    assert lib.cca_up_project(C.byref(cc), p, p, None, p, 0, None) == B.CCA_ERR_NULL


def test_backward_rejects_null_misaligned_and_small_workspace():
    lib = P.load_library()
    cfg = good()
    cc = cfg.c()
    p = C.c_void_p(0x10000)  # fake device addresses: validation fails before anything is dereferenced or enqueued
    w = B.cca_weights(p, p, p, p, p, None)
    sv = B.cca_saved(p, p, p, p, p, p, p, None)
    gr = B.cca_grads(p, p, p, p, p)
    n = C.c_size_t(0)
    assert lib.cca_backward_workspace_size(C.byref(cc), C.byref(n)) == B.CCA_OK and n.value > 0
    assert lib.cca_backward_workspace_size(C.byref(cc), None) == B.CCA_ERR_NULL
    need = n.value
    call = lambda w_, x, sv_, d_out, d_x, gr_, wsp, nb: lib.cca_backward(
        C.byref(cc), C.byref(w_), x, C.byref(sv_) if sv_ is not None else None, d_out, d_x,
        C.byref(gr_) if gr_ is not None else None, wsp, nb, None)
    assert call(w, None, sv, p, p, gr, p, need) == B.CCA_ERR_NULL
    assert call(w, p, None, p, p, gr, p, need) == B.CCA_ERR_NULL
    assert call(w, p, sv, None, p, gr, p, need) == B.CCA_ERR_NULL
    assert call(w, p, B.cca_saved(p, p, p, p, p, None, p, None), p, p, gr, p, need) == B.CCA_ERR_NULL  # lse missing
    assert call(w, p, B.cca_saved(p, p, p, p, p, p, None, None), p, p, gr, p, need) == B.CCA_ERR_NULL  # rnorm missing
    assert call(w, p, sv, p, C.c_void_p(0x10004), gr, p, need) == B.CCA_ERR_ALIGN
    assert call(w, p, sv, p, p, B.cca_grads(C.c_void_p(0x10002), p, p, p, p), p, need) == B.CCA_ERR_ALIGN
    assert call(w, p, sv, p, p, gr, p, need - 1) == B.CCA_ERR_WORKSPACE
    assert call(w, p, sv, p, p, gr, None, need) == B.CCA_ERR_WORKSPACE
    # the stage entry points
    assert lib.cca_attention_backward(C.byref(cc), p, p, p, p, None, None, p, p, p, p, p, 1 << 30, None) == B.CCA_ERR_NULL
    assert lib.cca_attention_backward(C.byref(cc), p, p, p, p, None, p, p, p, p, p, p, 16, None) == B.CCA_ERR_WORKSPACE
    assert lib.cca_prologue_backward(C.byref(cc), C.byref(w), p, p, p, None, p, p, p, p, None, p, 1 << 30,
                                     None) == B.CCA_ERR_NULL
    assert lib.cca_prologue_backward(C.byref(cc), C.byref(w), p, p, p, p, p, p, p, p, None, p, 16,
                                     None) == B.CCA_ERR_WORKSPACE


def test_decode_rejects_bad_arguments_and_reports_ring_depth():
    lib = P.load_library()
    cfg = good()
    cc = cfg.c()
    p = C.c_void_p(0x10000)  # fake device addresses: validation fails before anything is dereferenced or enqueued
    w = B.cca_weights(p, p, p, p, p, None)
    st = B.cca_decode_state(p, p, p)
    n, ring = C.c_size_t(0), C.c_int32(0)
    assert lib.cca_decode_workspace_size(C.byref(cc), C.byref(n), C.byref(ring)) == B.CCA_OK and n.value > 0
    assert ring.value == max(cfg.k_seq + cfg.k_ch - 2, 1) + 1  # both convolutions are on in the paper's flags
    assert lib.cca_decode_workspace_size(C.byref(cc), None, None) == B.CCA_ERR_NULL
    noconv = good()
    noconv.flags = B.CCA_FLAGS_MHA
    c2 = noconv.c()
    assert lib.cca_decode_workspace_size(C.byref(c2), C.byref(n), C.byref(ring)) == B.CCA_OK and ring.value == 2
    need = C.c_size_t(0)
    lib.cca_decode_workspace_size(C.byref(cc), C.byref(need), None)
    call = lambda w_, x, st_, pos, out, wsp, nb: lib.cca_decode_step(
        C.byref(cc), C.byref(w_), x, C.byref(st_) if st_ is not None else None, C.c_int32(pos), out, wsp,
        C.c_size_t(nb), None)
    assert call(w, None, st, 0, p, p, need.value) == B.CCA_ERR_NULL
    assert call(w, p, None, 0, p, p, need.value) == B.CCA_ERR_NULL
    assert call(w, p, B.cca_decode_state(p, None, p), 0, p, p, need.value) == B.CCA_ERR_NULL
    assert call(B.cca_weights(None, p, p, p, p, None), p, st, 0, p, p, need.value) == B.CCA_ERR_NULL
    assert call(w, p, st, -1, p, p, need.value) == B.CCA_ERR_SHAPE
    assert call(w, p, st, cfg.T, p, p, need.value) == B.CCA_ERR_SHAPE
    assert call(w, C.c_void_p(0x10004), st, 0, p, p, need.value) == B.CCA_ERR_ALIGN
    assert call(w, p, st, 0, p, p, need.value - 1) == B.CCA_ERR_WORKSPACE
    assert call(w, p, st, 0, p, None, need.value) == B.CCA_ERR_WORKSPACE
    # the ragged form: same checks, the host-side bound takes the place of the position
    rag = lambda pos_arr, mx, wsp, nb: lib.cca_decode_step_ragged(C.byref(cc), C.byref(w), p, C.byref(st), pos_arr,
                                                                  C.c_int32(mx), p, wsp, C.c_size_t(nb), None)
    assert rag(None, 0, p, need.value) == B.CCA_ERR_NULL
    assert rag(p, -1, p, need.value) == B.CCA_ERR_SHAPE
    assert rag(p, cfg.T, p, need.value) == B.CCA_ERR_SHAPE
    assert rag(C.c_void_p(0x10002), 0, p, need.value) == B.CCA_ERR_ALIGN
    assert rag(p, 0, p, need.value - 1) == B.CCA_ERR_WORKSPACE


def test_mfma_probe_rejects_bad_arguments_before_any_launch():
    lib = P.load_library()
    fl = C.c_double(0.0)
    fake = C.c_void_p(0x10000)  # never dereferenced: every case below is refused on the host
    call = lambda out, nbytes, blocks, iters, operands, f: lib.cca_probe_mfma_rate(out, nbytes, blocks, iters, operands, f, None)
    assert call(None, 1 << 20, 4, 8, 0, C.byref(fl)) == B.CCA_ERR_NULL
    assert call(fake, 1 << 20, 4, 8, 0, None) == B.CCA_ERR_NULL
    assert call(fake, 1 << 20, 0, 8, 0, C.byref(fl)) == B.CCA_ERR_SHAPE
    assert call(fake, 1 << 20, 4, 7, 1, C.byref(fl)) == B.CCA_ERR_SHAPE        # odd iteration count
    assert call(fake, 1 << 20, 4, 8, 2, C.byref(fl)) == B.CCA_ERR_UNSUPPORTED  # operand kinds are 0 and 1
    assert call(fake, 4 * 256 * 4 - 1, 4, 8, 0, C.byref(fl)) == B.CCA_ERR_WORKSPACE
    assert call(C.c_void_p(0x10004), 1 << 20, 4, 8, 0, C.byref(fl)) == B.CCA_ERR_ALIGN


def test_flop_counter_matches_cost_table():
    """Forward FLOPs of the cost table: (1/C1 + 1/C2) 4BSE^2 + 4BES^2/C1 + Conv
    (dense attention term; the grouped-conv term counted per actual MAC)."""
    cfg = P.CCAConfig(B=1, T=16384, d_model=2048, n_q_heads=8, n_kv_heads=2, head_dim=128,
                      flags=B.CCA_FLAGS_PAPER & ~B.CCA_CAUSAL)
    Bn, S, E, C1, C2 = 1, 16384, 2048, 2, 8
    f = P.forward_flops(cfg)
    assert f["proj"] == (1 / C1 + 1 / C2) * 4 * Bn * S * E * E
    assert f["attn"] == 4 * Bn * E * S * S / C1
    assert f["conv"] == 2 * Bn * S * ((E / C1 + E / C2) * 2 + (8 + 2) * 128 * 128 * 2)
    mha = P.CCAConfig(B=1, T=16384, d_model=2048, n_q_heads=16, n_kv_heads=16, head_dim=128, flags=0)
    fm = P.forward_flops(mha)
    assert fm["total"] == 8 * Bn * S * E * E + 4 * Bn * E * S * S


def test_cost_model_against_the_papers_cost_table():
    """Parameter count, KV-cache size and forward FLOPs of the four layouts of the latency grid against the paper's
    cost table evaluated at E = 2048, S = 16384 (tests/golden/cost_table_e2048_s16384.txt; the Conv term is covered
    by test_flop_counter_matches_cost_table)."""
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "cost_table_e2048_s16384.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, params, kv, flops = line.split()
                rows[name] = (int(params), int(kv), int(flops))
    layouts = {"MHA": (16, 16), "GQA_G8": (16, 2), "CCA_C4": (4, 4), "CCGQA_C1_2_C2_8": (8, 2)}
    assert set(rows) == set(layouts)
    for name, (hq, hk) in layouts.items():
        cfg = P.CCAConfig(B=1, T=16384, d_model=2048, n_q_heads=hq, n_kv_heads=hk, head_dim=128, flags=0)
        params, kv, flops = rows[name]
        assert cfg.d_model * cfg.n_lat + cfg.e_q * cfg.d_model == params, name   # w_down and w_out as the ABI takes them
        assert 2 * cfg.B * cfg.T * cfg.e_kv == kv, name                          # k_cache + v_cache of cca_decode_state
        f = P.forward_flops(cfg)
        assert f["conv"] == 0 and f["proj"] + f["attn_dense"] == flops, name
