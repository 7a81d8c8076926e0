"""ctypes binding of libcca (include/cca.h).

Argument marshalling only: every step of the block runs in the HIP kernels of
the shared library.  PyTorch supplies device memory and the current stream.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcca.so")

# status codes / enums of include/cca.h
CCA_OK = 0
CCA_ERR_NULL, CCA_ERR_SHAPE, CCA_ERR_LAYOUT, CCA_ERR_UNSUPPORTED = -1, -2, -3, -4
CCA_ERR_WORKSPACE, CCA_ERR_ALIGN, CCA_ERR_DTYPE, CCA_ERR_LAUNCH = -5, -6, -7, -8
CCA_BF16, CCA_F32 = 0, 1
CCA_CAUSAL, CCA_CONV_SEQ, CCA_CONV_CH, CCA_QK_MEAN = 1 << 0, 1 << 1, 1 << 2, 1 << 3
CCA_V_SHIFT, CCA_QK_NORM, CCA_KEY_TEMP, CCA_ROPE = 1 << 4, 1 << 5, 1 << 6, 1 << 7
CCA_ROPE_INTERLEAVED = 1 << 8
CCA_FLAGS_PAPER = (CCA_CAUSAL | CCA_CONV_SEQ | CCA_CONV_CH | CCA_QK_MEAN | CCA_V_SHIFT | CCA_QK_NORM
                   | CCA_KEY_TEMP | CCA_ROPE)
CCA_FLAGS_MHA = CCA_CAUSAL

EXPORTS = ("cca_workspace_size", "cca_backward_workspace_size", "cca_prepared_size", "cca_prepare", "cca_forward",
           "cca_backward", "cca_down_project",
           "cca_prologue", "cca_attention", "cca_attention_backward", "cca_prologue_backward", "cca_up_project",
           "cca_decode_workspace_size", "cca_decode_step", "cca_decode_step_ragged", "cca_decode_step_static", "cca_probe_mfma_rate", "cca_strerror", "cca_version")


class cca_config(C.Structure):
    _fields_ = [("B", C.c_int32), ("T", C.c_int32), ("d_model", C.c_int32),
                ("compress_q", C.c_int32), ("compress_kv", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("k_seq", C.c_int32), ("k_ch", C.c_int32), ("dtype", C.c_int32), ("flags", C.c_uint32),
                ("rope_base", C.c_float), ("softmax_scale", C.c_float), ("norm_eps", C.c_float)]


class cca_weights(C.Structure):
    _fields_ = [("w_down", C.c_void_p), ("w_conv_seq", C.c_void_p), ("w_conv_ch", C.c_void_p),
                ("temp", C.c_void_p), ("w_out", C.c_void_p), ("prepared", C.c_void_p)]


class cca_decode_state(C.Structure):
    _fields_ = [("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("lat_ring", C.c_void_p)]


class cca_saved(C.Structure):
    _fields_ = [("lat", C.c_void_p), ("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p),
                ("o", C.c_void_p), ("lse", C.c_void_p), ("rnorm", C.c_void_p), ("o_lo", C.c_void_p)]


class cca_grads(C.Structure):
    _fields_ = [("w_down", C.c_void_p), ("w_conv_seq", C.c_void_p), ("w_conv_ch", C.c_void_p),
                ("temp", C.c_void_p), ("w_out", C.c_void_p)]


class CCAError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {cca_strerror(status)} (status {status})")


_lib = None


def load_library() -> C.CDLL:
    """Loads libcca.so; raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(LIB_PATH)
    vp, sz = C.c_void_p, C.c_size_t
    cfgp = C.POINTER(cca_config)
    lib.cca_workspace_size.argtypes = [cfgp, C.POINTER(sz), C.POINTER(sz)]
    lib.cca_prepared_size.argtypes = [cfgp, C.POINTER(sz)]
    lib.cca_prepare.argtypes = [cfgp, C.POINTER(cca_weights), vp, sz, vp]
    lib.cca_decode_workspace_size.argtypes = [cfgp, C.POINTER(sz), C.POINTER(C.c_int32)]
    lib.cca_decode_step.argtypes = [cfgp, C.POINTER(cca_weights), vp, C.POINTER(cca_decode_state), C.c_int32, vp, vp,
                                    sz, vp]
    lib.cca_decode_step_ragged.argtypes = [cfgp, C.POINTER(cca_weights), vp, C.POINTER(cca_decode_state), vp, C.c_int32,
                                           vp, vp, sz, vp]
    lib.cca_forward.argtypes = [cfgp, C.POINTER(cca_weights), vp, vp, C.POINTER(cca_saved), vp, sz, vp]
    lib.cca_down_project.argtypes = [cfgp, vp, vp, vp, vp, sz, vp]
    lib.cca_up_project.argtypes = [cfgp, vp, vp, vp, vp, sz, vp]
    lib.cca_prologue.argtypes = [cfgp, C.POINTER(cca_weights), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cca_attention.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.cca_attention_backward.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cca_backward_workspace_size.argtypes = [cfgp, C.POINTER(sz)]
    lib.cca_backward.argtypes = [cfgp, C.POINTER(cca_weights), vp, C.POINTER(cca_saved), vp, vp,
                                 C.POINTER(cca_grads), vp, sz, vp]
    lib.cca_prologue_backward.argtypes = [cfgp, C.POINTER(cca_weights), vp, vp, vp, vp, vp, vp, vp, vp,
                                          C.POINTER(cca_grads), vp, sz, vp]
    lib.cca_decode_step_static.argtypes = [cfgp, C.POINTER(cca_weights), vp, C.POINTER(cca_decode_state), C.c_int32, vp,
                                           vp]
    lib.cca_probe_mfma_rate.argtypes = [vp, sz, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double), vp]
    for name in EXPORTS:
        getattr(lib, name).restype = C.c_int
    lib.cca_strerror.argtypes = [C.c_int]
    lib.cca_strerror.restype = C.c_char_p
    _lib = lib
    return lib


@dataclass
class CCAConfig:
    B: int
    T: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    k_seq: int = 2
    k_ch: int = 2
    dtype: int = CCA_BF16
    flags: int = CCA_FLAGS_PAPER
    rope_base: float = 10000.0
    softmax_scale: float = 0.0
    compress_q: int = 0    # 0: derived from the head layout
    compress_kv: int = 0
    norm_eps: float = 0.0

    def c(self) -> cca_config:
        return cca_config(self.B, self.T, self.d_model, self.compress_q, self.compress_kv, self.n_q_heads,
                          self.n_kv_heads, self.head_dim, self.k_seq, self.k_ch, self.dtype, self.flags,
                          self.rope_base, self.softmax_scale, self.norm_eps)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == CCA_BF16 else torch.float32

    @property
    def e_q(self):
        return self.n_q_heads * self.head_dim

    @property
    def e_kv(self):
        return self.n_kv_heads * self.head_dim

    @property
    def n_lat(self):
        return self.e_q + 2 * self.e_kv


@dataclass
class CCAWeights:
    w_down: torch.Tensor
    w_out: torch.Tensor
    w_conv_seq: torch.Tensor | None = None
    w_conv_ch: torch.Tensor | None = None
    temp: torch.Tensor | None = None
    prepared: torch.Tensor | None = None  # buffer filled by cca_prepare (optional)

    def c(self) -> cca_weights:
        return cca_weights(_ptr(self.w_down), _ptr(self.w_conv_seq), _ptr(self.w_conv_ch), _ptr(self.temp),
                           _ptr(self.w_out), _ptr(self.prepared))


@dataclass
class CCASaved:
    lat: torch.Tensor | None = None
    q: torch.Tensor | None = None
    k: torch.Tensor | None = None
    v: torch.Tensor | None = None
    o: torch.Tensor | None = None
    lse: torch.Tensor | None = None
    rnorm: torch.Tensor | None = None
    o_lo: torch.Tensor | None = None

    @staticmethod
    def allocate(cfg: CCAConfig, device) -> "CCASaved":
        dt = cfg.torch_dtype
        B, T = cfg.B, cfg.T
        return CCASaved(
            lat=torch.empty(B, T, cfg.n_lat, dtype=dt, device=device),
            q=torch.empty(B, T, cfg.n_q_heads, cfg.head_dim, dtype=dt, device=device),
            k=torch.empty(B, T, cfg.n_kv_heads, cfg.head_dim, dtype=dt, device=device),
            v=torch.empty(B, T, cfg.n_kv_heads, cfg.head_dim, dtype=dt, device=device),
            o=torch.empty(B, T, cfg.e_q, dtype=dt, device=device),
            lse=torch.empty(B, cfg.n_q_heads, T, dtype=torch.float32, device=device),
            rnorm=torch.empty(B, T, cfg.n_q_heads + cfg.n_kv_heads, dtype=torch.float32, device=device),
            o_lo=torch.empty(B, T, cfg.e_q, dtype=dt, device=device) if cfg.dtype == CCA_BF16 else None)

    def c(self) -> cca_saved:
        return cca_saved(_ptr(self.lat), _ptr(self.q), _ptr(self.k), _ptr(self.v), _ptr(self.o), _ptr(self.lse),
                         _ptr(self.rnorm), _ptr(self.o_lo))


@dataclass
class CCAGrads:
    """Gradients of the weights, same shapes / storage type as CCAWeights (temp fp32)."""
    w_down: torch.Tensor | None = None
    w_out: torch.Tensor | None = None
    w_conv_seq: torch.Tensor | None = None
    w_conv_ch: torch.Tensor | None = None
    temp: torch.Tensor | None = None

    @staticmethod
    def allocate_like(w: CCAWeights) -> "CCAGrads":
        e = lambda t: None if t is None else torch.empty_like(t)
        return CCAGrads(w_down=e(w.w_down), w_out=e(w.w_out), w_conv_seq=e(w.w_conv_seq), w_conv_ch=e(w.w_conv_ch),
                        temp=e(w.temp))

    def c(self) -> cca_grads:
        return cca_grads(_ptr(self.w_down), _ptr(self.w_conv_seq), _ptr(self.w_conv_ch), _ptr(self.temp),
                         _ptr(self.w_out))


def _ptr(t):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("libcca takes contiguous tensors")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != CCA_OK:
        raise CCAError(status, where)


def cca_strerror(status: int) -> str:
    return load_library().cca_strerror(int(status)).decode()


def cca_version() -> int:
    return load_library().cca_version()


def cca_workspace_size(cfg: CCAConfig) -> int:
    n = C.c_size_t(0)
    cc = cfg.c()
    _check(load_library().cca_workspace_size(C.byref(cc), C.byref(n), None), "cca_workspace_size")
    return n.value


def cca_prepared_size(cfg: CCAConfig) -> int:
    n = C.c_size_t(0)
    cc = cfg.c()
    _check(load_library().cca_prepared_size(C.byref(cc), C.byref(n)), "cca_prepared_size")
    return n.value


def cca_prepare(cfg: CCAConfig, w: CCAWeights) -> CCAWeights:
    """Runs the library's one-time set-up for these weights and returns a copy of `w` whose `prepared` buffer
    cca_forward reads instead of deriving the same data on every call."""
    lib = load_library()
    buf = torch.empty(max(cca_prepared_size(cfg), 256), dtype=torch.uint8, device=w.w_down.device)
    cc, cw = cfg.c(), w.c()
    _check(lib.cca_prepare(C.byref(cc), C.byref(cw), _ptr(buf), buf.numel(), _stream()), "cca_prepare")
    return CCAWeights(w_down=w.w_down, w_out=w.w_out, w_conv_seq=w.w_conv_seq, w_conv_ch=w.w_conv_ch, temp=w.temp,
                      prepared=buf)


def new_workspace(cfg: CCAConfig, device) -> torch.Tensor:
    return torch.empty(max(cca_workspace_size(cfg), 256), dtype=torch.uint8, device=device)


def cca_forward(cfg: CCAConfig, w: CCAWeights, x: torch.Tensor, out: torch.Tensor | None = None,
                saved: CCASaved | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    lib = load_library()
    if out is None:
        out = torch.empty(cfg.B, cfg.T, cfg.d_model, dtype=cfg.torch_dtype, device=x.device)
    if workspace is None:
        workspace = new_workspace(cfg, x.device)
    cc, cw = cfg.c(), w.c()
    cs = saved.c() if saved is not None else None
    _check(lib.cca_forward(C.byref(cc), C.byref(cw), _ptr(x), _ptr(out), C.byref(cs) if cs is not None else None,
                           _ptr(workspace), workspace.numel(), _stream()), "cca_forward")
    return out


def cca_down_project(cfg: CCAConfig, x, w_down, lat=None, workspace=None):
    lib = load_library()
    if lat is None:
        lat = torch.empty(cfg.B, cfg.T, cfg.n_lat, dtype=cfg.torch_dtype, device=x.device)
    if workspace is None:
        workspace = new_workspace(cfg, x.device)
    cc = cfg.c()
    _check(lib.cca_down_project(C.byref(cc), _ptr(x), _ptr(w_down), _ptr(lat), _ptr(workspace), workspace.numel(),
                                _stream()), "cca_down_project")
    return lat


def cca_up_project(cfg: CCAConfig, o, w_out, out=None, workspace=None):
    lib = load_library()
    if out is None:
        out = torch.empty(cfg.B, cfg.T, cfg.d_model, dtype=cfg.torch_dtype, device=o.device)
    if workspace is None:
        workspace = new_workspace(cfg, o.device)
    cc = cfg.c()
    _check(lib.cca_up_project(C.byref(cc), _ptr(o), _ptr(w_out), _ptr(out), _ptr(workspace), workspace.numel(),
                              _stream()), "cca_up_project")
    return out


def cca_prologue(cfg: CCAConfig, w: CCAWeights, lat, q=None, k=None, v=None, workspace=None, rnorm=None):
    lib = load_library()
    dt, dev = cfg.torch_dtype, lat.device
    if q is None:
        q = torch.empty(cfg.B, cfg.T, cfg.n_q_heads, cfg.head_dim, dtype=dt, device=dev)
    if k is None:
        k = torch.empty(cfg.B, cfg.T, cfg.n_kv_heads, cfg.head_dim, dtype=dt, device=dev)
    if v is None:
        v = torch.empty(cfg.B, cfg.T, cfg.n_kv_heads, cfg.head_dim, dtype=dt, device=dev)
    if workspace is None:
        workspace = new_workspace(cfg, dev)
    cc, cw = cfg.c(), w.c()
    _check(lib.cca_prologue(C.byref(cc), C.byref(cw), _ptr(lat), _ptr(q), _ptr(k), _ptr(v), _ptr(rnorm),
                            _ptr(workspace), workspace.numel(), _stream()), "cca_prologue")
    return q, k, v


def cca_attention(cfg: CCAConfig, q, k, v, o=None, lse=None, want_lse=False, temp=None, o_lo=None):
    lib = load_library()
    if o is None:
        o = torch.empty(cfg.B, cfg.T, cfg.e_q, dtype=cfg.torch_dtype, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty(cfg.B, cfg.n_q_heads, cfg.T, dtype=torch.float32, device=q.device)
    cc = cfg.c()
    _check(lib.cca_attention(C.byref(cc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(o_lo), _ptr(lse), _ptr(temp),
                             _stream()), "cca_attention")
    return (o, lse) if want_lse else o


def cca_attention_backward(cfg: CCAConfig, q, k, v, o, lse, d_o, d_q=None, d_k=None, d_v=None, workspace=None,
                           o_lo=None):
    lib = load_library()
    d_q = torch.empty_like(q) if d_q is None else d_q
    d_k = torch.empty_like(k) if d_k is None else d_k
    d_v = torch.empty_like(v) if d_v is None else d_v
    if workspace is None:
        n = cfg.B * cfg.n_q_heads * cfg.T * 4 + 256 + 2 * cfg.B * cfg.T * cfg.e_q * 4 + cfg.B * cfg.T * cfg.e_q * 2
        workspace = torch.empty(n, dtype=torch.uint8, device=q.device)
    cc = cfg.c()
    _check(lib.cca_attention_backward(C.byref(cc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(o_lo), _ptr(lse), _ptr(d_o),
                                      _ptr(d_q),
                                      _ptr(d_k), _ptr(d_v), _ptr(workspace), workspace.numel(), _stream()),
           "cca_attention_backward")
    return d_q, d_k, d_v


def cca_backward_workspace_size(cfg: CCAConfig) -> int:
    n = C.c_size_t(0)
    cc = cfg.c()
    _check(load_library().cca_backward_workspace_size(C.byref(cc), C.byref(n)), "cca_backward_workspace_size")
    return n.value


def new_backward_workspace(cfg: CCAConfig, device) -> torch.Tensor:
    return torch.empty(max(cca_backward_workspace_size(cfg), 256), dtype=torch.uint8, device=device)


def cca_backward(cfg: CCAConfig, w: CCAWeights, x, saved: CCASaved, d_out, d_x=None, grads: CCAGrads | None = None,
                 workspace=None, want_d_x=True):
    """Returns (d_x, grads).  grads=None allocates gradients for every weight of `w`."""
    lib = load_library()
    if d_x is None and want_d_x:
        d_x = torch.empty_like(x)
    if grads is None:
        grads = CCAGrads.allocate_like(w)
    if workspace is None:
        workspace = new_backward_workspace(cfg, x.device)
    cc, cw, cs, cg = cfg.c(), w.c(), saved.c(), grads.c()
    _check(lib.cca_backward(C.byref(cc), C.byref(cw), _ptr(x), C.byref(cs), _ptr(d_out), _ptr(d_x), C.byref(cg),
                            _ptr(workspace), workspace.numel(), _stream()), "cca_backward")
    return d_x, grads


def cca_prologue_backward(cfg: CCAConfig, w: CCAWeights, lat, q, k, rnorm, d_q, d_k, d_v, d_lat=None,
                          grads: CCAGrads | None = None, workspace=None):
    lib = load_library()
    if d_lat is None:
        d_lat = torch.empty_like(lat)
    if grads is None:
        grads = CCAGrads(w_conv_seq=None if w.w_conv_seq is None else torch.empty_like(w.w_conv_seq),
                         w_conv_ch=None if w.w_conv_ch is None else torch.empty_like(w.w_conv_ch),
                         temp=None if w.temp is None else torch.empty_like(w.temp))
    if workspace is None:
        workspace = new_backward_workspace(cfg, lat.device)
    cc, cw, cg = cfg.c(), w.c(), grads.c()
    _check(lib.cca_prologue_backward(C.byref(cc), C.byref(cw), _ptr(lat), _ptr(q), _ptr(k), _ptr(rnorm), _ptr(d_q),
                                     _ptr(d_k), _ptr(d_v), _ptr(d_lat), C.byref(cg), _ptr(workspace),
                                     workspace.numel(), _stream()), "cca_prologue_backward")
    return d_lat, grads


# ---- decode ----------------------------------------------------------------
def cca_decode_workspace_size(cfg: CCAConfig) -> tuple[int, int]:
    """(workspace bytes, ring depth P) of one decode step; cfg.T is the cache capacity."""
    n, p_ = C.c_size_t(0), C.c_int32(0)
    cc = cfg.c()
    _check(load_library().cca_decode_workspace_size(C.byref(cc), C.byref(n), C.byref(p_)), "cca_decode_workspace_size")
    return n.value, p_.value


@dataclass
class CCADecodeState:
    """Device state of a batch of sequences being decoded (see cca_decode_state in cca.h)."""
    k_cache: torch.Tensor   # (B, T, H_k, d_h)
    v_cache: torch.Tensor   # (B, T, H_k, d_h)
    lat_ring: torch.Tensor  # (B, P, N_lat)
    workspace: torch.Tensor

    @staticmethod
    def allocate(cfg: CCAConfig, device) -> "CCADecodeState":
        nbytes, P_ = cca_decode_workspace_size(cfg)
        dt = cfg.torch_dtype
        kv = lambda: torch.zeros(cfg.B, cfg.T, cfg.n_kv_heads, cfg.head_dim, dtype=dt, device=device)
        return CCADecodeState(kv(), kv(), torch.zeros(cfg.B, P_, cfg.n_lat, dtype=dt, device=device),
                              torch.empty(nbytes, dtype=torch.uint8, device=device))

    def load_prefill(self, saved: CCASaved, n_tokens: int) -> None:
        """Take over the first n_tokens of a prefill's saved k, v, lat (argument marshalling: tensor copies only)."""
        self.k_cache[:, :n_tokens].copy_(saved.k[:, :n_tokens])
        self.v_cache[:, :n_tokens].copy_(saved.v[:, :n_tokens])
        P_ = self.lat_ring.shape[1]
        for s in range(max(0, n_tokens - P_), n_tokens):
            self.lat_ring[:, s % P_].copy_(saved.lat[:, s])

    def c(self) -> cca_decode_state:
        return cca_decode_state(_ptr(self.k_cache), _ptr(self.v_cache), _ptr(self.lat_ring))


def cca_decode_step(cfg: CCAConfig, w: CCAWeights, x_new, state: CCADecodeState, pos: int, out=None):
    """out (B, E) for the token at position `pos`; updates `state` (cache row `pos`, latent ring)."""
    lib = load_library()
    if out is None:
        out = torch.empty(cfg.B, cfg.d_model, dtype=cfg.torch_dtype, device=x_new.device)
    cc, cw, cs = cfg.c(), w.c(), state.c()
    _check(lib.cca_decode_step(C.byref(cc), C.byref(cw), _ptr(x_new), C.byref(cs), C.c_int32(pos), _ptr(out),
                               _ptr(state.workspace), C.c_size_t(state.workspace.numel()), _stream()), "cca_decode_step")
    return out


def cca_decode_step_ragged(cfg: CCAConfig, w: CCAWeights, x_new, state: CCADecodeState, pos: torch.Tensor,
                           max_pos: int, out=None):
    """out (B, E): sequence b's new token is at position pos[b] (int32 device tensor of B entries, each within
    [0, max_pos]); updates `state` row pos[b] of each sequence."""
    lib = load_library()
    assert pos.dtype == torch.int32 and pos.is_cuda and pos.is_contiguous() and pos.numel() == cfg.B
    if out is None:
        out = torch.empty(cfg.B, cfg.d_model, dtype=cfg.torch_dtype, device=x_new.device)
    cc, cw, cs = cfg.c(), w.c(), state.c()
    _check(lib.cca_decode_step_ragged(C.byref(cc), C.byref(cw), _ptr(x_new), C.byref(cs), _ptr(pos), C.c_int32(max_pos),
                                      _ptr(out), _ptr(state.workspace), C.c_size_t(state.workspace.numel()), _stream()),
           "cca_decode_step_ragged")
    return out


CCA_DECODE_STATIC_BYTES = 16 << 20


def cca_decode_step_static(cfg: CCAConfig, w: CCAWeights, x_new, state: CCADecodeState, pos: int, out):
    """cca_decode_step on the library's built-in scratch: no workspace argument, nothing allocated (the caller
    passes `out`)."""
    lib = load_library()
    cc, cw, cs = cfg.c(), w.c(), state.c()
    _check(lib.cca_decode_step_static(C.byref(cc), C.byref(cw), _ptr(x_new), C.byref(cs), C.c_int32(pos), _ptr(out),
                                      _stream()), "cca_decode_step_static")
    return out


def cca_probe_mfma_rate(blocks: int = 2048, iters: int = 4096, repeats: int = 10, random_operands: bool = False) -> float:
    """Measured bf16 matrix-core rate in TFLOP/s: `repeats` back-to-back launches of the library's MFMA-only kernel
    under one event pair, after one untimed launch - the rate the chip sustains, not a first-launch burst.  On
    a few small constants or, with `random_operands`, on pseudo-random values as activations are (the chip holds a
    lower clock on those)."""
    lib = load_library()
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    fl = C.c_double(0.0)

    def launch():
        _check(lib.cca_probe_mfma_rate(_ptr(out), out.numel() * 4, blocks, iters, int(random_operands), C.byref(fl),
                                       _stream()), "cca_probe_mfma_rate")

    launch()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(repeats):
        launch()
    b.record()
    torch.cuda.synchronize()
    return repeats * fl.value / (a.elapsed_time(b) * 1e-3) / 1e12
