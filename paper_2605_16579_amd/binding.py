"""ctypes binding of the C ABI in ``include/arl2.h``: argument marshalling only.

Every step of the hybrid attention path runs in the HIP kernels of ``libarl2_hip.so``;
torch is used for device memory and streams.  There is no fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libarl2_hip.so")

ARL2_OK, ARL2_ERR_INVALID_ARG, ARL2_ERR_UNSUPPORTED, ARL2_ERR_WORKSPACE, ARL2_ERR_DEVICE = range(5)
ARL2_F32, ARL2_BF16 = 0, 1
ARL2_GATE_PER_HEAD, ARL2_GATE_PER_ELEMENT, ARL2_GATE_PER_TOKEN = 0, 1, 2

EXPORTS = ["arl2_workspace_bytes", "arl2_hybrid_attn_fwd", "arl2_state_commit", "arl2_state_commit_delta",
           "arl2_static_scratch_bytes", "arl2_state_commit_static", "arl2_state_commit_fm",
           "arl2_gdn_workspace_bytes", "arl2_state_commit_gdn", "arl2_hybrid_attn_fwd_ex", "arl2_hybrid_attn_fwd_fm", "arl2_feature_map", "arl2_gate_proj",
           "arl2_status_string", "arl2_last_error", "arl2_version"]


class arl2_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("Lq", ctypes.c_int32),
                ("Lkv", ctypes.c_int32), ("D", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("g_dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float), ("l2_eps", ctypes.c_float),
                ("g_mode", ctypes.c_int32), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("stream", ctypes.c_void_p)]


class Arl2Error(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name}: {detail}")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the built library (build it first with ``python -m paper_2605_16579_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -m paper_2605_16579_amd.build` (there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        dp = ctypes.POINTER(arl2_desc)
        lib.arl2_workspace_bytes.argtypes = [dp]
        lib.arl2_workspace_bytes.restype = ctypes.c_size_t
        lib.arl2_hybrid_attn_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        lib.arl2_hybrid_attn_fwd.restype = ctypes.c_int
        lib.arl2_state_commit.argtypes = [dp, vp, vp, vp, vp]
        lib.arl2_state_commit.restype = ctypes.c_int
        lib.arl2_state_commit_static.argtypes = [dp, vp, vp, vp, vp]
        lib.arl2_state_commit_static.restype = ctypes.c_int
        lib.arl2_static_scratch_bytes.argtypes = []
        lib.arl2_static_scratch_bytes.restype = ctypes.c_size_t
        lib.arl2_state_commit_fm.argtypes = [dp] + [vp] * 8
        lib.arl2_state_commit_fm.restype = ctypes.c_int
        lib.arl2_state_commit_delta.argtypes = [dp, vp, vp, vp, vp, vp]
        lib.arl2_state_commit_delta.restype = ctypes.c_int
        lib.arl2_hybrid_attn_fwd_ex.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        lib.arl2_hybrid_attn_fwd_ex.restype = ctypes.c_int
        lib.arl2_hybrid_attn_fwd_fm.argtypes = [dp] + [vp] * 10
        lib.arl2_hybrid_attn_fwd_fm.restype = ctypes.c_int
        lib.arl2_feature_map.argtypes = [dp, vp, vp, vp, vp, vp]
        lib.arl2_feature_map.restype = ctypes.c_int
        lib.arl2_gate_proj.argtypes = [dp, vp, vp, vp]
        lib.arl2_gate_proj.restype = ctypes.c_int
        lib.arl2_gdn_workspace_bytes.argtypes = [dp]
        lib.arl2_gdn_workspace_bytes.restype = ctypes.c_size_t
        lib.arl2_state_commit_gdn.argtypes = [dp, vp, vp, vp, vp, vp]
        lib.arl2_state_commit_gdn.restype = ctypes.c_int
        lib.arl2_status_string.argtypes = [ctypes.c_int]
        lib.arl2_status_string.restype = ctypes.c_char_p
        lib.arl2_last_error.argtypes = []
        lib.arl2_last_error.restype = ctypes.c_char_p
        lib.arl2_version.argtypes = []
        lib.arl2_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def _check(status: int) -> None:
    if status != ARL2_OK:
        lib = load_library()
        raise Arl2Error(status, lib.arl2_status_string(status).decode(), lib.arl2_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ARL2_F32
    if t.dtype == torch.bfloat16:
        return ARL2_BF16
    raise TypeError(f"unsupported dtype {t.dtype}: use float32 or bfloat16")


def _dev(t: Optional[torch.Tensor], name: str, shape=None, dtype=None) -> Optional[int]:
    """Device pointer of a contiguous CUDA/HIP tensor (None passes through as NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}")
    return t.data_ptr()


def make_desc(B, H, Lq, Lkv, D, io_dtype, g_dtype=ARL2_F32, sm_scale=0.0, l2_eps=0.0,
              workspace: Optional[torch.Tensor] = None, stream: Optional[int] = None) -> arl2_desc:
    d = arl2_desc()
    d.B, d.H, d.Lq, d.Lkv, d.D = B, H, Lq, Lkv, D
    d.io_dtype, d.g_dtype = io_dtype, g_dtype
    d.sm_scale, d.l2_eps = sm_scale, l2_eps
    d.g_mode = ARL2_GATE_PER_HEAD
    if workspace is not None:
        d.workspace = _dev(workspace, "workspace")
        d.workspace_bytes = workspace.numel() * workspace.element_size()
    else:
        d.workspace, d.workspace_bytes = None, 0
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    d.stream = stream
    return d


def arl2_workspace_bytes(B: int, H: int, L: int, D: int, io_dtype) -> int:
    """Device scratch bytes arl2_state_commit needs for this problem."""
    code = io_dtype if isinstance(io_dtype, int) else (ARL2_BF16 if io_dtype == torch.bfloat16 else ARL2_F32)
    d = make_desc(B, H, L, L, D, code, stream=0)
    return int(load_library().arl2_workspace_bytes(ctypes.byref(d)))


def _gate_layout(d: arl2_desc, g: Optional[torch.Tensor], B: int, Lq: int, H: int, D: int) -> tuple:
    """Sets d.g_mode from the rank of g and returns the shape g must have."""
    if g is not None and g.dim() == 4:                    # one gate per output feature
        d.g_mode = ARL2_GATE_PER_ELEMENT
        return (B, Lq, H, D)
    if g is not None and g.dim() == 2:                    # one gate per token, shared by the heads
        d.g_mode = ARL2_GATE_PER_TOKEN
        return (B, Lq)
    return (B, Lq, H)


def arl2_hybrid_attn_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                         S: Optional[torch.Tensor], g: Optional[torch.Tensor], out: torch.Tensor,
                         *, sm_scale: float = 0.0, l2_eps: float = 0.0, stream: Optional[int] = None) -> None:
    """Read-only denoising pass, enqueued on the current (or given) stream; writes ``out``."""
    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("q and k must be [B, L, H, D]")
    B, Lq, H, D = q.shape
    Lkv = k.shape[1]
    io = _dtype_code(q)
    d = make_desc(B, H, Lq, Lkv, D, io, _dtype_code(g) if g is not None else ARL2_F32, sm_scale, l2_eps,
                  stream=stream)
    g_shape = _gate_layout(d, g, B, Lq, H, D)
    st = load_library().arl2_hybrid_attn_fwd(
        ctypes.byref(d),
        _dev(q, "q"), _dev(k, "k", (B, Lkv, H, D), q.dtype), _dev(v, "v", (B, Lkv, H, D), q.dtype),
        _dev(S, "S", (B, H, D, D), torch.float32), _dev(g, "g", g_shape),
        _dev(out, "out", (B, Lq, H, D), q.dtype))
    _check(st)


def arl2_hybrid_attn_fwd_ex(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, q_lin: Optional[torch.Tensor],
                            S: Optional[torch.Tensor], g: Optional[torch.Tensor], out: torch.Tensor,
                            *, sm_scale: float = 0.0, l2_eps: float = 0.0, stream: Optional[int] = None) -> None:
    """The readout pass with the linear branch's own query ``q_lin`` (None: ``q``)."""
    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("q and k must be [B, L, H, D]")
    B, Lq, H, D = q.shape
    Lkv = k.shape[1]
    io = _dtype_code(q)
    d = make_desc(B, H, Lq, Lkv, D, io, _dtype_code(g) if g is not None else ARL2_F32, sm_scale, l2_eps,
                  stream=stream)
    g_shape = _gate_layout(d, g, B, Lq, H, D)
    st = load_library().arl2_hybrid_attn_fwd_ex(
        ctypes.byref(d),
        _dev(q, "q"), _dev(k, "k", (B, Lkv, H, D), q.dtype), _dev(v, "v", (B, Lkv, H, D), q.dtype),
        _dev(q_lin, "q_lin", (B, Lq, H, D), q.dtype),
        _dev(S, "S", (B, H, D, D), torch.float32), _dev(g, "g", g_shape),
        _dev(out, "out", (B, Lq, H, D), q.dtype))
    _check(st)


def arl2_hybrid_attn_fwd_fm(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, xq: torch.Tensor, Wq: torch.Tensor,
                            rope_cos: Optional[torch.Tensor], rope_sin: Optional[torch.Tensor],
                            S: torch.Tensor, g: Optional[torch.Tensor], out: torch.Tensor,
                            *, sm_scale: float = 0.0, l2_eps: float = 0.0, stream: Optional[int] = None) -> None:
    """The readout pass with the linear branch's query feature map RoPE(Wq[h] xq) computed inside the kernel."""
    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("q and k must be [B, L, H, D]")
    B, Lq, H, D = q.shape
    Lkv = k.shape[1]
    d = make_desc(B, H, Lq, Lkv, D, _dtype_code(q), _dtype_code(g) if g is not None else ARL2_F32, sm_scale, l2_eps,
                  stream=stream)
    g_shape = _gate_layout(d, g, B, Lq, H, D)
    st = load_library().arl2_hybrid_attn_fwd_fm(
        ctypes.byref(d),
        _dev(q, "q"), _dev(k, "k", (B, Lkv, H, D), q.dtype), _dev(v, "v", (B, Lkv, H, D), q.dtype),
        _dev(xq, "xq", (B, Lq, H, D), q.dtype), _dev(Wq, "Wq", (H, D, D), q.dtype),
        _dev(rope_cos, "rope_cos", (Lq, D // 2), torch.float32), _dev(rope_sin, "rope_sin", (Lq, D // 2), torch.float32),
        _dev(S, "S", (B, H, D, D), torch.float32), _dev(g, "g", g_shape),
        _dev(out, "out", (B, Lq, H, D), q.dtype))
    _check(st)


def arl2_feature_map(x: torch.Tensor, W: torch.Tensor, rope_cos: Optional[torch.Tensor],
                     rope_sin: Optional[torch.Tensor], y: torch.Tensor, *, stream: Optional[int] = None) -> None:
    """y = RoPE(W[h] x) per (token, head): the feature map of Eq. (3) without its L2Norm.
    x, y [B, L, H, D] bf16; W [H, D, D] bf16 indexed [head, out, in]; rope_cos, rope_sin [L, D/2] fp32 or None."""
    if x.dim() != 4:
        raise ValueError("x must be [B, L, H, D]")
    B, L, H, D = x.shape
    d = make_desc(B, H, L, L, D, _dtype_code(x), stream=stream)
    st = load_library().arl2_feature_map(
        ctypes.byref(d), _dev(x, "x"), _dev(W, "W", (H, D, D), x.dtype),
        _dev(rope_cos, "rope_cos", (L, D // 2), torch.float32), _dev(rope_sin, "rope_sin", (L, D // 2), torch.float32),
        _dev(y, "y", (B, L, H, D), x.dtype))
    _check(st)


def arl2_gate_proj(x: torch.Tensor, Wg: torch.Tensor, g: torch.Tensor, *, heads: Optional[int] = None,
                   stream: Optional[int] = None) -> None:
    """g = sigmoid(x Wg^T): the mix gate of Eq. (6).  x [B, L, H*D] bf16.  Headwise: Wg [H, H*D] bf16,
    g [B, L, H] fp32 or bf16 (written).  Scalar gate (one per token): Wg [1, H*D], g [B, L], and ``heads``
    names H.  Element-wise gate (one per feature): Wg [H*D, H*D], g [B, L, H, D]."""
    if x.dim() != 3 or Wg.dim() != 2:
        raise ValueError("x must be [B, L, H*D] and Wg [H, H*D], [1, H*D] or [H*D, H*D]")
    B, L, dm = x.shape
    scalar, elem = g.dim() == 2, g.dim() == 4
    if scalar and heads is None:
        raise ValueError("a scalar gate needs the number of heads")
    H = heads if heads is not None else (g.shape[2] if elem else Wg.shape[0])
    if H < 1 or dm % H:
        raise ValueError("the hidden size must be a multiple of the number of heads")
    d = make_desc(B, H, L, L, dm // H, _dtype_code(x), _dtype_code(g), stream=stream)
    if scalar:
        d.g_mode = ARL2_GATE_PER_TOKEN
    elif elem:
        d.g_mode = ARL2_GATE_PER_ELEMENT
    st = load_library().arl2_gate_proj(ctypes.byref(d), _dev(x, "x"),
                                       _dev(Wg, "Wg", (1 if scalar else dm if elem else H, dm), x.dtype),
                                       _dev(g, "g", (B, L) if scalar else (B, L, H, dm // H) if elem else (B, L, H)))
    _check(st)


def arl2_state_commit(k: torch.Tensor, v: torch.Tensor, gate: torch.Tensor, S: torch.Tensor,
                      workspace: torch.Tensor, *, l2_eps: float = 0.0, stream: Optional[int] = None) -> None:
    """Post-denoise update of ``S`` in place, enqueued on the current (or given) stream."""
    if k.dim() != 4:
        raise ValueError("k must be [B, L, H, D]")
    B, L, H, D = k.shape
    d = make_desc(B, H, L, L, D, _dtype_code(k), ARL2_F32, 0.0, l2_eps, workspace=workspace, stream=stream)
    st = load_library().arl2_state_commit(
        ctypes.byref(d), _dev(k, "k"), _dev(v, "v", (B, L, H, D), k.dtype),
        _dev(gate, "gate", (B, H), torch.float32), _dev(S, "S", (B, H, D, D), torch.float32))
    _check(st)


def arl2_static_scratch_bytes() -> int:
    return int(load_library().arl2_static_scratch_bytes())


def arl2_state_commit_static(k: torch.Tensor, v: torch.Tensor, gate: torch.Tensor, S: torch.Tensor, *,
                             l2_eps: float = 0.0, stream: Optional[int] = None) -> None:
    """``arl2_state_commit`` without a workspace: the partial sums go to the library's fixed device array."""
    if k.dim() != 4:
        raise ValueError("k must be [B, L, H, D]")
    B, L, H, D = k.shape
    d = make_desc(B, H, L, L, D, _dtype_code(k), ARL2_F32, 0.0, l2_eps, stream=stream)
    st = load_library().arl2_state_commit_static(
        ctypes.byref(d), _dev(k, "k"), _dev(v, "v", (B, L, H, D), k.dtype),
        _dev(gate, "gate", (B, H), torch.float32), _dev(S, "S", (B, H, D, D), torch.float32))
    _check(st)


def arl2_state_commit_fm(xk: torch.Tensor, Wk: torch.Tensor, rope_cos: Optional[torch.Tensor], rope_sin: Optional[torch.Tensor],
                         xv: torch.Tensor, Wv: torch.Tensor, gate: torch.Tensor, S: torch.Tensor,
                         workspace: torch.Tensor, *, l2_eps: float = 0.0, stream: Optional[int] = None) -> None:
    """``arl2_state_commit`` on RoPE(Wk xk) and Wv xv, the two feature maps computed inside the commit kernel."""
    if xk.dim() != 4:
        raise ValueError("xk must be [B, L, H, D]")
    B, L, H, D = xk.shape
    d = make_desc(B, H, L, L, D, _dtype_code(xk), ARL2_F32, 0.0, l2_eps, workspace=workspace, stream=stream)
    st = load_library().arl2_state_commit_fm(
        ctypes.byref(d), _dev(xk, "xk"), _dev(Wk, "Wk", (H, D, D), xk.dtype),
        _dev(rope_cos, "rope_cos", (L, D // 2), torch.float32), _dev(rope_sin, "rope_sin", (L, D // 2), torch.float32),
        _dev(xv, "xv", (B, L, H, D), xk.dtype), _dev(Wv, "Wv", (H, D, D), xk.dtype),
        _dev(gate, "gate", (B, H), torch.float32), _dev(S, "S", (B, H, D, D), torch.float32))
    _check(st)


def arl2_state_commit_delta(k: torch.Tensor, v: torch.Tensor, gate: torch.Tensor, beta: torch.Tensor,
                            S: torch.Tensor, workspace: torch.Tensor, *, l2_eps: float = 0.0,
                            stream: Optional[int] = None) -> None:
    """Delta-rule update of ``S`` in place (Eq. (4) literally), enqueued on the current (or given) stream."""
    if k.dim() != 4:
        raise ValueError("k must be [B, L, H, D]")
    B, L, H, D = k.shape
    d = make_desc(B, H, L, L, D, _dtype_code(k), ARL2_F32, 0.0, l2_eps, workspace=workspace, stream=stream)
    st = load_library().arl2_state_commit_delta(
        ctypes.byref(d), _dev(k, "k"), _dev(v, "v", (B, L, H, D), k.dtype),
        _dev(gate, "gate", (B, H), torch.float32), _dev(beta, "beta", (B, H), torch.float32),
        _dev(S, "S", (B, H, D, D), torch.float32))
    _check(st)


def arl2_gdn_workspace_bytes(B: int, H: int, L: int, D: int) -> int:
    d = make_desc(B, H, L, L, D, ARL2_BF16, stream=0)
    return int(load_library().arl2_gdn_workspace_bytes(ctypes.byref(d)))


def arl2_state_commit_gdn(k: torch.Tensor, v: torch.Tensor, alpha: torch.Tensor, beta: torch.Tensor,
                          S: torch.Tensor, workspace: torch.Tensor, *, l2_eps: float = 0.0,
                          stream: Optional[int] = None) -> None:
    """Token-sequential gated delta rule on ``S`` in place (Eq. (4) per token, per-token gates
    ``alpha``, ``beta`` of shape [B, L, H]), enqueued on the current (or given) stream."""
    if k.dim() != 4:
        raise ValueError("k must be [B, L, H, D]")
    B, L, H, D = k.shape
    d = make_desc(B, H, L, L, D, _dtype_code(k), ARL2_F32, 0.0, l2_eps, workspace=workspace, stream=stream)
    st = load_library().arl2_state_commit_gdn(
        ctypes.byref(d), _dev(k, "k"), _dev(v, "v", (B, L, H, D), k.dtype),
        _dev(alpha, "alpha", (B, L, H), torch.float32), _dev(beta, "beta", (B, L, H), torch.float32),
        _dev(S, "S", (B, H, D, D), torch.float32))
    _check(st)


def arl2_version() -> int:
    return int(load_library().arl2_version())


def alloc_workspace(B: int, H: int, L: int, D: int, dtype, device="cuda") -> torch.Tensor:
    """Convenience: a torch buffer of arl2_workspace_bytes() bytes."""
    n = arl2_workspace_bytes(B, H, L, D, dtype)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)
