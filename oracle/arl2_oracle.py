"""ctypes front end of the CPU oracle (``arl2_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Nothing here touches the GPU library, and the GPU library never imports this
module: the oracle is the independent definition that parity tests compare
against.  Only ``tests/``, the smoke check and the benchmark's ``cpu_baseline``
leg may use it.

Array conventions (numpy, C-contiguous):
  q [B,Lq,H,D], k,v [B,Lkv,H,D], g [B,Lq,H], S [B,H,D,D] (S[d_k, d_v]), gate [B,H].
q,k,v,g are converted to float32, which is exact for fp32 and bf16 stored
values; S and gate are float64 in the fp64 oracle.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "arl2_oracle.c")
_LIB = os.path.join(_HERE, "libarl2_oracle.so")
_LIB_SAN = os.path.join(_HERE, "libarl2_oracle_san.so")
_lib = None

L2_EPS = 1e-6  # the paper gives no epsilon for L2Norm in Eq. (3); this is the chosen reading


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc.  Building the checker is not using it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=native", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized(force: bool = False) -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (host code only), every finding
    fatal.  A process that loads it must have the AddressSanitizer runtime loaded first (see sanitizer_env)."""
    if force or not os.path.exists(_LIB_SAN) or os.path.getmtime(_LIB_SAN) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-o", _LIB_SAN, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_SAN


def sanitizer_env(env: dict) -> dict:
    """Environment for a child process that is to run the oracle from the sanitized library: the sanitizer
    runtime goes in front of whatever is preloaded already, leaks of the interpreter itself are not reported."""
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, stdout=subprocess.PIPE, text=True).stdout.strip()
    out = dict(env)
    out["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    out["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    out["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    out["ARL2_ORACLE_SANITIZED"] = "1"
    return out


def _load():
    global _lib
    if _lib is None:
        if os.environ.get("ARL2_ORACLE_SANITIZED") == "1":
            lib = ctypes.CDLL(build_sanitized())
        else:
            build()
            lib = ctypes.CDLL(_LIB)
        i32, f64, f32, vp = ctypes.c_int, ctypes.c_double, ctypes.c_float, ctypes.c_void_p
        lib.arl2o_fwd_f64.argtypes = [i32] * 5 + [vp] * 5 + [f64, f64, vp, i32, vp]
        lib.arl2o_fwd_f64.restype = i32
        lib.arl2o_commit_f64.argtypes = [i32] * 4 + [vp] * 3 + [f64, vp]
        lib.arl2o_commit_f64.restype = i32
        lib.arl2o_fwd_f32.argtypes = [i32] * 5 + [vp] * 5 + [f32, f32, vp, i32, vp]
        lib.arl2o_fwd_f32.restype = i32
        lib.arl2o_commit_f32.argtypes = [i32] * 4 + [vp] * 3 + [f32, vp]
        lib.arl2o_commit_f32.restype = i32
        lib.arl2o_commit_delta_f64.argtypes = [i32] * 4 + [vp] * 4 + [f64, vp]
        lib.arl2o_commit_delta_f64.restype = i32
        lib.arl2o_fwd_ex_f64.argtypes = [i32] * 5 + [vp] * 6 + [i32, f64, f64, vp, i32, vp]
        lib.arl2o_fwd_ex_f64.restype = i32
        lib.arl2o_feature_map_f64.argtypes = [i32] * 4 + [vp] * 5
        lib.arl2o_feature_map_f64.restype = i32
        lib.arl2o_gate_proj_f64.argtypes = [i32] * 4 + [vp] * 3
        lib.arl2o_gate_proj_f64.restype = i32
        lib.arl2o_commit_gdn_f64.argtypes = [i32] * 4 + [vp] * 4 + [f64, vp]
        lib.arl2o_commit_gdn_f64.restype = i32
        lib.arl2o_num_threads.restype = i32
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the oracle's OpenMP loops actually use."""
    return int(_load().arl2o_num_threads())


def _c(a, dtype):
    return np.ascontiguousarray(np.asarray(a), dtype=dtype)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_shapes(q, k, v, S, g):
    if q.ndim != 4 or k.ndim != 4 or v.ndim != 4:
        raise ValueError("q, k, v must be [B, L, H, D]")
    B, Lq, H, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[2] != H or k.shape[3] != D:
        raise ValueError("k, v must be [B, Lkv, H, D] matching q")
    if S is not None and S.shape != (B, H, D, D):
        raise ValueError("S must be [B, H, D, D]")
    if g is not None and g.shape != (B, Lq, H):
        raise ValueError("g must be [B, Lq, H]")
    return B, H, Lq, k.shape[1], D


def fwd(q, k, v, S=None, g=None, *, sm_scale: Optional[float] = None, l2_eps: float = L2_EPS,
        rows: Optional[Sequence[int]] = None, precision: str = "f64", q_lin=None) -> np.ndarray:
    """Readout pass: out = softmax(q k^T * sm_scale) v + g * L2Norm(q) S   (Eq. 2, 3, 5, 6).

    ``q_lin`` (fp64 path only), if given, is the row the inter branch normalises instead of q:
    RoPE(phi_q(Q)) of Eq. (3).  A 4-dimensional ``g`` [B, Lq, H, D] (fp64 path only) is one gate per
    output feature and a 2-dimensional ``g`` [B, Lq] one gate per token shared by the heads: the
    element-wise and the scalar granularity of the paper's gate ablation.

    ``rows`` restricts the computation to those query indices (each output row
    depends only on its own q row and on all of k, v, S); the result is then
    [B, len(rows), H, D].  ``precision`` is "f64" or "f32" (every operation in float).
    """
    lib = _load()
    q, k, v = _c(q, np.float32), _c(k, np.float32), _c(v, np.float32)
    g = None if g is None else _c(g, np.float32)
    st = np.float64 if precision == "f64" else np.float32
    S = None if S is None else _c(S, st)
    g_elem = g is not None and g.ndim == 4
    g_tok = g is not None and g.ndim == 2
    if g_elem and g.shape != q.shape:
        raise ValueError("an element-wise gate must have the shape of q")
    if g_tok and g.shape != q.shape[:2]:
        raise ValueError("a scalar gate must be [B, Lq]")
    B, H, Lq, Lkv, D = _check_shapes(q, k, v, S, None if (g_elem or g_tok) else g)
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(D)  # Eq. (1)
    if rows is None:
        rows_arr, nrows = None, Lq
    else:
        rows_arr = _c(rows, np.int32)
        nrows = int(rows_arr.size)
        if nrows and (rows_arr.min() < 0 or rows_arr.max() >= Lq):
            raise ValueError("row index out of range")
    out = np.empty((B, nrows, H, D), dtype=st)
    if q_lin is not None or g_elem or g_tok:
        if precision != "f64":
            raise ValueError("q_lin and element-wise or scalar gates are supported by the fp64 oracle only")
        if q_lin is not None:
            q_lin = _c(q_lin, np.float32)
            if q_lin.shape != q.shape:
                raise ValueError("q_lin must have the shape of q")
        rc = lib.arl2o_fwd_ex_f64(B, H, Lq, Lkv, D, _ptr(q), _ptr(k), _ptr(v), _ptr(q_lin), _ptr(S), _ptr(g),
                                  1 if g_elem else 2 if g_tok else 0, float(sm_scale), float(l2_eps), _ptr(rows_arr), nrows, _ptr(out))
        if rc != 0:
            raise MemoryError("oracle fwd failed")
        return out
    fn = lib.arl2o_fwd_f64 if precision == "f64" else lib.arl2o_fwd_f32
    rc = fn(B, H, Lq, Lkv, D, _ptr(q), _ptr(k), _ptr(v), _ptr(S), _ptr(g),
            float(sm_scale), float(l2_eps), _ptr(rows_arr), nrows, _ptr(out))
    if rc != 0:
        raise MemoryError("oracle fwd failed")
    return out


def commit(k, v, gate, S, *, l2_eps: float = L2_EPS, precision: str = "f64") -> np.ndarray:
    """State commit: returns gate * S + sum_i L2Norm(k_i)^T v_i   (Eq. 3, Eq. 4 with beta = 1,
    no delta term).  The input S is left untouched; a new array is returned."""
    lib = _load()
    k, v = _c(k, np.float32), _c(v, np.float32)
    st = np.float64 if precision == "f64" else np.float32
    if k.ndim != 4 or k.shape != v.shape:
        raise ValueError("k, v must be [B, L, H, D]")
    B, L, H, D = k.shape
    gate = _c(gate, st)
    S_new = np.array(S, dtype=st, order="C", copy=True)
    if gate.shape != (B, H) or S_new.shape != (B, H, D, D):
        raise ValueError("gate must be [B, H] and S [B, H, D, D]")
    fn = lib.arl2o_commit_f64 if precision == "f64" else lib.arl2o_commit_f32
    rc = fn(B, H, L, D, _ptr(k), _ptr(v), _ptr(gate), float(l2_eps), _ptr(S_new))
    if rc != 0:
        raise MemoryError("oracle commit failed")
    return S_new


def commit_delta(k, v, alpha, beta, S, *, l2_eps: float = L2_EPS) -> np.ndarray:
    """Frame-level gated delta rule, Eq. (4) literally: alpha * S + beta * K'^T (V - K' S), every
    token's correction using the same pre-update S.  fp64; returns a new array."""
    lib = _load()
    k, v = _c(k, np.float32), _c(v, np.float32)
    if k.ndim != 4 or k.shape != v.shape:
        raise ValueError("k, v must be [B, L, H, D]")
    B, L, H, D = k.shape
    alpha, beta = _c(alpha, np.float64), _c(beta, np.float64)
    S_new = np.array(S, dtype=np.float64, order="C", copy=True)
    if alpha.shape != (B, H) or beta.shape != (B, H) or S_new.shape != (B, H, D, D):
        raise ValueError("alpha, beta must be [B, H] and S [B, H, D, D]")
    rc = lib.arl2o_commit_delta_f64(B, H, L, D, _ptr(k), _ptr(v), _ptr(alpha), _ptr(beta), float(l2_eps), _ptr(S_new))
    if rc != 0:
        raise MemoryError("oracle commit_delta failed")
    return S_new


def commit_gdn(k, v, alpha, beta, S, *, l2_eps: float = L2_EPS) -> np.ndarray:
    """Token-sequential gated delta rule (Eq. (4) per token, in token order, per-token gates
    alpha, beta of shape [B, L, H]).  fp64; returns a new array."""
    lib = _load()
    k, v = _c(k, np.float32), _c(v, np.float32)
    if k.ndim != 4 or k.shape != v.shape:
        raise ValueError("k, v must be [B, L, H, D]")
    B, L, H, D = k.shape
    alpha, beta = _c(alpha, np.float64), _c(beta, np.float64)
    S_new = np.array(S, dtype=np.float64, order="C", copy=True)
    if alpha.shape != (B, L, H) or beta.shape != (B, L, H) or S_new.shape != (B, H, D, D):
        raise ValueError("alpha, beta must be [B, L, H] and S [B, H, D, D]")
    rc = lib.arl2o_commit_gdn_f64(B, H, L, D, _ptr(k), _ptr(v), _ptr(alpha), _ptr(beta), float(l2_eps), _ptr(S_new))
    if rc != 0:
        raise MemoryError("oracle commit_gdn failed")
    return S_new


def feature_map(x, W, cos=None, sin=None) -> np.ndarray:
    """Per-head feature map of Eq. (3) without the L2Norm: RoPE(W[h] x) per (token, head), fp64.
    x [B, L, H, D]; W [H, D, D] indexed [head, out, in]; cos, sin [L, D/2] (None: no rotation)."""
    lib = _load()
    x, W = _c(x, np.float32), _c(W, np.float32)
    if x.ndim != 4:
        raise ValueError("x must be [B, L, H, D]")
    B, L, H, D = x.shape
    if W.shape != (H, D, D) or D % 2:
        raise ValueError("W must be [H, D, D] and D even")
    if (cos is None) != (sin is None):
        raise ValueError("give both cos and sin or neither")
    if cos is not None:
        cos, sin = _c(cos, np.float64), _c(sin, np.float64)
        if cos.shape != (L, D // 2) or sin.shape != (L, D // 2):
            raise ValueError("cos, sin must be [L, D/2]")
    y = np.empty((B, L, H, D), dtype=np.float64)
    rc = lib.arl2o_feature_map_f64(B, H, L, D, _ptr(x), _ptr(W), _ptr(cos), _ptr(sin), _ptr(y))
    if rc != 0:
        raise MemoryError("oracle feature_map failed")
    return y


def gate_proj(x, Wg) -> np.ndarray:
    """Mix gate of Eq. (6): sigmoid(x W_g).  x [B, L, dm]; Wg [n, dm], one row per gate output (n = H for
    the headwise gate, 1 for the scalar gate of the gate ablation); fp64 [B, L, n]."""
    lib = _load()
    x, Wg = _c(x, np.float32), _c(Wg, np.float32)
    if x.ndim != 3 or Wg.ndim != 2 or Wg.shape[1] != x.shape[2]:
        raise ValueError("x must be [B, L, dm] and Wg [H, dm]")
    B, L, dm = x.shape
    H = Wg.shape[0]
    G = np.empty((B, L, H), dtype=np.float64)
    if lib.arl2o_gate_proj_f64(B, L, dm, H, _ptr(x), _ptr(Wg), _ptr(G)) != 0:
        raise MemoryError("oracle gate_proj failed")
    return G


def rollout(chunks, S0=None, *, l2_eps: float = L2_EPS, precision: str = "f64", rows=None):
    """Alg. 1's call pattern on given tensors: S starts at zero (or S0); per chunk every
    readout pass sees the same pre-update S, then one commit on the clean k, v.

    ``chunks`` is an iterable of dicts with keys
      "passes": list of (q, k, v, g) tuples,  "k_clean", "v_clean", "gate".
    Returns (list of per-chunk lists of outputs, list of S after each commit).
    """
    st = np.float64 if precision == "f64" else np.float32
    S = None if S0 is None else np.array(S0, dtype=st, copy=True)
    outs, states = [], []
    for ch in chunks:
        if S is None:
            B, _, H, D = np.asarray(ch["k_clean"]).shape
            S = np.zeros((B, H, D, D), dtype=st)
        chunk_outs = [fwd(q, k, v, S, g, l2_eps=l2_eps, rows=rows, precision=precision)
                      for (q, k, v, g) in ch["passes"]]
        outs.append(chunk_outs)
        S = commit(ch["k_clean"], ch["v_clean"], ch["gate"], S, l2_eps=l2_eps, precision=precision)
        states.append(S.copy())
    return outs, states
