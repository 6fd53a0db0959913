"""Seeded synthetic inputs for the ARL^2 hybrid attention step.

This module only draws random tensors of the right shapes and stored dtypes;
it holds none of the method's arithmetic and is the one module that both the
CPU oracle's tests and the GPU path's tests/benchmark may share.

The tensors stand in for the activations of a Wan-2.1-1.3B-lineage model at
832x480 (model dim 1536 = 12 heads x 128; one latent frame = 30 x 52 = 1560
patch tokens; a chunk of 3 latent frames = 4680 tokens): trained weights and
prompts are not available, so q, k, v are i.i.d. normal, the branch-mix gate G
is uniform in the range the paper reports for the learned gate (0.45..0.55),
and forget gates are uniform in the range each configuration names.

Every tensor is a pure function of (seed, configuration name, chunk, pass,
tensor tag) through numpy's counter-based Philox generator, so any part of a
rollout can be regenerated on its own.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int              # independent streams
    H: int              # heads
    D: int              # head dim (d_k = d_v)
    L: int              # tokens per chunk
    chunks: int         # chunks rolled out
    passes: int         # read-only denoising passes per chunk (then one commit)
    io_dtype: str       # "f32" or "bf16": stored dtype of q, k, v, out
    qkv_scale: float    # q, k, v ~ N(0,1) * qkv_scale
    gate_lo: float      # forget gate ~ U(gate_lo, gate_hi) per (stream, head, commit)
    gate_hi: float
    prefill: int        # random commits applied to S = 0 before the first chunk
    mix_lo: float = 0.45    # branch-mix gate G ~ U(mix_lo, mix_hi) per (token, head)
    mix_hi: float = 0.55


WORKLOADS: Dict[str, Workload] = {
    # tiny, fp32 throughout, CPU-checkable in full
    "tiny": Workload("tiny", 1, 2, 64, 64, 4, 2, "f32", 1.0 / 8.0, 0.85, 0.99, 0),
    # one Wan-2.1-1.3B-shaped layer: the configuration the headline metric is quoted on
    "wan_layer": Workload("wan_layer", 1, 12, 128, 4680, 1, 4, "bf16", 1.0, 0.9, 0.999, 8),
    # 64-chunk rollout of the same layer, state carried across chunks
    "wan_rollout": Workload("wan_rollout", 1, 12, 128, 4680, 64, 4, "bf16", 1.0, 0.9, 0.999, 0),
    # 8 independent streams
    "wan_batched": Workload("wan_batched", 8, 12, 128, 4680, 1, 4, "bf16", 1.0, 0.9, 0.999, 8),
    # reduced shapes used by parity tests: several tiles plus a ragged tail
    "ragged_small": Workload("ragged_small", 2, 3, 128, 328, 3, 2, "bf16", 1.0, 0.9, 0.999, 2),
}


def _generator(seed: int, name: str, *ids: int) -> np.random.Generator:
    tag = zlib.crc32(name.encode("utf-8"))
    ss = np.random.SeedSequence([int(seed), int(tag)] + [int(i) for i in ids])
    return np.random.Generator(np.random.Philox(ss))


def _store(x: np.ndarray, io_dtype: str) -> torch.Tensor:
    """fp32 values -> the stored dtype (bf16 rounds to nearest even, once)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16) if io_dtype == "bf16" else t


def normal(seed: int, w: Workload, shape, *ids: int, io_dtype=None) -> torch.Tensor:
    r = _generator(seed, w.name, *ids)
    x = r.standard_normal(size=shape, dtype=np.float32) * np.float32(w.qkv_scale)
    return _store(x, io_dtype or w.io_dtype)


def uniform(seed: int, w: Workload, shape, lo: float, hi: float, *ids: int) -> torch.Tensor:
    r = _generator(seed, w.name, *ids)
    x = r.random(size=shape, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)
    return torch.from_numpy(np.clip(x, lo, hi).astype(np.float32))


# tensor tags
_Q, _K, _V, _G, _KC, _VC, _GATE, _PK, _PV, _PGATE, _TALPHA, _TBETA, _WQ, _WK, _WV, _XH, _WG = range(17)


def pass_inputs(w: Workload, chunk: int, p: int, seed: int = 0
                ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """q, k, v [B,L,H,D] (stored dtype) and mix gate g [B,L,H] fp32 of denoising pass p."""
    shp = (w.B, w.L, w.H, w.D)
    q = normal(seed, w, shp, chunk, p, _Q)
    k = normal(seed, w, shp, chunk, p, _K)
    v = normal(seed, w, shp, chunk, p, _V)
    g = uniform(seed, w, (w.B, w.L, w.H), w.mix_lo, w.mix_hi, chunk, p, _G)
    return q, k, v, g


def clean_inputs(w: Workload, chunk: int, seed: int = 0
                 ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """k, v of the clean pass and the forget gate [B,H] fp32 used by the chunk's commit."""
    shp = (w.B, w.L, w.H, w.D)
    k = normal(seed, w, shp, chunk, 0, _KC)
    v = normal(seed, w, shp, chunk, 0, _VC)
    gate = uniform(seed, w, (w.B, w.H), w.gate_lo, w.gate_hi, chunk, 0, _GATE)
    return k, v, gate


def prefill_inputs(w: Workload, j: int, seed: int = 0
                   ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """k, v, gate of the j-th commit that pre-fills the state before the first chunk."""
    shp = (w.B, w.L, w.H, w.D)
    k = normal(seed, w, shp, j, 0, _PK)
    v = normal(seed, w, shp, j, 0, _PV)
    gate = uniform(seed, w, (w.B, w.H), w.gate_lo, w.gate_hi, j, 0, _PGATE)
    return k, v, gate


def token_gates(w: Workload, chunk: int, seed: int = 0) -> Tuple[torch.Tensor, torch.Tensor]:
    """Per-token forget gates and learning rates [B,L,H] fp32 for the token-sequential commit.

    The forget gates of a chunk multiply to about the chunk-level gate of the same workload
    (each is gate ** (2 u / L), u ~ U(0,1), gate ~ U(gate_lo, gate_hi) per stream and head);
    the learning rates are U(0.05, 0.95), the open unit interval a sigmoid projection produces."""
    gate = uniform(seed, w, (w.B, 1, w.H), w.gate_lo, w.gate_hi, chunk, 1, _GATE)
    u = uniform(seed, w, (w.B, w.L, w.H), 0.0, 1.0, chunk, 0, _TALPHA)
    alpha = torch.pow(gate, 2.0 * u / w.L).to(torch.float32).contiguous()
    beta = uniform(seed, w, (w.B, w.L, w.H), 0.05, 0.95, chunk, 0, _TBETA)
    return alpha, beta


def feature_weights(w: Workload, seed: int = 0) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Stand-ins for the learned per-head 1x1 maps phi_q, phi_k, phi_v: [H, D, D] indexed [head, out, in],
    identity plus N(0, 1/(4 D)) noise (a map adapted from, and still close to, the pretrained
    representation), stored in the workload's dtype."""
    eye = np.eye(w.D, dtype=np.float64)[None]
    out = []
    for tag in (_WQ, _WK, _WV):
        noise = _generator(seed, w.name, 0, 0, tag).standard_normal((w.H, w.D, w.D)) * (0.5 / np.sqrt(w.D))
        out.append(_store(eye + noise, w.io_dtype))
    return tuple(out)


def gate_inputs(w: Workload, chunk: int, p: int, seed: int = 0, n_out: int = 0) -> Tuple[torch.Tensor, torch.Tensor]:
    """Hidden state x [B, L, H*D] ~ N(0,1) and gate weights Wg [n_out, H*D] ~ N(0, 0.01 / (H*D)) in the stored
    dtype (n_out = H rows unless given: H*D rows make the element-wise gate): logits with standard deviation
    0.1, i.e. gates spread over about 0.45..0.55 like the learned ones."""
    dm = w.H * w.D
    x = _store(_generator(seed, w.name, chunk, p, _XH).standard_normal((w.B, w.L, dm), dtype=np.float32), w.io_dtype)
    Wg = _store(_generator(seed, w.name, 0, 0, _WG).standard_normal((n_out or w.H, dm)) * (0.1 / np.sqrt(dm)), w.io_dtype)
    return x, Wg


def rope_tables(w: Workload, grid: Tuple[int, int] = (30, 52)) -> Tuple[torch.Tensor, torch.Tensor]:
    """cos, sin [L, D/2] fp32 of a three-axis rotary embedding over (latent frame, row, column): token l
    sits at (l // (rows * cols), (l // cols) % rows, l % cols); the D/2 pairs are split over the three axes
    (the first takes the remainder), each axis with frequencies 10000 ** (-i / n_axis)."""
    rows, cols = grid
    l = np.arange(w.L)
    pos = np.stack([l // (rows * cols), (l // cols) % rows, l % cols], axis=1).astype(np.float64)
    half = w.D // 2
    n_sp = half // 3
    sizes = [half - 2 * n_sp, n_sp, n_sp]
    ang = np.concatenate([pos[:, a:a + 1] * (10000.0 ** (-np.arange(n) / max(n, 1)))[None, :]
                          for a, n in enumerate(sizes)], axis=1)
    return (torch.from_numpy(np.cos(ang).astype(np.float32)).contiguous(),
            torch.from_numpy(np.sin(ang).astype(np.float32)).contiguous())


def as_f32_numpy(t: torch.Tensor) -> np.ndarray:
    """Stored values widened to float32 (exact for bf16 and fp32)."""
    return t.detach().cpu().to(torch.float32).numpy()
