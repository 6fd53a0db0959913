"""Shared helpers of the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np
import torch

import workloads as W

# Tolerances of the parity bar: max |gpu - oracle| / max |oracle| per tensor
TOL_BF16_OUT = 2e-2     # bf16 outputs
TOL_STATE = 1e-4        # fp32 state, also after 64 chained commits
TOL_F32 = 1e-5          # fp32-throughout configuration


def rel_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in the GPU result"
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def rel_err_per_head(got, ref) -> float:
    """Worst per-(stream, head) slice error of a state tensor [B,H,D,D]."""
    B, H = ref.shape[:2]
    return max(rel_err(got[b, h], ref[b, h]) for b in range(B) for h in range(H))


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float32).numpy()


def sample_rows(L: int, n: int, seed: int, block: int = 128) -> np.ndarray:
    """n random rows plus the rows at the edges of the first, a middle and the last query tile."""
    r = np.random.default_rng(seed)
    rows = set(r.choice(L, size=min(n, L), replace=False).tolist())
    last0 = (L - 1) // block * block
    for x in (0, 31, 32, 63, 64, 127, 128, last0 - 1, last0, L - 1):
        if 0 <= x < L:
            rows.add(x)
    return np.array(sorted(rows), dtype=np.int32)
