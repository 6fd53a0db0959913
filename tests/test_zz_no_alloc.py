"""The commit entry point that allocates nothing (its partial sums go to a fixed device array) against the
entry point that takes a workspace: same kernels, so the states must agree bit for bit; two calls in a row,
the second on a smaller problem, so that what the first call left in the array is visible to the second."""
import ctypes
import dataclasses

import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def _commit_both(A, w, chunk, S0):
    k, v, gate = (t.cuda() for t in W.clean_inputs(w, chunk))
    lib = A.load_library()
    ws = A.alloc_workspace(w.B, w.H, w.L, w.D, k.dtype)
    S_ref, S_new = S0.clone(), S0.clone()
    d = A.make_desc(w.B, w.H, w.L, w.L, w.D, A.ARL2_BF16 if k.dtype == torch.bfloat16 else A.ARL2_F32, workspace=ws, stream=0)
    vp = ctypes.c_void_p
    assert lib.arl2_state_commit(ctypes.byref(d), vp(k.data_ptr()), vp(v.data_ptr()), vp(gate.data_ptr()), vp(S_ref.data_ptr())) == 0
    d2 = A.make_desc(w.B, w.H, w.L, w.L, w.D, d.io_dtype, stream=0)          # no workspace at all
    assert d2.workspace is None and d2.workspace_bytes == 0
    before = torch.cuda.memory_allocated()
    st = lib.arl2_state_commit_static(ctypes.byref(d2), vp(k.data_ptr()), vp(v.data_ptr()), vp(gate.data_ptr()), vp(S_new.data_ptr()))
    assert st == 0, lib.arl2_last_error()
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return S_ref, S_new


def test_static_scratch_commit_matches_workspace_commit():
    import paper_2605_16579_amd as A
    lib = A.load_library()
    assert lib.arl2_static_scratch_bytes() == 16 << 20
    big = W.WORKLOADS["wan_layer"]
    small = dataclasses.replace(W.WORKLOADS["ragged_small"], name="no_alloc_small")
    torch.manual_seed(0)
    for w, chunk in ((big, 0), (small, 1), (W.WORKLOADS["tiny"], 0)):      # a smaller problem after the large one; fp32 last
        S0 = torch.randn(w.B, w.H, w.D, w.D, device="cuda")
        S_ref, S_new = _commit_both(A, w, chunk, S0)
        assert not torch.equal(S_ref, S0)
        assert torch.equal(S_ref, S_new), f"{w.name}: max diff {(S_ref - S_new).abs().max().item():.3e}"
    # beyond the array: a clear error, nothing launched
    d = A.make_desc(64, 12, 4680, 4680, 128, A.ARL2_BF16, stream=0)
    assert lib.arl2_state_commit_static(ctypes.byref(d), 0x1000, 0x2000, 0x3000, 0x4000) == 2      # ARL2_ERR_UNSUPPORTED
    assert b"scratch" in lib.arl2_last_error()
