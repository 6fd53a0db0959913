"""Host-side behaviour of the C ABI that needs no GPU: the library loads, exports every declared
symbol, validates arguments before any launch and reports errors as status codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def A():
    import paper_2605_16579_amd as A
    if not os.path.exists(A.binding.LIB_PATH):
        from paper_2605_16579_amd import build
        build.build()
    A.load_library()
    return A


def test_every_declared_symbol_is_exported(A):
    header = open(os.path.join(ROOT, "include", "arl2.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(arl2_[a-z_0-9]+)\s*\(", header))
    assert declared == set(A.binding.EXPORTS), declared ^ set(A.binding.EXPORTS)
    lib = A.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_desc_struct_matches_header(A):
    header = open(os.path.join(ROOT, "include", "arl2.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} arl2_desc;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = re.findall(r"\b(\w+)\s*;", body)
    assert names == [f[0] for f in A.arl2_desc._fields_]
    assert ctypes.sizeof(A.arl2_desc) == 64


def test_status_strings_and_version(A):
    lib = A.load_library()
    assert lib.arl2_status_string(0) == b"ARL2_OK"
    assert lib.arl2_status_string(3) == b"ARL2_ERR_WORKSPACE"
    assert A.arl2_version() >= 100


def test_workspace_bytes(A):
    assert A.arl2_workspace_bytes(1, 2, 64, 64, A.ARL2_F32) == 1 * 64 * 2 * 4
    n = A.arl2_workspace_bytes(1, 12, 4680, 128, A.ARL2_BF16)
    assert n > 0 and n % (12 * 128 * 128 * 4) == 0
    d = A.make_desc(1, 2, 64, 64, 96, A.ARL2_BF16, stream=0)      # unsupported head dim
    assert A.load_library().arl2_workspace_bytes(ctypes.byref(d)) == 0


def _fwd(A, d, q=0x10000000, k=0x20000000, v=0x30000000, S=0x40000000, g=0x50000000, out=0x60000000):
    # the pointers are never dereferenced: every call below must fail validation before any launch
    return A.load_library().arl2_hybrid_attn_fwd(ctypes.byref(d), q, k, v, S, g, out)


def test_fwd_rejects_bad_arguments_before_launch(A):
    lib = A.load_library()
    ok = dict(B=1, H=2, Lq=64, Lkv=64, D=64, io_dtype=A.ARL2_BF16)
    assert lib.arl2_hybrid_attn_fwd(None, 1, 1, 1, 1, 1, 1) == 1
    for bad in (dict(B=0), dict(H=-1), dict(Lq=0), dict(Lkv=0), dict(io_dtype=7)):
        d = A.make_desc(**{**ok, **bad}, stream=0)
        assert _fwd(A, d) == 1, bad
    assert _fwd(A, A.make_desc(**{**ok, "D": 80}, stream=0)) == 2
    d = A.make_desc(**ok, stream=0)
    assert _fwd(A, d, q=None) == 1
    assert _fwd(A, d, out=None) == 1
    assert _fwd(A, d, q=0x10000004) == 1                      # misaligned
    assert _fwd(A, d, out=0x10000000) == 1                    # out aliases q
    assert _fwd(A, d, out=0x10000100) == 1 and b"overlap" in lib.arl2_last_error()   # out = q + one row: overlaps, not equal
    assert _fwd(A, d, out=0x40000040) == 1                    # out inside the state
    assert _fwd(A, d, out=0x20000000 - 256) == 1              # out ends inside k
    d2 = A.make_desc(**{**ok, "Lkv": 128}, stream=0)
    assert _fwd(A, d2) == 1                               # Lkv != Lq with a state
    assert b"Lkv" in lib.arl2_last_error()
    d3 = A.make_desc(**ok, sm_scale=-1.0, stream=0)
    assert _fwd(A, d3) == 1


def test_commit_rejects_bad_arguments_before_launch(A):
    lib = A.load_library()
    d = A.make_desc(1, 2, 64, 64, 64, A.ARL2_BF16, stream=0)
    call = lambda d, k=0x10000000, v=0x20000000, gate=0x30000000, S=0x40000000: lib.arl2_state_commit(ctypes.byref(d), k, v, gate, S)
    assert call(d) == 3                                   # no workspace
    d.workspace, d.workspace_bytes = 0x70000000, 16
    assert call(d) == 3                                   # too small
    d.workspace_bytes = A.arl2_workspace_bytes(1, 2, 64, 64, A.ARL2_BF16)
    assert call(d, S=None) == 1
    assert call(d, gate=0x30000002) == 1
    d.Lkv = 32
    assert call(d) == 1
    # delta-rule variant: needs beta, and bf16 inputs
    d.Lkv = 64
    delta = lambda d, beta=0x50000000: lib.arl2_state_commit_delta(ctypes.byref(d), 0x10000000, 0x20000000, 0x30000000, beta, 0x40000000)
    assert delta(d, beta=None) == 1
    assert delta(d, beta=0x50000002) == 1
    df = A.make_desc(1, 2, 64, 64, 64, A.ARL2_F32, stream=0)
    df.workspace, df.workspace_bytes = 0x70000000, 1 << 20
    assert delta(df) == 2
    # token-sequential variant: its own workspace size, per-token gates, bf16 inputs
    gdn = lambda d, alpha=0x30000000, beta=0x50000000: lib.arl2_state_commit_gdn(ctypes.byref(d), 0x10000000, 0x20000000, alpha, beta, 0x40000000)
    need = A.arl2_gdn_workspace_bytes(1, 2, 64, 64)
    assert need == 2 * (64 * 64 * 8 + 1024)               # two heads, one block of 64 tokens each: Z^T hi/lo, K, V^T, scalars
    assert A.arl2_gdn_workspace_bytes(1, 2, 65, 64) == 2 * need
    d.workspace_bytes = need - 1
    assert gdn(d) == 3                                    # one byte short
    d.workspace_bytes = need
    assert gdn(d, alpha=None) == 1
    assert gdn(d, beta=0x50000002) == 1
    df.workspace_bytes = 1 << 24
    assert gdn(df) == 2


def test_fused_feature_map_commit_rejects_bad_arguments(A):
    lib = A.load_library()
    d = A.make_desc(1, 2, 64, 64, 64, A.ARL2_BF16, stream=0)
    call = lambda d, xk=0x10000000, Wk=0x20000000, c=0x30000000, s=0x34000000, xv=0x40000000, Wv=0x50000000, gate=0x54000000, S=0x60000000: \
        lib.arl2_state_commit_fm(ctypes.byref(d), xk, Wk, c, s, xv, Wv, gate, S)
    assert call(d) == 3                                   # no workspace
    d.workspace, d.workspace_bytes = 0x70000000, A.arl2_workspace_bytes(1, 2, 64, 64, A.ARL2_BF16)
    assert call(d, Wv=None) == 1
    assert call(d, xk=None) == 1
    assert call(d, s=None) == 1                           # cosines without sines
    assert call(d, c=0x30000004) == 1                     # tables must be 8-byte aligned
    assert call(d, gate=0x54000002) == 1
    assert call(d, S=0x10000400) == 1                     # S inside xk
    assert b"overlap" in lib.arl2_last_error()
    assert call(d, Wk=0x70000040) == 1                    # Wk inside the workspace
    d.Lkv = 32
    assert call(d) == 1
    df = A.make_desc(1, 2, 64, 64, 64, A.ARL2_F32, stream=0)
    df.workspace, df.workspace_bytes = 0x70000000, 1 << 20
    assert call(df) == 2                                  # bf16 only


def test_feature_map_and_fwd_ex_reject_bad_arguments(A):
    lib = A.load_library()
    d = A.make_desc(1, 2, 64, 64, 64, A.ARL2_BF16, stream=0)
    fm = lambda d, x=0x10000000, W=0x20000000, c=0x30000000, s=0x40000000, y=0x50000000: lib.arl2_feature_map(ctypes.byref(d), x, W, c, s, y)
    assert fm(d, W=None) == 1
    assert fm(d, c=None) == 1                             # cosines without sines
    assert fm(d, c=0x30000004) == 1                           # tables must be 8-byte aligned
    assert fm(d, y=0x10000000) == 1                           # in place
    df = A.make_desc(1, 2, 64, 64, 64, A.ARL2_F32, stream=0)
    assert fm(df) == 2
    dg = A.make_desc(1, 2, 64, 64, 64, A.ARL2_BF16, stream=0)
    dg.g_mode = 7
    assert lib.arl2_hybrid_attn_fwd(ctypes.byref(dg), 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x74000000, 0x50000000) == 1   # not a gate mode
    dg.g_mode = A.ARL2_GATE_PER_ELEMENT
    assert lib.arl2_hybrid_attn_fwd(ctypes.byref(dg), 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x74000004, 0x50000000) == 1   # element-wise g: 16-byte aligned
    ex = lambda d, ql=0x60000000, out=0x50000000: lib.arl2_hybrid_attn_fwd_ex(ctypes.byref(d), 0x10000000, 0x20000000, 0x30000000, ql, 0x40000000, None, out)
    assert ex(d, ql=0x60000008) == 1                          # misaligned q_lin
    assert ex(d, ql=0x50000000) == 1                          # out aliases q_lin


def test_fused_feature_map_readout_rejects_bad_arguments(A):
    lib = A.load_library()
    d = A.make_desc(1, 2, 64, 64, 64, A.ARL2_BF16, stream=0)
    fm = lambda d, xq=0x60000000, W=0x74000000, c=0x78000000, s=0x7c000000, S=0x40000000, out=0x50000000: lib.arl2_hybrid_attn_fwd_fm(
        ctypes.byref(d), 0x10000000, 0x20000000, 0x30000000, xq, W, c, s, S, None, out)
    assert fm(d, S=None) == 1                             # no state, no linear branch
    assert fm(d, xq=None) == 1
    assert fm(d, s=None) == 1                             # cosines without sines
    assert fm(d, out=0x60000000) == 1                         # out aliases xq
    assert fm(A.make_desc(1, 2, 64, 64, 64, A.ARL2_F32, stream=0)) == 2
    assert fm(A.make_desc(1, 2, 64, 32, 64, A.ARL2_BF16, stream=0)) == 1


def test_gate_proj_rejects_bad_arguments(A):
    lib = A.load_library()
    d = A.make_desc(1, 12, 64, 64, 128, A.ARL2_BF16, stream=0)
    gp = lambda d, x=0x10000000, W=0x20000000, g=0x30000000: lib.arl2_gate_proj(ctypes.byref(d), x, W, g)
    assert gp(d, x=None) == 1
    assert gp(d, W=0x20000008) == 1
    assert gp(d, g=0x10000000) == 1
    assert gp(A.make_desc(1, 12, 64, 64, 128, A.ARL2_F32, stream=0)) == 2


def test_sizes_beyond_the_kernels_addressing_are_refused(A):
    """One stream's k, v (the whole x for the feature map and the gate projection) are addressed with
    32-bit byte offsets: larger problems return ARL2_ERR_UNSUPPORTED instead of launching."""
    lib = A.load_library()
    big = A.make_desc(1, 64, 200000, 200000, 128, A.ARL2_BF16, stream=0)     # 3.3 GB per stream
    big.workspace, big.workspace_bytes = 0x70000000, 1 << 62
    assert lib.arl2_hybrid_attn_fwd(ctypes.byref(big), 0x10000000, 0x20000000, 0x30000000, None, None, 0x50000000) == 2
    assert lib.arl2_state_commit(ctypes.byref(big), 0x10000000, 0x20000000, 0x30000000, 0x40000000) == 2
    assert lib.arl2_state_commit_gdn(ctypes.byref(big), 0x10000000, 0x20000000, 0x30000000, 0x60000000, 0x40000000) == 2
    assert lib.arl2_feature_map(ctypes.byref(big), 0x10000000, 0x20000000, None, None, 0x50000000) == 2
    many = A.make_desc(64, 12, 32768, 32768, 128, A.ARL2_BF16, stream=0)     # each stream small, x as a whole 6.4 GB
    assert lib.arl2_feature_map(ctypes.byref(many), 0x10000000, 0x20000000, None, None, 0x50000000) == 2
    assert lib.arl2_gate_proj(ctypes.byref(many), 0x10000000, 0x20000000, 0x30000000) == 2
    de = A.make_desc(1, 256, 64, 64, 128, A.ARL2_BF16, stream=0)             # element-wise gate: Wg is 32768 x 32768, 2 GiB
    de.g_mode = A.ARL2_GATE_PER_ELEMENT
    assert lib.arl2_gate_proj(ctypes.byref(de), 0x10000000, 0x20000000, 0x30000000) == 2
    assert b"Wg" in lib.arl2_last_error()
    empty = A.make_desc(1, 2, 0, 0, 64, A.ARL2_BF16, stream=0)               # no tokens
    assert lib.arl2_hybrid_attn_fwd(ctypes.byref(empty), 0x10000000, 0x20000000, 0x30000000, None, None, 0x50000000) == 1


def test_binding_refuses_host_tensors(A):
    import torch
    q = torch.zeros((1, 64, 2, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        A.arl2_hybrid_attn_fwd(q, q, q, None, None, torch.empty_like(q))


def test_overlapping_buffers_are_refused(A):
    """Buffers that share bytes without being equal pointers are caught by extent, not by pointer equality."""
    lib = A.load_library()
    d = A.make_desc(1, 2, 64, 64, 64, A.ARL2_BF16, stream=0)
    d.workspace, d.workspace_bytes = 0x70000000, A.arl2_workspace_bytes(1, 2, 64, 64, A.ARL2_BF16)
    k, v, gate, S = 0x10000000, 0x20000000, 0x30000000, 0x40000000
    assert lib.arl2_state_commit(ctypes.byref(d), k, v, gate, 0x70000100) == 1        # S inside the workspace
    assert b"overlap" in lib.arl2_last_error()
    assert lib.arl2_state_commit(ctypes.byref(d), k, v, gate, k + 1024) == 1          # S inside k
    assert lib.arl2_state_commit(ctypes.byref(d), k, 0x70000000 + 4096, gate, S) == 1   # v inside the workspace
    assert lib.arl2_state_commit_delta(ctypes.byref(d), k, v, gate, S + 16, S) == 1   # beta inside S
    d.workspace_bytes = A.arl2_gdn_workspace_bytes(1, 2, 64, 64)
    assert lib.arl2_state_commit_gdn(ctypes.byref(d), k, v, gate, 0x50000000, v + 256) == 1   # S inside v
    assert lib.arl2_feature_map(ctypes.byref(d), k, v, None, None, k + 4096) == 1     # y inside x
    assert lib.arl2_gate_proj(ctypes.byref(d), k, v, k + 64) == 1                      # g inside x
    assert lib.arl2_hybrid_attn_fwd_ex(ctypes.byref(d), k, v, gate, 0x50000000, S, None, 0x50000000 + 2048) == 1   # out inside q_lin
