"""Pins for the CPU oracle: hand-derived values, closed forms, library routines,
brute-force unrollings and invariants.  None of these re-uses the oracle's code.

Each pin names the mistake it is there to catch.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
rng = np.random.default_rng(1234)


def rand(*shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float32)


def l2n(x, eps):
    x = x.astype(np.float64)
    return x / np.sqrt((x * x).sum(-1, keepdims=True) + eps)


# ---------------------------------------------------------------- hand-derived values

def test_hand_example_fwd(oracle):
    ex = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))["fwd"]
    k = np.array([[0.0, 0.0], [math.log(3.0) / 3.0, 0.0]], dtype=np.float64)
    q = np.array(ex["q"])[None, :, None, :]
    v = np.array(ex["v"])[None, :, None, :]
    S = np.array(ex["S"])[None, None]
    g = np.array(ex["g"])[None, :, None]
    # float32 storage of ln3/3 is inexact; recompute the expected weights from the stored value
    k32 = k.astype(np.float32)
    w2 = math.exp(3.0 * float(k32[1, 0]))
    p = np.array([1.0, w2]) / (1.0 + w2)
    assert abs(p[1] - 0.75) < 1e-7
    out = oracle.fwd(q, k32[None, :, None, :], v, S, g, sm_scale=ex["sm_scale"], l2_eps=ex["l2_eps"])
    np.testing.assert_allclose(out[0, :, 0, :], np.array(ex["out"]), rtol=0, atol=2e-6)
    o_intra = oracle.fwd(q, k32[None, :, None, :], v, None, None, sm_scale=1.0, l2_eps=0.0)
    np.testing.assert_allclose(o_intra[0, :, 0, :], np.array(ex["O_intra"]), rtol=0, atol=2e-6)
    # inter branch alone: out(g=1) - out(S=None)
    o_full = oracle.fwd(q, k32[None, :, None, :], v, S, None, sm_scale=1.0, l2_eps=0.0)
    np.testing.assert_allclose((o_full - o_intra)[0, :, 0, :], np.array(ex["O_inter"]), rtol=0, atol=1e-12)


def test_hand_example_commit(oracle):
    ex = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))["commit"]
    k = np.array(ex["k"])[None, :, None, :]
    v = np.array(ex["v"])[None, :, None, :]
    S_old = np.array(ex["S_old"])[None, None]
    for prec, tol in (("f64", 1e-12), ("f32", 1e-5)):
        S_new = oracle.commit(k, v, np.array([[ex["gate"]]]), S_old, l2_eps=ex["l2_eps"], precision=prec)
        np.testing.assert_allclose(S_new[0, 0], np.array(ex["S_new"]), rtol=0, atol=tol)
    # the input state is not modified by the wrapper
    assert np.array_equal(S_old[0, 0], np.array(ex["S_old"]))


# ---------------------------------------------------------------- library routine: zero state = softmax attention

@pytest.mark.parametrize("B,H,Lq,Lkv,D", [(1, 2, 64, 64, 64), (2, 3, 37, 53, 128), (1, 1, 5, 1, 8)])
def test_zero_state_is_softmax_attention(oracle, B, H, Lq, Lkv, D):
    """Catches: wrong scale, softmax over the wrong axis, q/k/v indexing or stride mistakes."""
    q, k, v = rand(B, Lq, H, D), rand(B, Lkv, H, D), rand(B, Lkv, H, D)
    tq, tk, tv = (torch.from_numpy(x).double().permute(0, 2, 1, 3) for x in (q, k, v))
    ref = torch.softmax(tq @ tk.transpose(-1, -2) / math.sqrt(D), dim=-1) @ tv
    ref = ref.permute(0, 2, 1, 3).numpy()
    for S in (None, np.zeros((B, H, D, D))):
        out = oracle.fwd(q, k, v, S, None)
        np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    out32 = oracle.fwd(q, k, v, None, None, precision="f32")
    np.testing.assert_allclose(out32, ref, rtol=0, atol=2e-6)
    # torch's fused kernel as a second library routine
    ref2 = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(oracle.fwd(q, k, v), ref2, rtol=1e-10, atol=1e-12)


def test_softmax_closed_forms(oracle):
    """v == 1 gives 1; k == 0 gives the column mean of v; large logits stay finite."""
    B, H, L, D = 1, 2, 19, 16
    q, k, v = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    np.testing.assert_allclose(oracle.fwd(q, k, np.ones_like(v)), 1.0, rtol=1e-14)
    out = oracle.fwd(q, np.zeros_like(k), v)
    np.testing.assert_allclose(out, np.broadcast_to(v.astype(np.float64).mean(1, keepdims=True), out.shape), rtol=1e-13, atol=1e-15)
    big = oracle.fwd(q * 300, k * 300, v)
    assert np.isfinite(big).all()
    # with huge logits softmax picks the arg-max key's value
    s = np.einsum("blhd,bmhd->bhlm", q.astype(np.float64) * 300, k.astype(np.float64) * 300)
    pick = s.argmax(-1)  # [B,H,L]
    want = np.stack([[v[b, pick[b, h], h, :] for h in range(H)] for b in range(B)])  # [B,H,L,D]
    np.testing.assert_allclose(big, want.transpose(0, 2, 1, 3), rtol=0, atol=1e-6)


# ---------------------------------------------------------------- inter branch

def test_inter_branch_matches_einsum(oracle):
    """out(S) - out(0) = g * L2Norm(q) S, with d_k contracted (not d_v)."""
    B, H, L, D = 2, 3, 11, 32
    q, k, v = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    S = rng.standard_normal((B, H, D, D))
    g = rng.uniform(0, 1, (B, L, H)).astype(np.float32)
    eps = 1e-6
    diff = oracle.fwd(q, k, v, S, g) - oracle.fwd(q, k, v, None, None)
    want = np.einsum("blhd,bhde->blhe", l2n(q, eps), S) * g[..., None].astype(np.float64)
    np.testing.assert_allclose(diff, want, rtol=1e-10, atol=1e-12)
    # g == None means a gate of one; g == 0 switches the branch off
    diff1 = oracle.fwd(q, k, v, S, None) - oracle.fwd(q, k, v, None, None)
    np.testing.assert_allclose(diff1, np.einsum("blhd,bhde->blhe", l2n(q, eps), S), rtol=1e-10, atol=1e-12)
    assert np.array_equal(oracle.fwd(q, k, v, S, np.zeros_like(g)), oracle.fwd(q, k, v, None, None))


def test_query_scale_invariance_and_linearity(oracle):
    """L2Norm makes O_inter independent of |q| (O_intra is not); out is affine in S."""
    B, H, L, D = 1, 2, 9, 16
    q, k, v = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    S1, S2 = rng.standard_normal((B, H, D, D)), rng.standard_normal((B, H, D, D))
    o0 = oracle.fwd(q, k, v, None, None, l2_eps=0.0)
    i1 = oracle.fwd(q, k, v, S1, None, l2_eps=0.0) - o0
    i1_scaled = oracle.fwd(4 * q, k, v, S1, None, l2_eps=0.0) - oracle.fwd(4 * q, k, v, None, None, l2_eps=0.0)
    np.testing.assert_allclose(i1, i1_scaled, rtol=1e-9, atol=1e-12)
    assert np.abs(oracle.fwd(4 * q, k, v) - o0).max() > 1e-3
    i2 = oracle.fwd(q, k, v, S2, None, l2_eps=0.0) - o0
    i12 = oracle.fwd(q, k, v, S1 + S2, None, l2_eps=0.0) - o0
    np.testing.assert_allclose(i12, i1 + i2, rtol=1e-9, atol=1e-11)


def test_zero_rows_do_not_produce_nan(oracle):
    """An all-zero q or k row is defined by eps: it contributes 0, not NaN."""
    B, H, L, D = 1, 1, 4, 8
    q, k, v = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    q[0, 1] = 0
    k[0, 2] = 0
    S = rng.standard_normal((B, H, D, D))
    out = oracle.fwd(q, k, v, S, None)
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out[0, 1], oracle.fwd(q, k, v)[0, 1], rtol=1e-14)
    Sn = oracle.commit(k, v, np.ones((B, H)), np.zeros((B, H, D, D)))
    assert np.isfinite(Sn).all()
    k2, v2 = np.delete(k, 2, axis=1), np.delete(v, 2, axis=1)
    np.testing.assert_allclose(Sn, oracle.commit(k2, v2, np.ones((B, H)), np.zeros((B, H, D, D))), rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- commit

def test_commit_matches_einsum_and_gate_cases(oracle):
    """Catches: transposed outer product, gate applied to the new term, k not normalised."""
    B, H, L, D = 2, 3, 23, 16
    k, v = rand(B, L, H, D), rand(B, L, H, D)
    S = rng.standard_normal((B, H, D, D))
    gate = rng.uniform(0.5, 1.0, (B, H))
    eps = 1e-6
    kv = np.einsum("blhd,blhe->bhde", l2n(k, eps), v.astype(np.float64))
    np.testing.assert_allclose(oracle.commit(k, v, gate, S), gate[..., None, None] * S + kv, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.commit(k, v, np.zeros((B, H)), S), kv, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.commit(k, v, np.ones((B, H)), S), S + kv, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.commit(k, v, gate, S, precision="f32"), gate[..., None, None] * S + kv, rtol=0, atol=2e-5)


def test_associative_memory_identity(oracle):
    """One stored (k, v) pair, gate 1, S = 0: querying with c*k returns v exactly (|k'| = 1)."""
    D = 16
    k, v = rand(1, 1, 1, D), rand(1, 1, 1, D)
    S = oracle.commit(k, v, np.ones((1, 1)), np.zeros((1, 1, D, D)), l2_eps=0.0)
    for c in (1.0, 0.25, 7.0):
        q = (c * k).astype(np.float32)
        inter = oracle.fwd(q, k, v, S, None, l2_eps=0.0) - oracle.fwd(q, k, v, None, None, l2_eps=0.0)
        np.testing.assert_allclose(inter[0, 0, 0], v[0, 0, 0].astype(np.float64), rtol=1e-6, atol=1e-7)


def _tiny_rollout_inputs(N=4, P=2, B=1, H=2, L=12, D=8):
    chunks = []
    for _ in range(N):
        passes = [(rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D),
                   rng.uniform(0.45, 0.55, (B, L, H)).astype(np.float32)) for _ in range(P)]
        chunks.append({"passes": passes, "k_clean": rand(B, L, H, D), "v_clean": rand(B, L, H, D),
                       "gate": rng.uniform(0.85, 0.99, (B, H))})
    return chunks


def test_state_is_unrolled_gated_sum(oracle):
    """After N commits S_N = sum_j (prod_{i>j} gate_i) K'_j^T V_j, computed with no running state."""
    chunks = _tiny_rollout_inputs()
    _, states = oracle.rollout(chunks)
    eps = oracle.L2_EPS
    for N in range(1, len(chunks) + 1):
        want = 0.0
        for j in range(N):
            decay = np.ones_like(chunks[0]["gate"])
            for i in range(j + 1, N):
                decay = decay * chunks[i]["gate"]
            kv = np.einsum("blhd,blhe->bhde", l2n(chunks[j]["k_clean"], eps), chunks[j]["v_clean"].astype(np.float64))
            want = want + decay[..., None, None] * kv
        np.testing.assert_allclose(states[N - 1], want, rtol=1e-11, atol=1e-12)


def test_inter_readout_is_cross_chunk_linear_attention(oracle):
    """O_inter of chunk N equals sum_{j<N} decay * (Q' K'_j^T) V_j: a score-matrix form that never builds S."""
    chunks = _tiny_rollout_inputs()
    outs, _ = oracle.rollout(chunks)
    eps = oracle.L2_EPS
    for N, ch in enumerate(chunks):
        for p, (q, k, v, g) in enumerate(ch["passes"]):
            intra = oracle.fwd(q, k, v, None, None)
            want = np.zeros_like(intra)
            for j in range(N):
                decay = np.ones_like(chunks[0]["gate"])
                for i in range(j + 1, N):
                    decay = decay * chunks[i]["gate"]
                scores = np.einsum("blhd,bmhd->bhlm", l2n(q, eps), l2n(chunks[j]["k_clean"], eps))
                want += np.einsum("bhlm,bmhe->blhe", scores * decay[..., None, None], chunks[j]["v_clean"].astype(np.float64))
            want = intra + g[..., None].astype(np.float64) * want
            np.testing.assert_allclose(outs[N][p], want, rtol=1e-10, atol=1e-11)


def test_all_tokens_see_the_same_state(oracle):
    """Readout is permutation-equivariant over the chunk's tokens and commit is permutation-invariant:
    a token-sequential state update would fail both."""
    B, H, L, D = 1, 2, 17, 8
    q, k, v = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    g = rng.uniform(0, 1, (B, L, H)).astype(np.float32)
    S = rng.standard_normal((B, H, D, D))
    perm = rng.permutation(L)
    out = oracle.fwd(q, k, v, S, g)
    out_p = oracle.fwd(q[:, perm], k[:, perm], v[:, perm], S, g[:, perm])
    np.testing.assert_allclose(out_p, out[:, perm], rtol=1e-11, atol=1e-12)
    # reordering only the keys/values leaves every row unchanged
    np.testing.assert_allclose(oracle.fwd(q, k[:, perm], v[:, perm], S, g), out, rtol=1e-11, atol=1e-12)
    gate = np.full((B, H), 0.9)
    np.testing.assert_allclose(oracle.commit(k[:, perm], v[:, perm], gate, S), oracle.commit(k, v, gate, S), rtol=1e-11, atol=1e-12)
    # row subset: each row depends only on its own q and g
    rows = [3, 0, 16]
    np.testing.assert_array_equal(oracle.fwd(q, k, v, S, g, rows=rows), out[:, rows])


def test_state_is_read_only_in_readout(oracle):
    """Denoising passes never write S; only commit changes it."""
    B, H, L, D = 1, 2, 10, 8
    q, k, v = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    S = np.ascontiguousarray(rng.standard_normal((B, H, D, D)))
    snap = S.tobytes()
    first = oracle.fwd(q, k, v, S, None)
    for _ in range(3):
        assert np.array_equal(oracle.fwd(q, k, v, S, None), first)
    assert S.tobytes() == snap
    S2 = oracle.commit(k, v, np.full((B, H), 0.9), S)
    assert S.tobytes() == snap and not np.array_equal(S2, S)
    # rollout: every pass of a chunk used the pre-update state of that chunk
    chunks = _tiny_rollout_inputs(N=3, P=3)
    outs, states = oracle.rollout(chunks)
    Sprev = np.zeros_like(states[0])
    for n, ch in enumerate(chunks):
        for p, (q, k, v, g) in enumerate(ch["passes"]):
            assert np.array_equal(outs[n][p], oracle.fwd(q, k, v, Sprev, g))
        Sprev = states[n]


def test_f32_and_f64_oracles_agree_on_tiny_workload(oracle):
    """Bounds the fp32 oracle's own rounding on the fp32-throughout configuration."""
    import workloads as W
    w = W.WORKLOADS["tiny"]
    S64 = np.zeros((w.B, w.H, w.D, w.D))
    S32 = S64.astype(np.float32)
    for c in range(w.chunks):
        for p in range(w.passes):
            q, k, v, g = (W.as_f32_numpy(t) for t in W.pass_inputs(w, c, p))
            o64, o32 = oracle.fwd(q, k, v, S64, g), oracle.fwd(q, k, v, S32, g, precision="f32")
            assert np.abs(o64 - o32).max() <= 1e-5 * max(np.abs(o64).max(), 1e-30)
        k, v, gate = (W.as_f32_numpy(t) for t in W.clean_inputs(w, c))
        S64 = oracle.commit(k, v, gate, S64)
        S32 = oracle.commit(k, v, gate, S32, precision="f32")
        assert np.abs(S64 - S32).max() <= 1e-5 * np.abs(S64).max()


def test_stored_bf16_values_reach_the_oracle_exactly():
    import workloads as W
    w = W.WORKLOADS["ragged_small"]
    q, _, _, _ = W.pass_inputs(w, 0, 0)
    assert q.dtype == torch.bfloat16
    f = W.as_f32_numpy(q)
    assert torch.equal(torch.from_numpy(f).to(torch.bfloat16), q)
    q2, _, _, _ = W.pass_inputs(w, 0, 0)
    assert torch.equal(q, q2)
    q3, _, _, _ = W.pass_inputs(w, 0, 1)
    assert not torch.equal(q, q3)


# ---------------------------------------------------------------- delta-rule commit (Eq. (4) literally)

def test_delta_commit_matches_expanded_form(oracle):
    """alpha S + beta K'^T (V - K' S) = (alpha I - beta K'^T K') S + beta K'^T V, via einsum."""
    B, H, L, D = 2, 2, 19, 8
    k, v = rand(B, L, H, D), rand(B, L, H, D)
    S = rng.standard_normal((B, H, D, D))
    alpha, beta = rng.uniform(0.8, 1.0, (B, H)), rng.uniform(0.05, 0.3, (B, H))
    eps = oracle.L2_EPS
    kn = l2n(k, eps)
    G = np.einsum("blhd,blhe->bhde", kn, kn)
    M = np.einsum("blhd,blhe->bhde", kn, v.astype(np.float64))
    want = alpha[..., None, None] * S - beta[..., None, None] * np.einsum("bhdj,bhje->bhde", G, S) + beta[..., None, None] * M
    np.testing.assert_allclose(oracle.commit_delta(k, v, alpha, beta, S), want, rtol=1e-11, atol=1e-12)


def test_delta_commit_special_cases(oracle):
    B, H, L, D = 1, 2, 13, 8
    k, v = rand(B, L, H, D), rand(B, L, H, D)
    S = rng.standard_normal((B, H, D, D))
    alpha, beta = rng.uniform(0.8, 1.0, (B, H)), rng.uniform(0.05, 0.3, (B, H))
    # beta = 0: only the decay remains
    np.testing.assert_allclose(oracle.commit_delta(k, v, alpha, np.zeros((B, H)), S), alpha[..., None, None] * S, rtol=1e-14)
    # zero state: no correction term, so it is beta times the plain outer-product sum
    plain = oracle.commit(k, v, np.zeros((B, H)), np.zeros_like(S))
    np.testing.assert_allclose(oracle.commit_delta(k, v, alpha, beta, np.zeros_like(S)), beta[..., None, None] * plain, rtol=1e-12, atol=1e-14)
    # the input state is left untouched
    snap = S.copy()
    oracle.commit_delta(k, v, alpha, beta, S)
    assert np.array_equal(S, snap)


def test_delta_rule_overwrites_the_stored_value(oracle):
    """One token, alpha = beta = 1: whatever the old state held, querying the key now returns v
    exactly (k' S_new = k' S + (k' k'^T)(v - k' S) = v).  The plain rule would return k' S + v."""
    D = 8
    k, v = rand(1, 1, 1, D), rand(1, 1, 1, D)
    S = rng.standard_normal((1, 1, D, D))
    one = np.ones((1, 1))
    S_new = oracle.commit_delta(k, v, one, one, S, l2_eps=0.0)
    kn = l2n(k, 0.0)[0, 0, 0]
    np.testing.assert_allclose(kn @ S_new[0, 0], v[0, 0, 0].astype(np.float64), rtol=1e-6, atol=1e-6)
    S_plain = oracle.commit(k, v, one, S, l2_eps=0.0)
    assert np.abs(kn @ S_plain[0, 0] - v[0, 0, 0]).max() > 1e-2


def test_delta_commit_hand_example(oracle):
    ex = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))["commit_delta"]
    k = np.array(ex["k"])[None, :, None, :]
    v = np.array(ex["v"])[None, :, None, :]
    S_old = np.array(ex["S_old"])[None, None]
    S_new = oracle.commit_delta(k, v, np.array([[ex["alpha"]]]), np.array([[ex["beta"]]]), S_old, l2_eps=ex["l2_eps"])
    np.testing.assert_allclose(S_new[0, 0], np.array(ex["S_new"]), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- token-sequential gated delta rule

def _gdn_inputs(B, H, L, D, lo=0.7):
    k, v = rand(B, L, H, D), rand(B, L, H, D)
    S = rng.standard_normal((B, H, D, D))
    alpha, beta = rng.uniform(lo, 1.0, (B, L, H)), rng.uniform(0.1, 0.9, (B, L, H))
    return k, v, alpha, beta, S


def test_gdn_commit_hand_example(oracle):
    ex = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))["commit_gdn"]
    k = np.array(ex["k"])[None, :, None, :]
    v = np.array(ex["v"])[None, :, None, :]
    a = np.array(ex["alpha"])[None, :, None]
    b = np.array(ex["beta"])[None, :, None]
    S_new = oracle.commit_gdn(k, v, a, b, np.array(ex["S_old"])[None, None], l2_eps=ex["l2_eps"])
    np.testing.assert_allclose(S_new[0, 0], np.array(ex["S_new"]), rtol=0, atol=1e-12)


def test_gdn_commit_single_token_is_the_frame_level_rule(oracle):
    """With L = 1 'sequential over the tokens' and 'all tokens against the old state' coincide."""
    B, H, D = 2, 3, 8
    k, v, alpha, beta, S = _gdn_inputs(B, H, 1, D)
    want = oracle.commit_delta(k, v, alpha[:, 0], beta[:, 0], S)
    np.testing.assert_allclose(oracle.commit_gdn(k, v, alpha, beta, S), want, rtol=1e-13, atol=1e-14)


def test_gdn_commit_transition_matrix_product(oracle):
    """Each token is the affine map S -> (alpha I - beta k'^T k') S + beta k'^T v; compose them with
    explicit matrices (catches a correction that reads the wrong state or a gate on the wrong term)."""
    B, H, L, D = 1, 2, 23, 6
    k, v, alpha, beta, S = _gdn_inputs(B, H, L, D)
    kn = l2n(k, oracle.L2_EPS)
    got = oracle.commit_gdn(k, v, alpha, beta, S)
    for h in range(H):
        P, Q = np.eye(D), np.zeros((D, D))
        for j in range(L):
            kj = kn[0, j, h][None, :]
            Tj = alpha[0, j, h] * np.eye(D) - beta[0, j, h] * kj.T @ kj
            P, Q = Tj @ P, Tj @ Q + beta[0, j, h] * kj.T @ v[0, j, h][None, :].astype(np.float64)
        np.testing.assert_allclose(got[0, h], P @ S[0, h] + Q, rtol=1e-11, atol=1e-12)


def test_gdn_commit_orthonormal_keys_closed_form(oracle):
    """Mutually orthogonal keys do not see each other's writes, so every correction reads only the
    decayed initial state: S_L = g_L S_0 + sum_j (prod_{m>j} alpha_m) beta_j k_j^T (v_j - g_{j-1} k_j S_0)."""
    D = L = 8
    Qm, _ = np.linalg.qr(rng.standard_normal((D, D)))
    k = (Qm * rng.uniform(0.5, 3.0, (L, 1))).astype(np.float32)[None, :, None, :]     # rows: scaled orthonormal
    v = rand(1, L, 1, D)
    S = rng.standard_normal((1, 1, D, D))
    alpha, beta = rng.uniform(0.6, 1.0, (1, L, 1)), rng.uniform(0.1, 0.9, (1, L, 1))
    kn = l2n(k, 0.0)[0, :, 0]
    a, b = alpha[0, :, 0], beta[0, :, 0]
    g = np.concatenate([[1.0], np.cumprod(a)])            # g[j] = alpha_1 ... alpha_j
    want = g[L] * S[0, 0]
    for j in range(L):
        tail = np.prod(a[j + 1:])
        want = want + tail * b[j] * np.outer(kn[j], v[0, j, 0].astype(np.float64) - g[j] * (kn[j] @ S[0, 0]))
    np.testing.assert_allclose(oracle.commit_gdn(k, v, alpha, beta, S, l2_eps=0.0)[0, 0], want, rtol=1e-6, atol=1e-6)


def _gdn_chunkwise(kn, v, a, b, S, C):
    """Blocked evaluation of the same recurrence (an algebraically different route): inside a block of
    C tokens the pseudo-values w_i = beta_i (v_i - k_i S_{i-1}) solve a unit lower-triangular system,
    after which the block is one affine map of the state."""
    L, D = kn.shape
    for c0 in range(0, L, C):
        K, V, al, be = kn[c0:c0 + C], v[c0:c0 + C], a[c0:c0 + C], b[c0:c0 + C]
        n = K.shape[0]
        gam = np.concatenate([[1.0], np.cumprod(al)])     # gam[i] = alpha_1..alpha_i inside the block
        A = np.zeros((n, n))
        for i in range(n):
            for j in range(i):
                A[i, j] = be[i] * np.prod(al[j + 1:i]) * (K[i] @ K[j])
        rhs = be[:, None] * V - (be * gam[:n])[:, None] * (K @ S)
        Wp = np.linalg.solve(np.eye(n) + A, rhs)
        tail = np.array([np.prod(al[j + 1:]) for j in range(n)])
        S = gam[n] * S + (tail[:, None] * K).T @ Wp
    return S


@pytest.mark.parametrize("C", [1, 4, 7, 64])
def test_gdn_commit_matches_blocked_evaluation(oracle, C):
    B, H, L, D = 1, 2, 37, 8
    k, v, alpha, beta, S = _gdn_inputs(B, H, L, D)
    got = oracle.commit_gdn(k, v, alpha, beta, S)
    kn = l2n(k, oracle.L2_EPS)
    for h in range(H):
        want = _gdn_chunkwise(kn[0, :, h], v[0, :, h].astype(np.float64), alpha[0, :, h], beta[0, :, h], S[0, h], C)
        np.testing.assert_allclose(got[0, h], want, rtol=1e-10, atol=1e-11)


def test_gdn_commit_special_cases(oracle):
    B, H, L, D = 1, 2, 11, 8
    k, v, alpha, beta, S = _gdn_inputs(B, H, L, D)
    # beta = 0 everywhere: only the product of the per-token forget gates remains
    got = oracle.commit_gdn(k, v, alpha, np.zeros_like(beta), S)
    np.testing.assert_allclose(got, alpha.prod(axis=1)[..., None, None] * S, rtol=1e-13)
    # alpha = beta = 1, eps = 0: the last token's value is stored exactly under its key
    one = np.ones_like(alpha)
    got = oracle.commit_gdn(k, v, one, one, S, l2_eps=0.0)
    kn = l2n(k, 0.0)
    for h in range(H):
        np.testing.assert_allclose(kn[0, -1, h] @ got[0, h], v[0, -1, h].astype(np.float64), rtol=1e-6, atol=1e-6)
    # a gate of zero at the last token leaves only that token's write, a rank-one matrix whose
    # correction term still saw the state before it (the gate multiplies the old state only)
    a0 = alpha.copy()
    a0[:, -1] = 0.0
    got = oracle.commit_gdn(k, v, a0, beta, S)
    before = oracle.commit_gdn(k[:, :-1], v[:, :-1], alpha[:, :-1], beta[:, :-1], S)
    kn = l2n(k, oracle.L2_EPS)
    for h in range(H):
        kl = kn[0, -1, h]
        want = beta[0, -1, h] * np.outer(kl, v[0, -1, h].astype(np.float64) - kl @ before[0, h])
        np.testing.assert_allclose(got[0, h], want, rtol=1e-12, atol=1e-13)
    # the input state is left untouched; token order matters (it is not the frame-level rule)
    snap = S.copy()
    fwd_order = oracle.commit_gdn(k, v, alpha, beta, S)
    assert np.array_equal(S, snap)
    rev = oracle.commit_gdn(k[:, ::-1], v[:, ::-1], alpha[:, ::-1], beta[:, ::-1], S)
    assert np.abs(fwd_order - rev).max() > 1e-3


def test_gdn_commit_splits_into_consecutive_calls(oracle):
    """Committing tokens 1..L in one call equals committing 1..m and then m+1..L."""
    B, H, L, D = 2, 2, 21, 8
    k, v, alpha, beta, S = _gdn_inputs(B, H, L, D)
    whole = oracle.commit_gdn(k, v, alpha, beta, S)
    m = 8
    half = oracle.commit_gdn(k[:, :m], v[:, :m], alpha[:, :m], beta[:, :m], S)
    np.testing.assert_allclose(oracle.commit_gdn(k[:, m:], v[:, m:], alpha[:, m:], beta[:, m:], half), whole, rtol=1e-13, atol=1e-14)


# ---------------------------------------------------------------- feature maps of Eq. (3) and the inter branch's own query

def test_feature_map_hand_example_and_identity(oracle):
    # D = 2: W x = (1*1 + 2*1, 3*1 + 4*1) = (3, 7); a quarter turn maps (3, 7) to (-7, 3)
    x = np.array([1.0, 1.0], dtype=np.float32).reshape(1, 1, 1, 2)
    Wm = np.array([[1.0, 2.0], [3.0, 4.0]], dtype=np.float32).reshape(1, 2, 2)
    np.testing.assert_allclose(oracle.feature_map(x, Wm)[0, 0, 0], [3.0, 7.0], atol=1e-15)
    y = oracle.feature_map(x, Wm, np.array([[0.0]]), np.array([[1.0]]))
    np.testing.assert_allclose(y[0, 0, 0], [-7.0, 3.0], atol=1e-15)
    # identity weights, no rotation: the input comes back
    xr = rand(2, 5, 3, 8)
    eye = np.broadcast_to(np.eye(8, dtype=np.float32), (3, 8, 8)).copy()
    np.testing.assert_array_equal(oracle.feature_map(xr, eye), xr.astype(np.float64))


def test_feature_map_matches_einsum_and_complex_rotation(oracle):
    """W is indexed [head, out, in] (a transposed or head-shared weight fails); the rotation of a pair
    is multiplication of y0 + i y1 by exp(i theta)."""
    B, L, H, D = 2, 7, 3, 8
    x, Wm = rand(B, L, H, D), rand(H, D, D)
    th = rng.uniform(-3.0, 3.0, (L, D // 2))
    y = oracle.feature_map(x, Wm, np.cos(th), np.sin(th))
    lin = np.einsum("hed,blhd->blhe", Wm.astype(np.float64), x.astype(np.float64))
    z = (lin[..., 0::2] + 1j * lin[..., 1::2]) * np.exp(1j * th)[None, :, None, :]
    want = np.empty_like(lin)
    want[..., 0::2], want[..., 1::2] = z.real, z.imag
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-13)


def test_rope_depends_on_relative_position_only(oracle):
    """With theta_i(l) = l * w_i the inner product of two rotated rows is a function of the distance."""
    L, D = 12, 8
    w = 1.0 / (100.0 ** (np.arange(D // 2) / (D // 2)))
    th = np.arange(L)[:, None] * w[None, :]
    eye = np.eye(D, dtype=np.float32)[None]
    a, b = rand(D), rand(D)
    ya = oracle.feature_map(np.broadcast_to(a, (1, L, 1, D)).copy(), eye, np.cos(th), np.sin(th))[0, :, 0]
    yb = oracle.feature_map(np.broadcast_to(b, (1, L, 1, D)).copy(), eye, np.cos(th), np.sin(th))[0, :, 0]
    np.testing.assert_allclose(ya[3] @ yb[1], ya[9] @ yb[7], rtol=1e-12)
    np.testing.assert_allclose(ya[0] @ yb[5], ya[6] @ yb[11], rtol=1e-12)
    assert abs(ya[3] @ yb[1] - ya[3] @ yb[2]) > 1e-3
    np.testing.assert_allclose((ya * ya).sum(-1), (a.astype(np.float64) ** 2).sum(), rtol=1e-12)   # a rotation


def test_inter_branch_reads_its_own_query(oracle):
    B, L, H, D = 1, 9, 2, 8
    q, k, v, ql = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    S = rng.standard_normal((B, H, D, D))
    g = rng.uniform(0.2, 0.8, (B, L, H)).astype(np.float32)
    eps = oracle.L2_EPS
    # given q itself, nothing changes; without a state the argument is not read
    np.testing.assert_array_equal(oracle.fwd(q, k, v, S, g, q_lin=q), oracle.fwd(q, k, v, S, g))
    np.testing.assert_array_equal(oracle.fwd(q, k, v, None, None, q_lin=ql), oracle.fwd(q, k, v, None, None))
    # out = intra(q) + g * L2Norm(q_lin) S: the softmax branch never sees q_lin, the linear one never sees q
    intra = oracle.fwd(q, k, v, None, None)
    inter = np.einsum("blhd,bhde->blhe", l2n(ql, eps), S) * g[..., None].astype(np.float64)
    np.testing.assert_allclose(oracle.fwd(q, k, v, S, g, q_lin=ql), intra + inter, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.fwd(q, k, v, S, g, q_lin=3.0 * ql), intra + inter, rtol=1e-5, atol=1e-5)   # up to eps and the fp32 rounding of 3 q


# ---------------------------------------------------------------- headwise mix gate, Eq. (6)

def test_gate_proj_pins(oracle):
    from scipy.special import expit
    B, L, dm, H = 2, 11, 24, 3
    x, Wg = rand(B, L, dm), rand(H, dm, scale=0.3)
    G = oracle.gate_proj(x, Wg)
    np.testing.assert_allclose(G, expit(np.einsum("blj,hj->blh", x.astype(np.float64), Wg.astype(np.float64))), rtol=1e-13)
    assert G.shape == (B, L, H) and np.all((G > 0) & (G < 1))
    # zero weights: every gate is one half; a head's gate depends on that head's weight row only
    np.testing.assert_array_equal(oracle.gate_proj(x, np.zeros_like(Wg)), np.full((B, L, H), 0.5))
    W2 = Wg.copy()
    W2[1] = 0.0
    G2 = oracle.gate_proj(x, W2)
    np.testing.assert_array_equal(G2[..., 0], G[..., 0])
    np.testing.assert_array_equal(G2[..., 1], np.full((B, L), 0.5))
    # hand example: x = (1, 2), w = (ln 3, 0) -> sigmoid(ln 3) = 3/4; w = (0, -ln(3)/2) -> sigmoid(-ln 3) = 1/4
    xh = np.array([[[1.0, 2.0]]], dtype=np.float32)
    wh = np.array([[math.log(3.0), 0.0], [0.0, -math.log(3.0) / 2.0]], dtype=np.float32)
    np.testing.assert_allclose(oracle.gate_proj(xh, wh)[0, 0], [0.75, 0.25], rtol=1e-7)


def test_gate_granularities(oracle):
    """Eq. (6)'s gate is one value per (token, head).  The two other granularities of the paper's gate
    ablation: one value per token (the same [B, L, H] array with equal entries per head) and one value per
    output feature ([B, L, H, D], multiplying the linear branch element by element)."""
    B, L, H, D = 1, 7, 3, 8
    q, k, v = rand(B, L, H, D), rand(B, L, H, D), rand(B, L, H, D)
    S = rng.standard_normal((B, H, D, D))
    g = rng.uniform(0.2, 0.8, (B, L, H)).astype(np.float32)
    base = oracle.fwd(q, k, v, S, g)
    # an element-wise gate that is constant over the features is the headwise gate
    ge = np.repeat(g[..., None], D, axis=-1)
    np.testing.assert_array_equal(oracle.fwd(q, k, v, S, ge), base)
    # in general: out = intra + g (.) inter, element by element
    ge = rng.uniform(0.0, 1.0, (B, L, H, D)).astype(np.float32)
    intra = oracle.fwd(q, k, v, None, None)
    inter = oracle.fwd(q, k, v, S, None) - intra
    np.testing.assert_allclose(oracle.fwd(q, k, v, S, ge), intra + ge.astype(np.float64) * inter, rtol=1e-12, atol=1e-13)
    # a per-token gate is the headwise array with the token's value repeated for every head
    gt = rng.uniform(0.2, 0.8, (B, L, 1)).astype(np.float32)
    got = oracle.fwd(q, k, v, S, np.repeat(gt, H, axis=2))
    np.testing.assert_allclose(got, intra + gt[..., None].astype(np.float64) * inter, rtol=1e-12, atol=1e-13)
    # ... and the [B, L] scalar gate is that array without the repetition
    np.testing.assert_array_equal(oracle.fwd(q, k, v, S, gt[..., 0]), got)
    np.testing.assert_array_equal(oracle.fwd(q, k, v, S, gt[..., 0], rows=[5, 0]), got[:, [5, 0]])
    with pytest.raises(ValueError):
        oracle.fwd(q, k, v, S, np.ones((B, L + 1), np.float32))
    # its projection has a single weight row (d_model parameters per layer)
    from scipy.special import expit
    x, w1 = rand(B, L, H * D), rand(1, H * D, scale=0.3)
    np.testing.assert_allclose(oracle.gate_proj(x, w1)[..., 0], expit(x.astype(np.float64) @ w1[0].astype(np.float64)), rtol=1e-13)


def test_pins_hold_under_address_and_undefined_behaviour_sanitizers():
    """The whole pin suite once more in a child process whose oracle is built with -fsanitize=address,undefined
    (every finding aborts): an out-of-bounds index or a signed overflow in the oracle's loops fails here even
    where it happens not to change a pinned value."""
    import os
    import subprocess
    import sys
    from oracle import arl2_oracle as O
    if os.environ.get("ARL2_ORACLE_SANITIZED") == "1":
        return                                      # this is the child
    O.build_sanitized()
    env = O.sanitizer_env(os.environ)
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                         env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900,
                         cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    tail = "\n".join(res.stdout.splitlines()[-25:])
    assert res.returncode == 0, tail
    assert " passed" in tail and "failed" not in tail, tail
