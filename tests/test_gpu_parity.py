"""GPU parity: the HIP library, called through its C ABI (ctypes binding), against the CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import workloads as W
from helpers import (TOL_BF16_OUT, TOL_F32, TOL_STATE, rel_err, rel_err_per_head, sample_rows, to_np)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2605_16579_amd as A
    A.load_library()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return A


def dev(t):
    return t.cuda() if t is not None else None


def gpu_fwd(A, q, k, v, S, g):
    out = torch.empty_like(q, device="cuda")
    A.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S), dev(g), out)
    torch.cuda.synchronize()
    return out


def gpu_commit(A, k, v, gate, S_dev):
    B, L, H, D = k.shape
    ws = A.alloc_workspace(B, H, L, D, k.dtype)
    A.arl2_state_commit(dev(k), dev(v), dev(gate), S_dev, ws)
    torch.cuda.synchronize()


def run_rollout_parity(A, oracle, w, tol_out, tol_state, precision="f64", seed=0):
    """Alg. 1 call pattern on workload w: every pass output and every committed state is compared."""
    S_ref = np.zeros((w.B, w.H, w.D, w.D))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    for j in range(w.prefill):
        k, v, gate = W.prefill_inputs(w, j, seed)
        S_ref = oracle.commit(to_np(k), to_np(v), to_np(gate), S_ref)
        gpu_commit(A, k, v, gate, S_dev)
    worst_out = worst_state = 0.0
    for c in range(w.chunks):
        S_before = S_dev.clone()
        for p in range(w.passes):
            q, k, v, g = W.pass_inputs(w, c, p, seed)
            # the oracle reads its own fp64 state chain: nothing the GPU produced ever reaches it
            ref = oracle.fwd(to_np(q), to_np(k), to_np(v), S_ref, to_np(g))
            got = gpu_fwd(A, q, k, v, S_dev, g)
            e = rel_err(to_np(got), ref)
            worst_out = max(worst_out, e)
            assert e <= tol_out, f"{w.name} chunk {c} pass {p}: out error {e:.3e}"
            assert torch.equal(S_dev, S_before), "a readout pass wrote the state"
        k, v, gate = W.clean_inputs(w, c, seed)
        S_ref = oracle.commit(to_np(k), to_np(v), to_np(gate), S_ref)   # fp64 chain, never re-synced to the GPU
        gpu_commit(A, k, v, gate, S_dev)
        assert not torch.equal(S_dev, S_before), "commit left the state unchanged"
        e = rel_err_per_head(to_np(S_dev), S_ref)
        worst_state = max(worst_state, e)
        assert e <= tol_state, f"{w.name} chunk {c}: state error {e:.3e}"
    print(f"[{w.name}] worst out err {worst_out:.3e}, worst state err {worst_state:.3e}", flush=True)


def test_tiny_fp32_rollout(lib, oracle):
    run_rollout_parity(lib, oracle, W.WORKLOADS["tiny"], TOL_F32, TOL_F32)


def test_ragged_small_bf16_rollout(lib, oracle):
    run_rollout_parity(lib, oracle, W.WORKLOADS["ragged_small"], TOL_BF16_OUT, TOL_STATE)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_other_head_dims(lib, oracle, D, io):
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"hd{D}{io}", D=D, io_dtype=io, L=200, chunks=2)
    tol_o, tol_s = (TOL_BF16_OUT, TOL_STATE) if io == "bf16" else (TOL_F32, TOL_F32)
    run_rollout_parity(lib, oracle, w, tol_o, tol_s)


@pytest.mark.parametrize("L", [1, 7, 63, 64, 65, 127, 128, 129, 191, 256, 333])
def test_branches_separately_and_ragged_lengths(lib, oracle, L):
    """Each branch alone (the linear branch is ~100x larger with these inputs and would hide an
    intra-branch error in a combined max-norm check), for lengths around the tile edges."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"len{L}", L=L, B=1, H=2)
    q, k, v, g = W.pass_inputs(w, 0, 0)
    kc, vc, gate = W.clean_inputs(w, 0)
    S = torch.from_numpy(oracle.commit(to_np(kc), to_np(vc), to_np(gate), np.zeros((w.B, w.H, w.D, w.D)))).float()
    # intra alone: no state
    e = rel_err(to_np(gpu_fwd(lib, q, k, v, None, None)), oracle.fwd(to_np(q), to_np(k), to_np(v)))
    assert e <= TOL_BF16_OUT, f"intra L={L}: {e:.3e}"
    # inter alone: v = 0 makes the softmax branch vanish
    vz = torch.zeros_like(v)
    ref = oracle.fwd(to_np(q), to_np(k), to_np(vz), to_np(S).astype(np.float64), to_np(g))
    e = rel_err(to_np(gpu_fwd(lib, q, k, vz, S, g)), ref)
    assert e <= TOL_BF16_OUT, f"inter L={L}: {e:.3e}"
    # gate of one (g == NULL) and gate of zero
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), None)
    assert rel_err(to_np(gpu_fwd(lib, q, k, v, S, None)), ref) <= TOL_BF16_OUT
    g0 = torch.zeros_like(g)
    assert torch.equal(gpu_fwd(lib, q, k, v, S, g0), gpu_fwd(lib, q, k, v, None, None))
    # bf16 gate tensor
    gb = g.to(torch.bfloat16)
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), to_np(gb))
    assert rel_err(to_np(gpu_fwd(lib, q, k, v, S, gb)), ref) <= TOL_BF16_OUT
    # commit at this length
    S_dev = S.cuda()
    gpu_commit(lib, k, v, gate, S_dev)
    ref = oracle.commit(to_np(k), to_np(v), to_np(gate), to_np(S).astype(np.float64))
    assert rel_err_per_head(to_np(S_dev), ref) <= TOL_STATE


@pytest.mark.parametrize("Lq,Lkv", [(100, 300), (128, 64), (1, 500), (200, 1)])
@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_softmax_over_longer_kv(lib, oracle, Lq, Lkv, io):
    """S == NULL with Lkv != Lq: softmax over a KV cache in which every cached token is visible."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name="kvcache", io_dtype=io)
    q = W.normal(1, w, (w.B, Lq, w.H, w.D), 1)
    k = W.normal(1, w, (w.B, Lkv, w.H, w.D), 2)
    v = W.normal(1, w, (w.B, Lkv, w.H, w.D), 3)
    got = gpu_fwd(lib, q, k, v, None, None)
    e = rel_err(to_np(got), oracle.fwd(to_np(q), to_np(k), to_np(v)))
    assert e <= (TOL_BF16_OUT if io == "bf16" else TOL_F32), f"{e:.3e}"


def test_peaked_softmax_and_large_logits(lib, oracle):
    """Rows whose maximum moves late in the key sequence and logits of a few hundred: the running-max
    rescale must stay exact and finite."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name="peaked", B=1, H=2, L=300)
    q, k, v, _ = W.pass_inputs(w, 0, 0)
    k = k.float()
    k[:, 250:260] *= 8.0          # large keys near the end
    q = (q.float() * 3.0).to(torch.bfloat16)
    k = k.to(torch.bfloat16)
    got = gpu_fwd(lib, q, k, v, None, None)
    e = rel_err(to_np(got), oracle.fwd(to_np(q), to_np(k), to_np(v)))
    assert e <= TOL_BF16_OUT, f"{e:.3e}"


def test_commit_is_deterministic_and_fwd_repeatable(lib):
    w = W.WORKLOADS["ragged_small"]
    q, k, v, g = W.pass_inputs(w, 0, 0)
    kc, vc, gate = W.clean_inputs(w, 0)
    S0 = torch.randn((w.B, w.H, w.D, w.D), generator=torch.Generator().manual_seed(3))
    results = []
    for _ in range(3):
        S_dev = S0.cuda()
        gpu_commit(lib, kc, vc, gate, S_dev)
        results.append(S_dev.clone())
    assert torch.equal(results[0], results[1]) and torch.equal(results[0], results[2])
    o1 = gpu_fwd(lib, q, k, v, S0, g)
    o2 = gpu_fwd(lib, q, k, v, S0, g)
    assert torch.equal(o1, o2)


def test_wan_layer_full_size(lib, oracle):
    """The headline shape (12 heads x 128, 4680 tokens): state pre-filled by 8 oracle commits, four
    readout passes checked on sampled rows (each row depends only on its own q and all of k, v, S),
    then one commit checked in full."""
    w = W.WORKLOADS["wan_layer"]
    S_ref = np.zeros((w.B, w.H, w.D, w.D))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    for j in range(w.prefill):
        k, v, gate = W.prefill_inputs(w, j)
        S_ref = oracle.commit(to_np(k), to_np(v), to_np(gate), S_ref)
        gpu_commit(lib, k, v, gate, S_dev)
    e = rel_err_per_head(to_np(S_dev), S_ref)
    print(f"[wan_layer] state after 8 prefill commits: {e:.3e}", flush=True)
    assert e <= TOL_STATE
    S_before = S_dev.clone()
    for p in range(w.passes):
        q, k, v, g = W.pass_inputs(w, 0, p)
        rows = sample_rows(w.L, 256, seed=p)
        got = to_np(gpu_fwd(lib, q, k, v, S_dev, g))[:, rows]
        e = rel_err(got, oracle.fwd(to_np(q), to_np(k), to_np(v), S_ref, to_np(g), rows=rows))
        # intra branch alone on the same rows
        got_i = to_np(gpu_fwd(lib, q, k, v, None, None))[:, rows]
        ei = rel_err(got_i, oracle.fwd(to_np(q), to_np(k), to_np(v), rows=rows))
        print(f"[wan_layer] pass {p}: out {e:.3e}  intra-only {ei:.3e}  ({len(rows)} rows/head)", flush=True)
        assert e <= TOL_BF16_OUT and ei <= TOL_BF16_OUT
        assert torch.equal(S_dev, S_before)
    k, v, gate = W.clean_inputs(w, 0)
    S_ref = oracle.commit(to_np(k), to_np(v), to_np(gate), S_ref)
    gpu_commit(lib, k, v, gate, S_dev)
    e = rel_err_per_head(to_np(S_dev), S_ref)
    print(f"[wan_layer] state after the chunk's commit: {e:.3e}", flush=True)
    assert e <= TOL_STATE


def test_wan_batched_full_size(lib, oracle):
    """8 streams at the headline shape: sampled rows of one pass, full state after one commit."""
    w = W.WORKLOADS["wan_batched"]
    kc, vc, gate = W.prefill_inputs(w, 0)
    S_ref = oracle.commit(to_np(kc), to_np(vc), to_np(gate), np.zeros((w.B, w.H, w.D, w.D)))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    gpu_commit(lib, kc, vc, gate, S_dev)
    e = rel_err_per_head(to_np(S_dev), S_ref)
    print(f"[wan_batched] state after one commit: {e:.3e}", flush=True)
    assert e <= TOL_STATE
    q, k, v, g = W.pass_inputs(w, 0, 0)
    rows = sample_rows(w.L, 24, seed=7)
    got = to_np(gpu_fwd(lib, q, k, v, S_dev, g))[:, rows]
    e = rel_err(got, oracle.fwd(to_np(q), to_np(k), to_np(v), S_ref, to_np(g), rows=rows))
    print(f"[wan_batched] out: {e:.3e}", flush=True)
    assert e <= TOL_BF16_OUT


def test_wan_rollout_64_chained_commits(lib, oracle):
    """State drift over 64 chained commits at the headline shape against the fp64 oracle chain,
    with readout rows checked on the first, a middle and the last chunk."""
    w = W.WORKLOADS["wan_rollout"]
    S_ref = np.zeros((w.B, w.H, w.D, w.D))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    worst = 0.0
    for c in range(w.chunks):
        if c in (0, 31, 63):
            q, k, v, g = W.pass_inputs(w, c, 0)
            rows = sample_rows(w.L, 32, seed=c)
            got = to_np(gpu_fwd(lib, q, k, v, S_dev, g))[:, rows]
            e = rel_err(got, oracle.fwd(to_np(q), to_np(k), to_np(v), S_ref, to_np(g), rows=rows))
            assert e <= TOL_BF16_OUT, f"chunk {c}: out {e:.3e}"
            # the same rows with the state branch off: the softmax term alone
            got = to_np(gpu_fwd(lib, q, k, v, None, None))[:, rows]
            e = rel_err(got, oracle.fwd(to_np(q), to_np(k), to_np(v), rows=rows))
            assert e <= TOL_BF16_OUT, f"chunk {c}: softmax-only out {e:.3e}"
        k, v, gate = W.clean_inputs(w, c)
        S_ref = oracle.commit(to_np(k), to_np(v), to_np(gate), S_ref)
        gpu_commit(lib, k, v, gate, S_dev)
        e = rel_err_per_head(to_np(S_dev), S_ref)
        worst = max(worst, e)
        if c % 8 == 7:
            print(f"[wan_rollout] chunk {c}: state err {e:.3e}", flush=True)
        assert e <= TOL_STATE, f"chunk {c}: state {e:.3e}"
    print(f"[wan_rollout] worst state err over 64 chained commits {worst:.3e}", flush=True)


def test_softmax_over_full_kv_cache_shape(lib, oracle):
    """Layers that keep softmax over a KV cache: one 4680-token chunk of queries against the cache of a
    21-latent-frame horizon (32760 keys), no state.  Sampled rows against the oracle."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["wan_layer"], name="kv_cache_full")
    Lq, Lkv = 4680, 32760
    q = W.normal(5, w, (1, Lq, w.H, w.D), 1)
    k = W.normal(5, w, (1, Lkv, w.H, w.D), 2)
    v = W.normal(5, w, (1, Lkv, w.H, w.D), 3)
    rows = sample_rows(Lq, 16, seed=11, block=256)
    got = to_np(gpu_fwd(lib, q, k, v, None, None))[:, rows]
    e = rel_err(got, oracle.fwd(to_np(q), to_np(k), to_np(v), rows=rows))
    print(f"[kv_cache_full] Lq={Lq} Lkv={Lkv}: out err {e:.3e} on {len(rows)} rows/head", flush=True)
    assert e <= TOL_BF16_OUT


def test_rollout_step_latency_is_flat(lib):
    """Per-chunk cost does not grow with the number of chunks already generated: the state has a
    fixed size.  64 chunk steps (4 readout passes + 1 commit) at the headline shape, timed with
    events on the launch stream; the same inputs are reused so that only the state evolves."""
    w = W.WORKLOADS["wan_rollout"]
    passes = [tuple(dev(t) for t in W.pass_inputs(w, 0, p)) for p in range(w.passes)]
    kc, vc, gate = (dev(t) for t in W.clean_inputs(w, 0))
    out = torch.empty_like(passes[0][0])
    S = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    ws = lib.alloc_workspace(w.B, w.H, w.L, w.D, kc.dtype)

    def step():
        for (q, k, v, g) in passes:
            lib.arl2_hybrid_attn_fwd(q, k, v, S, g, out)
        lib.arl2_state_commit(kc, vc, gate, S, ws)

    for _ in range(30):          # clocks and caches settle
        step()

    def series():
        S.zero_()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(w.chunks + 1)]
        ev[0].record()
        for c in range(w.chunks):
            step()
            ev[c + 1].record()
        torch.cuda.synchronize()
        ms = np.array([ev[c].elapsed_time(ev[c + 1]) for c in range(w.chunks)])
        med = float(np.median(ms))
        slope = float(np.polyfit(np.arange(w.chunks), ms, 1)[0])
        print(f"[wan_rollout] step latency over {w.chunks} chunks: median {med:.4f} ms, max/median {ms.max() / med:.3f}, "
              f"min/median {ms.min() / med:.3f}, least-squares drift over the rollout {slope * w.chunks / med * 100:+.2f} % of median",
              flush=True)
        print("[wan_rollout] ms per chunk:", " ".join(f"{x:.3f}" for x in ms), flush=True)
        return slope * w.chunks < 0.03 * med, np.percentile(ms, 90) < 1.05 * med

    # a cost that grew with the history (a cache of past chunks) would show up as hundreds of per cent; recorded
    # series on this hardware: drift between -3.6 % and +0.5 % of the median over the rollout, 90th percentile
    # within 1 % of the median, single slow chunks (the first one, clock changes) up to 5 % above it.  The margins
    # are a few per cent, and the clock of a shared machine can move by that much within one series: a series that
    # misses them is measured once more, and both are printed (growth with the history fails every series).
    flat, tight = series()
    if not (flat and tight):
        flat, tight = series()
    assert flat, "per-chunk latency grows with the chunk index"
    assert tight, "the 90th percentile of the per-chunk latency is more than 5 % above the median"
    assert torch.isfinite(S).all()


@pytest.mark.parametrize("D,L", [(128, 328), (64, 200), (128, 64), (128, 1)])
def test_delta_rule_commit_small(lib, oracle, D, L):
    """Eq. (4) with the delta-correction term, element by element, three chained updates."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"delta{D}", D=D, L=L)
    S_ref = np.zeros((w.B, w.H, w.D, w.D))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    ws = lib.alloc_workspace(w.B, w.H, w.L, w.D, torch.bfloat16)
    for c in range(3):
        k, v, alpha = W.clean_inputs(w, c)
        beta = W.uniform(0, w, (w.B, w.H), 0.2 * D / max(L, D), 1.0 * D / max(L, D), c, 0, 77)
        S_ref = oracle.commit_delta(to_np(k), to_np(v), to_np(alpha), to_np(beta), S_ref)
        lib.arl2_state_commit_delta(dev(k), dev(v), dev(alpha), dev(beta), S_dev, ws)
        torch.cuda.synchronize()
        e = rel_err_per_head(to_np(S_dev), S_ref)
        assert e <= TOL_STATE, f"D={D} L={L} update {c}: {e:.3e}"


def test_delta_rule_commit_full_size(lib, oracle):
    """Headline shape: state pre-filled by plain commits, then four chained delta-rule updates with
    beta in the range where the frame-level rule is a contraction (below 2 D / L)."""
    w = W.WORKLOADS["wan_layer"]
    S_ref = np.zeros((w.B, w.H, w.D, w.D))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    ws = lib.alloc_workspace(w.B, w.H, w.L, w.D, torch.bfloat16)
    for j in range(2):
        k, v, gate = W.prefill_inputs(w, j)
        S_ref = oracle.commit(to_np(k), to_np(v), to_np(gate), S_ref)
        lib.arl2_state_commit(dev(k), dev(v), dev(gate), S_dev, ws)
    worst = 0.0
    for c in range(4):
        k, v, alpha = W.clean_inputs(w, c)
        beta = W.uniform(0, w, (w.B, w.H), 0.2 * w.D / w.L, 1.0 * w.D / w.L, c, 0, 77)
        S_ref = oracle.commit_delta(to_np(k), to_np(v), to_np(alpha), to_np(beta), S_ref)
        lib.arl2_state_commit_delta(dev(k), dev(v), dev(alpha), dev(beta), S_dev, ws)
        torch.cuda.synchronize()
        e = rel_err_per_head(to_np(S_dev), S_ref)
        worst = max(worst, e)
        assert e <= TOL_STATE, f"update {c}: {e:.3e}"
    print(f"[wan_layer] delta-rule commit, worst state err over 4 chained updates {worst:.3e}", flush=True)
    # deterministic
    S2 = S_dev.clone()
    k, v, alpha = W.clean_inputs(w, 9)
    beta = W.uniform(0, w, (w.B, w.H), 0.005, 0.02, 9, 0, 77)
    lib.arl2_state_commit_delta(dev(k), dev(v), dev(alpha), dev(beta), S_dev, ws)
    lib.arl2_state_commit_delta(dev(k), dev(v), dev(alpha), dev(beta), S2, ws)
    torch.cuda.synchronize()
    assert torch.equal(S_dev, S2)


# ---------------------------------------------------------------- token-sequential gated delta rule

def _gdn_ws(lib, w):
    return torch.empty(lib.arl2_gdn_workspace_bytes(w.B, w.H, w.L, w.D), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("D,L", [(128, 328), (64, 200), (128, 64), (128, 65), (64, 63), (128, 1)])
def test_gdn_commit_small(lib, oracle, D, L):
    """Eq. (4) token by token with per-token gates, element by element, three chained updates;
    sizes below, at and above one 64-token block, both head dimensions."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"gdn{D}", D=D, L=L)
    S_ref = np.zeros((w.B, w.H, w.D, w.D))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    ws = _gdn_ws(lib, w)
    for c in range(3):
        k, v, _ = W.clean_inputs(w, c)
        alpha, beta = W.token_gates(w, c)
        S_ref = oracle.commit_gdn(to_np(k), to_np(v), to_np(alpha), to_np(beta), S_ref)
        lib.arl2_state_commit_gdn(dev(k), dev(v), dev(alpha), dev(beta), S_dev, ws)
        torch.cuda.synchronize()
        e = rel_err_per_head(to_np(S_dev), S_ref)
        assert e <= TOL_STATE, f"D={D} L={L} update {c}: {e:.3e}"


@pytest.mark.parametrize("D,L", [(128, 1700), (128, 3141), (64, 1700)])
def test_gdn_commit_long_chunks(lib, oracle, D, L):
    """Chunks long enough that the blocks of a head are walked as several runs at the same time (six and
    eight runs here, of lengths that differ by one), whose composite maps are then applied in order."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"gdn_long{D}", B=1, H=2, D=D, L=L)
    S0 = W.normal(5, w, (w.B, w.H, w.D, w.D), 0, 0, 92, io_dtype="f32")
    S_ref = to_np(S0).astype(np.float64)
    S_dev = dev(S0).clone()
    ws = _gdn_ws(lib, w)
    for c in range(2):
        k, v, _ = W.clean_inputs(w, c)
        alpha, beta = W.token_gates(w, c)
        S_ref = oracle.commit_gdn(to_np(k), to_np(v), to_np(alpha), to_np(beta), S_ref)
        lib.arl2_state_commit_gdn(dev(k), dev(v), dev(alpha), dev(beta), S_dev, ws)
        torch.cuda.synchronize()
        e = rel_err_per_head(to_np(S_dev), S_ref)
        assert e <= TOL_STATE, f"D={D} L={L} update {c}: {e:.3e}"


def test_gdn_commit_gate_edge_values(lib, oracle):
    """Gates of exactly 0 and 1 and learning rates of exactly 0 and 1 inside and across blocks."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name="gdn_edges", L=200)
    k, v, _ = W.clean_inputs(w, 0)
    alpha, beta = W.token_gates(w, 0)
    alpha[:, 5] = 0.0
    alpha[:, 63] = 0.0
    alpha[:, 64] = 1.0
    alpha[0, 130:140] = 0.0
    beta[:, 7] = 0.0
    beta[:, 100] = 1.0
    beta[1, 64:128] = 0.0
    S0 = W.normal(3, w, (w.B, w.H, w.D, w.D), 0, 0, 91, io_dtype="f32")
    S_ref = oracle.commit_gdn(to_np(k), to_np(v), to_np(alpha), to_np(beta), to_np(S0).astype(np.float64))
    S_dev = dev(S0).clone()
    lib.arl2_state_commit_gdn(dev(k), dev(v), dev(alpha), dev(beta), S_dev, _gdn_ws(lib, w))
    torch.cuda.synchronize()
    assert torch.isfinite(S_dev).all()
    e = rel_err_per_head(to_np(S_dev), S_ref)
    assert e <= TOL_STATE, f"{e:.3e}"


def test_gdn_commit_full_size(lib, oracle):
    """Headline shape: four chained token-sequential updates of a pre-filled state."""
    w = W.WORKLOADS["wan_layer"]
    S_ref = np.zeros((w.B, w.H, w.D, w.D))
    S_dev = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device="cuda")
    ws_plain = lib.alloc_workspace(w.B, w.H, w.L, w.D, torch.bfloat16)
    ws = _gdn_ws(lib, w)
    for j in range(2):
        k, v, gate = W.prefill_inputs(w, j)
        S_ref = oracle.commit(to_np(k), to_np(v), to_np(gate), S_ref)
        lib.arl2_state_commit(dev(k), dev(v), dev(gate), S_dev, ws_plain)
    worst = 0.0
    for c in range(4):
        k, v, _ = W.clean_inputs(w, c)
        alpha, beta = W.token_gates(w, c)
        S_ref = oracle.commit_gdn(to_np(k), to_np(v), to_np(alpha), to_np(beta), S_ref)
        lib.arl2_state_commit_gdn(dev(k), dev(v), dev(alpha), dev(beta), S_dev, ws)
        torch.cuda.synchronize()
        e = rel_err_per_head(to_np(S_dev), S_ref)
        worst = max(worst, e)
        assert e <= TOL_STATE, f"update {c}: {e:.3e}"
    print(f"[wan_layer] token-sequential commit, worst state err over 4 chained updates {worst:.3e}", flush=True)
    # deterministic
    S2 = S_dev.clone()
    lib.arl2_state_commit_gdn(dev(k), dev(v), dev(alpha), dev(beta), S_dev, ws)
    lib.arl2_state_commit_gdn(dev(k), dev(v), dev(alpha), dev(beta), S2, ws)
    torch.cuda.synchronize()
    assert torch.equal(S_dev, S2)


def test_gdn_commit_batched_full_size(lib, oracle):
    """8 streams at the headline shape (96 heads: more scan workgroups than one round of CUs)."""
    w = W.WORKLOADS["wan_batched"]
    k, v, _ = W.clean_inputs(w, 0)
    alpha, beta = W.token_gates(w, 0)
    S0 = W.normal(17, w, (w.B, w.H, w.D, w.D), 0, 0, 99, io_dtype="f32") * 0.2
    S_dev = dev(S0).clone()
    lib.arl2_state_commit_gdn(dev(k), dev(v), dev(alpha), dev(beta), S_dev, _gdn_ws(lib, w))
    torch.cuda.synchronize()
    S_ref = oracle.commit_gdn(to_np(k), to_np(v), to_np(alpha), to_np(beta), to_np(S0).astype(np.float64))
    e = rel_err_per_head(to_np(S_dev), S_ref)
    print(f"[wan_batched] token-sequential commit: state err {e:.3e}", flush=True)
    assert e <= TOL_STATE


# ---------------------------------------------------------------- feature maps of Eq. (3), the linear branch's own query

def _bf16_round(x64):
    """What storing an fp64 oracle intermediate in bf16 gives (round to nearest even, once)."""
    return torch.from_numpy(np.ascontiguousarray(x64, dtype=np.float32)).to(torch.bfloat16)


@pytest.mark.parametrize("D,L,B,H", [(128, 328, 2, 3), (64, 200, 2, 3), (128, 1, 1, 2), (128, 129, 1, 1)])
def test_feature_map_small(lib, oracle, D, L, B, H):
    """y = RoPE(W[h] x), element by element; with and without the rotation; ragged tails of the 128-token tile."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"fmap{D}", D=D, L=L, B=B, H=H)
    x = W.normal(11, w, (w.B, w.L, w.H, w.D), 0, 0, 93)
    Wq, Wk, Wv = W.feature_weights(w)
    cs, sn = W.rope_tables(w)
    y = torch.empty_like(x, device="cuda")
    for Wm, rope in ((Wq, True), (Wv, False), (Wk, True)):
        lib.arl2_feature_map(dev(x), dev(Wm), dev(cs) if rope else None, dev(sn) if rope else None, y)
        torch.cuda.synchronize()
        ref = oracle.feature_map(to_np(x), to_np(Wm), to_np(cs) if rope else None, to_np(sn) if rope else None)
        e = rel_err(to_np(y), ref)
        assert e <= TOL_BF16_OUT, f"D={D} L={L} rope={rope}: {e:.3e}"
        # one bf16 rounding of an fp32-accurate result: a few ulp at most, element by element
        assert np.all(np.abs(to_np(y) - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-6 * np.abs(ref).max())


def test_identity_feature_map_is_exact_without_rotation(lib):
    w = W.WORKLOADS["ragged_small"]
    x = W.normal(12, w, (w.B, w.L, w.H, w.D), 0, 0, 94)
    eye = torch.eye(w.D, dtype=torch.bfloat16).repeat(w.H, 1, 1).contiguous()
    y = torch.empty_like(x, device="cuda")
    lib.arl2_feature_map(dev(x), dev(eye), None, None, y)
    torch.cuda.synchronize()
    assert torch.equal(y.cpu(), x)


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_readout_with_own_linear_query(lib, oracle, io):
    """arl2_hybrid_attn_fwd_ex: the softmax branch sees q, the linear branch q_lin."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name="fwd_ex_" + io, io_dtype=io, L=200 if io == "f32" else 328)
    q, k, v, g = W.pass_inputs(w, 0, 0)
    q_lin = W.normal(13, w, (w.B, w.L, w.H, w.D), 0, 0, 95)
    S = W.normal(14, w, (w.B, w.H, w.D, w.D), 0, 0, 96, io_dtype="f32") * 0.2
    out = torch.empty_like(q, device="cuda")
    lib.arl2_hybrid_attn_fwd_ex(dev(q), dev(k), dev(v), dev(q_lin), dev(S), dev(g), out)
    torch.cuda.synchronize()
    prec = "f64"
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), to_np(g), q_lin=to_np(q_lin), precision=prec)
    e = rel_err(to_np(out), ref)
    tol = TOL_BF16_OUT if io == "bf16" else TOL_F32
    assert e <= tol, f"{io}: {e:.3e}"
    # q_lin = None and q_lin = q are the plain entry point, bit for bit
    o1, o2, o3 = (torch.empty_like(q, device="cuda") for _ in range(3))
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S), dev(g), o1)
    lib.arl2_hybrid_attn_fwd_ex(dev(q), dev(k), dev(v), None, dev(S), dev(g), o2)
    lib.arl2_hybrid_attn_fwd_ex(dev(q), dev(k), dev(v), dev(q), dev(S), dev(g), o3)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(o1, o3)
    # the linear branch does not depend on q: v = 0 leaves g * L2Norm(q_lin) S
    vz = torch.zeros_like(v)
    lib.arl2_hybrid_attn_fwd_ex(dev(q), dev(k), dev(vz), dev(q_lin), dev(S), dev(g), o1)
    lib.arl2_hybrid_attn_fwd_ex(dev(k), dev(k), dev(vz), dev(q_lin), dev(S), dev(g), o2)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)


@pytest.mark.parametrize("D,L,rope", [(128, 328, True), (64, 200, True), (128, 257, False)])
def test_readout_with_fused_feature_map(lib, oracle, D, L, rope):
    """arl2_hybrid_attn_fwd_fm against the oracle chain (feature map in fp64, rounded to bf16 where the
    kernel rounds its fragments, then the readout with that query), and against the two-launch path."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"fm{D}", D=D, L=L)
    q, k, v, g = W.pass_inputs(w, 0, 0)
    xq = W.normal(22, w, (w.B, w.L, w.H, w.D), 0, 0, 104)
    Wq, _, _ = W.feature_weights(w)
    cs, sn = W.rope_tables(w) if rope else (None, None)
    S = W.normal(23, w, (w.B, w.H, w.D, w.D), 0, 0, 105, io_dtype="f32") * 0.2
    out = torch.empty_like(q, device="cuda")
    lib.arl2_hybrid_attn_fwd_fm(dev(q), dev(k), dev(v), dev(xq), dev(Wq), dev(cs), dev(sn), dev(S), dev(g), out)
    torch.cuda.synchronize()
    ql_ref = to_np(_bf16_round(oracle.feature_map(to_np(xq), to_np(Wq), None if cs is None else to_np(cs), None if sn is None else to_np(sn))))
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), to_np(g), q_lin=ql_ref)
    e = rel_err(to_np(out), ref)
    assert e <= TOL_BF16_OUT, f"D={D} L={L}: {e:.3e}"
    # the two-launch path computes the same thing: same MFMA order, same roundings
    ql = torch.empty_like(q, device="cuda")
    out2 = torch.empty_like(out)
    lib.arl2_feature_map(dev(xq), dev(Wq), dev(cs), dev(sn), ql)
    lib.arl2_hybrid_attn_fwd_ex(dev(q), dev(k), dev(v), ql, dev(S), dev(g), out2)
    torch.cuda.synchronize()
    assert rel_err(to_np(out), to_np(out2).astype(np.float64)) <= 2.0 ** -7


def _feature_chain(lib, oracle, w, rows=None):
    """Eq. (2)-(7) with the feature maps in place, from pre-RoPE projections: one readout pass and one
    commit on the GPU, and the same chain in the oracle (intermediates rounded to bf16 where the GPU
    stores bf16; nothing the GPU produced reaches the oracle)."""
    xq, xk, xv, g = W.pass_inputs(w, 0, 0)
    xkc, xvc, gate = W.clean_inputs(w, 0)
    Wq, Wk, Wv = W.feature_weights(w)
    cs, sn = W.rope_tables(w)
    eye = torch.eye(w.D, dtype=torch.bfloat16).repeat(w.H, 1, 1).contiguous()
    S0 = W.normal(15, w, (w.B, w.H, w.D, w.D), 0, 0, 97, io_dtype="f32") * 0.2
    # ---- GPU
    d = {n: torch.empty_like(xq, device="cuda") for n in ("q", "k", "ql", "kl", "vl")}
    lib.arl2_feature_map(dev(xq), dev(eye), dev(cs), dev(sn), d["q"])        # RoPE(Q)           Eq. (2)
    lib.arl2_feature_map(dev(xk), dev(eye), dev(cs), dev(sn), d["k"])        # RoPE(K)
    lib.arl2_feature_map(dev(xq), dev(Wq), dev(cs), dev(sn), d["ql"])        # RoPE(phi_q(Q))    Eq. (3)
    lib.arl2_feature_map(dev(xkc), dev(Wk), dev(cs), dev(sn), d["kl"])       # RoPE(phi_k(K)) of the clean pass
    lib.arl2_feature_map(dev(xvc), dev(Wv), None, None, d["vl"])             # phi_v(V)
    S_dev = dev(S0).clone()
    out = torch.empty_like(xq, device="cuda")
    lib.arl2_hybrid_attn_fwd_ex(d["q"], d["k"], dev(xv), d["ql"], S_dev, dev(g), out)
    ws = lib.alloc_workspace(w.B, w.H, w.L, w.D, torch.bfloat16)
    lib.arl2_state_commit(d["kl"], d["vl"], dev(gate), S_dev, ws)
    torch.cuda.synchronize()
    # ---- oracle
    f = to_np
    o = {"q": oracle.feature_map(f(xq), f(eye), f(cs), f(sn)), "k": oracle.feature_map(f(xk), f(eye), f(cs), f(sn)),
         "ql": oracle.feature_map(f(xq), f(Wq), f(cs), f(sn)), "kl": oracle.feature_map(f(xkc), f(Wk), f(cs), f(sn)),
         "vl": oracle.feature_map(f(xvc), f(Wv))}
    o = {n: to_np(_bf16_round(x)) for n, x in o.items()}
    S64 = to_np(S0).astype(np.float64)
    ref = oracle.fwd(o["q"], o["k"], f(xv), S64, f(g), q_lin=o["ql"], rows=rows)
    S_ref = oracle.commit(o["kl"], o["vl"], f(gate), S64)
    got = to_np(out) if rows is None else to_np(out)[:, rows]
    return rel_err(got, ref), rel_err_per_head(to_np(S_dev), S_ref)


def test_feature_map_chain_small(lib, oracle):
    e_out, e_state = _feature_chain(lib, oracle, W.WORKLOADS["ragged_small"])
    # a bf16 intermediate of the GPU may fall one ulp from the oracle's: the state tolerance is the bf16 one here
    assert e_out <= TOL_BF16_OUT and e_state <= 2e-3, f"out {e_out:.3e} state {e_state:.3e}"


def test_feature_map_chain_full_size(lib, oracle):
    w = W.WORKLOADS["wan_layer"]
    e_out, e_state = _feature_chain(lib, oracle, w, rows=sample_rows(w.L, 64, seed=3))
    print(f"[wan_layer] feature-map chain: out {e_out:.3e}, state {e_state:.3e}", flush=True)
    assert e_out <= TOL_BF16_OUT and e_state <= 2e-3


# ---------------------------------------------------------------- headwise mix gate, Eq. (6)

@pytest.mark.parametrize("B,L,H,D,gdt", [(2, 328, 3, 128, "f32"), (1, 200, 12, 128, "bf16"), (1, 33, 5, 64, "f32"), (1, 1, 32, 64, "f32")])
def test_gate_projection_small(lib, oracle, B, L, H, D, gdt):
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"gate{H}x{D}", B=B, L=L, H=H, D=D)
    x, Wg = W.gate_inputs(w, 0, 0)
    Wg = Wg * 8.0                                            # wider logits than the recipe: gates from about 0.1 to 0.9
    g = torch.full((B, L, H), -1.0, dtype=torch.float32 if gdt == "f32" else torch.bfloat16, device="cuda")
    lib.arl2_gate_proj(dev(x), dev(Wg), g)
    torch.cuda.synchronize()
    ref = oracle.gate_proj(to_np(x), to_np(Wg))
    assert ref.min() < 0.3 and ref.max() > 0.7
    err = np.abs(to_np(g) - ref).max()
    assert err <= (2e-6 if gdt == "f32" else 2.0 ** -9), f"{err:.3e}"


@pytest.mark.parametrize("B,L,H,D,n_out,gdt", [
    (2, 200, 2, 64, 0, "f32"),        # element-wise, one output tile, two steps of the hidden dimension
    (1, 333, 3, 64, 0, "bf16"),       # ragged token tile and ragged output tile, odd number of steps
    (1, 130, 5, 64, 0, "f32"),        # three output tiles, five steps
    (3, 77, 2, 128, 0, "f32"),        # fewer tokens than a tile per stream, tiles across streams
    (1, 150, 40, 64, 40, "f32"),      # headwise with more heads than the skinny kernel takes
    (2, 90, 33, 64, 33, "bf16"),      # rows of g that are not 16-byte aligned: element-by-element stores
])
def test_gate_projection_dense(lib, oracle, B, L, H, D, n_out, gdt):
    """More than 32 gate outputs per token (the element-wise gate, or very many heads): the dense kernel."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"gated{H}x{D}", B=B, L=L, H=H, D=D)
    elem = n_out == 0
    x, Wg = W.gate_inputs(w, 0, 0, n_out=H * D if elem else n_out)
    Wg = (Wg * 8.0).contiguous()
    gdtype = torch.float32 if gdt == "f32" else torch.bfloat16
    g = torch.full((B, L, H, D) if elem else (B, L, H), -1.0, dtype=gdtype, device="cuda")
    lib.arl2_gate_proj(dev(x), dev(Wg), g)
    torch.cuda.synchronize()
    ref = oracle.gate_proj(to_np(x), to_np(Wg)).reshape(g.shape)
    assert ref.min() < 0.3 and ref.max() > 0.7
    err = np.abs(to_np(g) - ref).max()
    # fp32 arithmetic: 2e-6; a bf16 gate adds its rounding, half an ulp below 1 = 2^-9
    assert err <= (2e-6 if gdt == "f32" else 2.0 ** -9 + 2e-6), f"{err:.3e}"


@pytest.mark.parametrize("B,L,H,D,gdt", [
    (3, 4400, 39, 64, "f32"),         # 52 x 10 tiles of 256 x 256: ragged last token tile, last output tile 192 wide
    (8, 4680, 12, 128, "bf16"),       # the batched workload: 147 x 6 tiles
])
def test_gate_projection_dense_large_tiles(lib, oracle, B, L, H, D, gdt):
    """Problems that fill the chip at least twice with 256 x 256 tiles take the large-tile kernel: sampled
    tokens against the oracle, and every element written."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"gatebig{H}x{D}", B=B, L=L, H=H, D=D)
    dm = H * D
    assert ((B * L + 255) // 256) * ((dm + 255) // 256) >= 512
    x, Wg = W.gate_inputs(w, 0, 0, n_out=dm)
    Wg = (Wg * 8.0).contiguous()
    g = torch.full((B, L, H, D), -1.0, dtype=torch.float32 if gdt == "f32" else torch.bfloat16, device="cuda")
    lib.arl2_gate_proj(dev(x), dev(Wg), g)
    torch.cuda.synchronize()
    assert float(g.min()) > 0.0 and float(g.max()) < 1.0
    rows = sample_rows(L, 24, seed=7, block=256)
    ref = oracle.gate_proj(to_np(x)[:, rows], to_np(Wg)).reshape(B, len(rows), H, D)
    err = np.abs(to_np(g)[:, rows] - ref).max()
    # fp32 arithmetic: 2e-6; a bf16 gate adds its rounding, half an ulp below 1 = 2^-9
    assert err <= (2e-6 if gdt == "f32" else 2.0 ** -9 + 2e-6), f"{err:.3e}"


def test_elementwise_gate_projection_feeds_the_readout_full_size(lib, oracle):
    """Headline shape: the element-wise gate G = sigmoid(x W_g), W_g 1536 x 1536, on the GPU against the
    oracle on sampled tokens, then used as the readout's gate."""
    w = W.WORKLOADS["wan_layer"]
    dm = w.H * w.D
    x, Wg = W.gate_inputs(w, 0, 0, n_out=dm)
    g = torch.full((w.B, w.L, w.H, w.D), -1.0, dtype=torch.float32, device="cuda")
    lib.arl2_gate_proj(dev(x), dev(Wg), g)
    torch.cuda.synchronize()
    rows = sample_rows(w.L, 48, seed=6)
    g_ref = oracle.gate_proj(to_np(x)[:, rows], to_np(Wg)).reshape(w.B, len(rows), w.H, w.D)
    err = np.abs(to_np(g)[:, rows] - g_ref).max()
    print(f"[wan_layer] element-wise gate projection: max abs err {err:.3e}, gates in [{g_ref.min():.3f}, {g_ref.max():.3f}]", flush=True)
    assert err <= 2e-6
    assert float(g.min()) > 0.0 and float(g.max()) < 1.0          # every element was written
    q, k, v, _ = W.pass_inputs(w, 0, 0)
    S0 = W.normal(16, w, (w.B, w.H, w.D, w.D), 0, 0, 98, io_dtype="f32") * 0.2
    out = torch.empty_like(q, device="cuda")
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S0), g, out)
    torch.cuda.synchronize()
    g_rows = np.full((w.B, w.L, w.H, w.D), 0.5, dtype=np.float32)
    g_rows[:, rows] = g_ref.astype(np.float32)
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S0).astype(np.float64), g_rows, rows=rows)
    e = rel_err(to_np(out)[:, rows], ref)
    assert e <= TOL_BF16_OUT, f"{e:.3e}"


def test_gate_projection_feeds_the_readout_full_size(lib, oracle):
    """Headline shape: G = sigmoid(x W_g) on the GPU against the oracle, then used as the readout's gate."""
    w = W.WORKLOADS["wan_layer"]
    x, Wg = W.gate_inputs(w, 0, 0)
    g = torch.empty((w.B, w.L, w.H), dtype=torch.float32, device="cuda")
    lib.arl2_gate_proj(dev(x), dev(Wg), g)
    torch.cuda.synchronize()
    g_ref = oracle.gate_proj(to_np(x), to_np(Wg))
    err = np.abs(to_np(g) - g_ref).max()
    print(f"[wan_layer] gate projection: max abs err {err:.3e}, gates in [{g_ref.min():.3f}, {g_ref.max():.3f}]", flush=True)
    assert err <= 2e-6
    q, k, v, _ = W.pass_inputs(w, 0, 0)
    S0 = W.normal(16, w, (w.B, w.H, w.D, w.D), 0, 0, 98, io_dtype="f32") * 0.2
    rows = sample_rows(w.L, 32, seed=5)
    out = torch.empty_like(q, device="cuda")
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S0), g, out)
    torch.cuda.synchronize()
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S0).astype(np.float64), g_ref.astype(np.float32), rows=rows)
    e = rel_err(to_np(out)[:, rows], ref)
    assert e <= TOL_BF16_OUT, f"{e:.3e}"


@pytest.mark.parametrize("io,gdt", [("bf16", "f32"), ("bf16", "bf16"), ("f32", "f32")])
def test_elementwise_gate(lib, oracle, io, gdt):
    """One gate per output feature ([B, L, H, D]), the finest granularity of the paper's gate ablation."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name="gate_elem_" + io, io_dtype=io, L=200 if io == "f32" else 328)
    q, k, v, g_head = W.pass_inputs(w, 0, 0)
    ge = W.uniform(19, w, (w.B, w.L, w.H, w.D), 0.0, 1.0, 0, 0, 101)
    if gdt == "bf16":
        ge = ge.to(torch.bfloat16)
    S = W.normal(20, w, (w.B, w.H, w.D, w.D), 0, 0, 102, io_dtype="f32") * 0.2
    out = torch.empty_like(q, device="cuda")
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S), dev(ge), out)
    torch.cuda.synchronize()
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), to_np(ge))
    e = rel_err(to_np(out), ref)
    assert e <= (TOL_BF16_OUT if io == "bf16" else TOL_F32), f"{io}/{gdt}: {e:.3e}"
    # constant over the features it is the headwise gate, bit for bit
    gc = g_head[..., None].expand(-1, -1, -1, w.D).contiguous()
    o1, o2 = torch.empty_like(out), torch.empty_like(out)
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S), dev(gc), o1)
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S), dev(g_head), o2)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)


@pytest.mark.parametrize("io,gdt", [("bf16", "f32"), ("bf16", "bf16"), ("f32", "f32")])
def test_scalar_gate(lib, oracle, io, gdt):
    """One gate per token shared by the heads ([B, L]), the coarsest granularity of the paper's gate
    ablation (Tab. 4), projected on the GPU from a single weight row and used by the readout."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name="gate_tok_" + io, io_dtype=io, L=200 if io == "f32" else 328)
    q, k, v, _ = W.pass_inputs(w, 0, 0)
    wb = dataclasses.replace(w, io_dtype="bf16")
    x, Wg = W.gate_inputs(wb, 0, 0)
    w1 = (Wg[:1] * 8.0).contiguous()                        # one weight row: d_model parameters
    gt = torch.full((w.B, w.L), -1.0, dtype=torch.float32 if gdt == "f32" else torch.bfloat16, device="cuda")
    lib.arl2_gate_proj(dev(x), dev(w1), gt, heads=w.H)
    torch.cuda.synchronize()
    g_ref = oracle.gate_proj(to_np(x), to_np(w1))[..., 0]
    assert g_ref.min() < 0.35 and g_ref.max() > 0.65
    err = np.abs(to_np(gt) - g_ref).max()
    assert err <= (2e-6 if gdt == "f32" else 2.0 ** -9), f"{err:.3e}"
    S = W.normal(20, w, (w.B, w.H, w.D, w.D), 0, 0, 104, io_dtype="f32") * 0.2
    out = torch.empty_like(q, device="cuda")
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S), gt, out)
    torch.cuda.synchronize()
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), to_np(gt))   # the gate values the GPU read
    e = rel_err(to_np(out), ref)
    assert e <= (TOL_BF16_OUT if io == "bf16" else TOL_F32), f"{io}/{gdt}: {e:.3e}"
    ref2 = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), g_ref.astype(np.float32))   # the oracle's own gates
    assert rel_err(to_np(out), ref2) <= (TOL_BF16_OUT if io == "bf16" else TOL_F32)
    # repeated for every head it is the headwise gate, bit for bit
    gh = gt[..., None].expand(-1, -1, w.H).contiguous()
    o2 = torch.empty_like(out)
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k), dev(v), dev(S), gh, o2)
    torch.cuda.synchronize()
    assert torch.equal(out, o2)


def test_degenerate_rows(lib, oracle):
    """All-zero query and key rows (L2Norm gives 0, not NaN), identical keys (uniform softmax), and a
    state commit whose keys are all zero (only the gate acts)."""
    w = W.WORKLOADS["ragged_small"]
    q, k, v, g = W.pass_inputs(w, 0, 0)
    q[:, 5] = 0
    q[:, 100:110] = 0
    k[:, 7] = 0
    k[:, 200:] = k[:, 200:201]                            # a run of identical keys
    S = W.normal(21, w, (w.B, w.H, w.D, w.D), 0, 0, 103, io_dtype="f32") * 0.2
    out = gpu_fwd(lib, q, k, v, S, g)
    assert torch.isfinite(out.float()).all()
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), to_np(g))
    assert rel_err(to_np(out), ref) <= TOL_BF16_OUT
    kz = torch.zeros_like(k)
    _, _, gate = W.clean_inputs(w, 0)
    S_dev = dev(S).clone()
    gpu_commit(lib, kz, v, gate, S_dev)
    np.testing.assert_allclose(to_np(S_dev), to_np(S) * to_np(gate)[..., None, None], rtol=1e-6, atol=1e-7)
    alpha, beta = W.token_gates(w, 0)
    S_dev = dev(S).clone()
    lib.arl2_state_commit_gdn(dev(kz), dev(v), dev(alpha), dev(beta), S_dev, _gdn_ws(lib, w))
    torch.cuda.synchronize()
    want = to_np(S).astype(np.float64) * to_np(alpha).astype(np.float64).prod(axis=1)[..., None, None]
    assert rel_err_per_head(to_np(S_dev), want) <= TOL_STATE


# ---------------------------------------------------------------- stream capture

@pytest.mark.parametrize("long_chunk", [False, True])
def test_chunk_step_replays_from_a_captured_graph(lib, long_chunk):
    """The library neither allocates nor synchronises, so a whole chunk step (readout passes, feature map,
    gate projection, the commit with and without fused maps and from the static scratch array, the delta and the
    token-sequential rule) can be captured into a graph.  Every replay must reproduce the
    eager result bit for bit, with eager work and synchronisations between the replays.  The long chunk
    makes the token-sequential commit walk its blocks as several runs (three launches)."""
    import dataclasses
    w = W.WORKLOADS["ragged_small"]
    if long_chunk:
        w = dataclasses.replace(w, name="graph_long", B=1, H=2, L=1700)
    q, k, v, g = (dev(t) for t in W.pass_inputs(w, 0, 0))
    kc, vc, gate = (dev(t) for t in W.clean_inputs(w, 0))
    alpha, beta_t = (dev(t) for t in W.token_gates(w, 0))
    beta = torch.full((w.B, w.H), 0.1, device="cuda")
    Wq, Wk, Wv = (dev(t) for t in W.feature_weights(w))
    cs, sn = (dev(t) for t in W.rope_tables(w))
    xh, Wg = (dev(t) for t in W.gate_inputs(w, 0, 0))
    S0 = dev(W.normal(18, w, (w.B, w.H, w.D, w.D), 0, 0, 100, io_dtype="f32")) * 0.2
    ws = lib.alloc_workspace(w.B, w.H, w.L, w.D, torch.bfloat16)
    ws_gdn = _gdn_ws(lib, w)
    S = S0.clone()
    out, out_fm, ql, gg = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q), torch.empty_like(g)

    def step():
        lib.arl2_gate_proj(xh, Wg, gg)
        lib.arl2_feature_map(q, Wq, cs, sn, ql)
        lib.arl2_hybrid_attn_fwd_ex(q, k, v, ql, S, gg, out)
        lib.arl2_hybrid_attn_fwd_fm(q, k, v, q, Wq, cs, sn, S, gg, out_fm)
        lib.arl2_state_commit(kc, vc, gate, S, ws)
        lib.arl2_state_commit_fm(kc, Wk, cs, sn, vc, Wv, gate, S, ws)
        lib.arl2_state_commit_static(kc, vc, gate, S)
        lib.arl2_state_commit_delta(kc, vc, gate, beta, S, ws)
        lib.arl2_state_commit_gdn(kc, vc, alpha, beta_t, S, ws_gdn)

    step()                                               # eager reference: one step from S0
    torch.cuda.synchronize()
    out_ref, fm_ref, S_ref = out.clone(), out_fm.clone(), S.clone()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    S.copy_(S0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    for _ in range(3):
        S.copy_(S0)                                      # eager work between the replays
        out.zero_()
        out_fm.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, out_ref) and torch.equal(out_fm, fm_ref) and torch.equal(S, S_ref)


def test_bench_stack_report_runs(lib):
    """The layer-stack report of bench.py (a harness around the same calls) on a shortened rollout."""
    import importlib.util, os
    spec = importlib.util.spec_from_file_location("arl2_bench", os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    r = bench.stack_report(lib, W, torch, torch.device("cuda:0"), chunks=2, reps=1)
    assert r["speedup"] > 1.0 and 0.0 < r["memory_ratio"] < 1.0
    t = r["per_call_ms"]["softmax_kv_pass_by_cached_chunks"]
    assert len(t) == 2 and t[1] > t[0] > 0.0


def test_bench_stack_executed_agrees_with_weighted_sum(lib):
    """The full-stack configuration executed (30 layers, KV caches appended to per chunk, every layer pass and commit
    launched, 3 chunks here) against the weighted sum of separately timed calls: attention time within 5 %, and the
    peak device memory of caches + states against the analytic byte count."""
    import importlib.util, os
    spec = importlib.util.spec_from_file_location("arl2_bench", os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    d = torch.device("cuda:0")
    # (two timings of the same work on a shared machine: if the clock moved between them by more than the margin, both
    # are taken once more; every attempt is printed)
    for attempt in range(2):
        est = bench.stack_report(lib, W, torch, d, chunks=3, reps=3)
        ex = bench.stack_execute(lib, W, torch, d, chunks=3)
        ratios = {name: ex[name]["attention_ms"] / est[name]["attention_ms"] for name in ("hybrid_stack", "softmax_stack")}
        for name, ratio in ratios.items():
            print(f"[stack] {name}: executed {ex[name]['attention_ms']:.1f} ms, weighted sum {est[name]['attention_ms']:.1f} ms, ratio {ratio:.3f}; "
                  f"peak memory {ex[name]['peak_memory_bytes'] / 1e9:.3f} GB, counted {est[name]['memory_bytes'] / 1e9:.3f} GB", flush=True)
        if all(abs(r - 1.0) <= 0.05 for r in ratios.values()):
            break
    for name in ("hybrid_stack", "softmax_stack"):
        assert abs(ratios[name] - 1.0) <= 0.05, (name, ratios[name])
        assert ex[name]["readout_calls"] == 3 * 4 * 30
        # allocator granularity and the commit workspace (hybrid stack only) are all that may come on top
        assert est[name]["memory_bytes"] <= ex[name]["peak_memory_bytes"] <= est[name]["memory_bytes"] + (64 << 20)
    assert ex["speedup"] > 1.0


def _sweep_shapes():
    """Seeded draw of problem shapes around the kernels' tile edges (32-row blocks, 64-key tiles, 256-row
    workgroups), odd head counts and both head dimensions."""
    r = np.random.default_rng(20240607)
    Ls = [1, 2, 31, 32, 33, 63, 64, 65, 127, 129, 255, 256, 257, 300, 511, 513, 640]
    shapes = []
    for i in range(18):
        shapes.append((int(r.integers(1, 4)), int(r.choice([1, 2, 3, 5, 9, 13])), int(r.choice(Ls)), int(r.choice([64, 128]))))
    return shapes


@pytest.mark.parametrize("B,H,L,D", _sweep_shapes())
def test_shape_sweep(lib, oracle, B, H, L, D):
    """One readout pass, one plain commit and one token-sequential commit per drawn shape, element by element."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"sweep_{B}_{H}_{L}_{D}", B=B, H=H, L=L, D=D)
    q, k, v, g = W.pass_inputs(w, 0, 0)
    S0 = W.normal(23, w, (B, H, D, D), 0, 0, 105, io_dtype="f32") * 0.2
    S64 = to_np(S0).astype(np.float64)
    out = gpu_fwd(lib, q, k, v, S0, g)
    e = rel_err(to_np(out), oracle.fwd(to_np(q), to_np(k), to_np(v), S64, to_np(g)))
    assert e <= TOL_BF16_OUT, f"readout {B}x{H}x{L}x{D}: {e:.3e}"
    # a softmax-only layer over a longer key range (cached tokens ahead of the chunk's own), no state
    extra = [0, 1, 63, 64, 200][(B + H + L) % 5]
    wk = dataclasses.replace(w, name=w.name + "_kv", L=L + extra)
    _, k2, v2, _ = W.pass_inputs(wk, 0, 1)
    out2 = torch.empty_like(q, device="cuda")
    lib.arl2_hybrid_attn_fwd(dev(q), dev(k2), dev(v2), None, None, out2)
    torch.cuda.synchronize()
    e = rel_err(to_np(out2), oracle.fwd(to_np(q), to_np(k2), to_np(v2), None, None))
    assert e <= TOL_BF16_OUT, f"softmax over {L + extra} keys {B}x{H}x{L}x{D}: {e:.3e}"
    kc, vc, gate = W.clean_inputs(w, 0)
    S_dev = dev(S0).clone()
    gpu_commit(lib, kc, vc, gate, S_dev)
    e = rel_err_per_head(to_np(S_dev), oracle.commit(to_np(kc), to_np(vc), to_np(gate), S64))
    assert e <= TOL_STATE, f"commit {B}x{H}x{L}x{D}: {e:.3e}"
    alpha, beta = W.token_gates(w, 0)
    S_dev = dev(S0).clone()
    lib.arl2_state_commit_gdn(dev(kc), dev(vc), dev(alpha), dev(beta), S_dev, _gdn_ws(lib, w))
    torch.cuda.synchronize()
    e = rel_err_per_head(to_np(S_dev), oracle.commit_gdn(to_np(kc), to_np(vc), to_np(alpha), to_np(beta), S64))
    assert e <= TOL_STATE, f"gdn commit {B}x{H}x{L}x{D}: {e:.3e}"


@pytest.mark.parametrize("B,H,L,D", _sweep_shapes()[::2])
def test_shape_sweep_maps_and_gates(lib, oracle, B, H, L, D):
    """The feature map, the readout with the fused query map, and the headwise and scalar gate projections
    on every other drawn shape."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["ragged_small"], name=f"sweepfm_{B}_{H}_{L}_{D}", B=B, H=H, L=L, D=D)
    q, k, v, _ = W.pass_inputs(w, 0, 0)
    xq = W.normal(22, w, (B, L, H, D), 0, 0, 104)
    Wq, _, _ = W.feature_weights(w)
    cs, sn = W.rope_tables(w)
    S = W.normal(23, w, (B, H, D, D), 0, 0, 105, io_dtype="f32") * 0.2
    x, Wg = W.gate_inputs(w, 0, 0)
    Wg = Wg * 8.0
    # gates: headwise [B, L, H] and scalar [B, L]
    g = torch.empty((B, L, H), dtype=torch.float32, device="cuda")
    gt = torch.empty((B, L), dtype=torch.float32, device="cuda")
    lib.arl2_gate_proj(dev(x), dev(Wg), g)
    lib.arl2_gate_proj(dev(x), dev(Wg[:1].contiguous()), gt, heads=H)
    y = torch.empty_like(xq, device="cuda")
    lib.arl2_feature_map(dev(xq), dev(Wq), dev(cs), dev(sn), y)
    torch.cuda.synchronize()
    g_ref = oracle.gate_proj(to_np(x), to_np(Wg))
    assert np.abs(to_np(g) - g_ref).max() <= 2e-6
    assert np.abs(to_np(gt) - g_ref[..., 0]).max() <= 2e-6
    y_ref = oracle.feature_map(to_np(xq), to_np(Wq), to_np(cs), to_np(sn))
    assert rel_err(to_np(y), y_ref) <= 2.0 ** -8
    # fused query map, with the oracle's own gates
    out = torch.empty_like(q, device="cuda")
    g32 = torch.from_numpy(g_ref.astype(np.float32))
    lib.arl2_hybrid_attn_fwd_fm(dev(q), dev(k), dev(v), dev(xq), dev(Wq), dev(cs), dev(sn), dev(S), dev(g32), out)
    torch.cuda.synchronize()
    ref = oracle.fwd(to_np(q), to_np(k), to_np(v), to_np(S).astype(np.float64), g_ref.astype(np.float32),
                     q_lin=to_np(_bf16_round(y_ref)))
    e = rel_err(to_np(out), ref)
    assert e <= TOL_BF16_OUT, f"fused map {B}x{H}x{L}x{D}: {e:.3e}"
