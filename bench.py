#!/usr/bin/env python3
"""Benchmark of the ARL^2 hybrid attention chunk step on one MI355X.

One "step" is one pass of the whole hot path over one chunk of synthetic input: `passes`
read-only denoising passes (arl2_hybrid_attn_fwd) that all see the same state, then one
arl2_state_commit.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-step throughput in chunk tokens/s, the roofline figures of the dominant
kernel (the fused flash + readout kernel, timed live with HIP events on the launch stream), and the
CPU oracle timed on a bounded sample of the same workload as a baseline for context.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


def fwd_flops(B, H, L, D):
    """Algorithmic flops of one readout pass: QK^T and PV (4 L^2 D) plus the state readout (2 L D^2)."""
    return B * H * (4.0 * L * L * D + 2.0 * L * D * D)


def commit_flops(B, H, L, D):
    return B * H * 2.0 * L * D * D


def fwd_bytes(B, H, L, D, io_bytes):
    return B * (4.0 * L * H * D * io_bytes + H * D * D * 4.0 + L * H * 4.0)


def commit_bytes(B, H, L, D, io_bytes, rule="plain"):
    """Algorithmic bytes of one commit: k and v read once, S read and written, per-token gates if any."""
    gates = 2.0 * L * H * 4.0 if rule == "gdn" else 0.0
    return B * (2.0 * L * H * D * io_bytes + 2.0 * H * D * D * 4.0 + gates)


def cpu_baseline(w, passes_inputs, clean, S0, steps, rule="plain", rule_inputs=None):
    """The oracle as it stands (fp64, OpenMP over independent rows), timed on this machine's host cores
    on whole chunk steps of the same workload: every readout pass in full, then the commit."""
    import numpy as np

    import workloads as W
    from oracle import arl2_oracle as O
    O.build()
    f = W.as_f32_numpy
    S64 = S0.astype(np.float64)
    ins = [tuple(f(t) for t in pi) for pi in passes_inputs]
    kc, vc, gate = (f(t) for t in clean)
    O.fwd(ins[0][0][:, :8], ins[0][1], ins[0][2], S64, ins[0][3][:, :8])     # warm-up: load the library, spin up threads
    t0 = time.perf_counter()
    for _ in range(steps):
        for (q, k, v, g) in ins:
            O.fwd(q, k, v, S64, g)
        if rule == "plain":
            S64 = O.commit(kc, vc, gate, S64)
        elif rule == "delta":
            S64 = O.commit_delta(kc, vc, gate, f(rule_inputs[0]), S64)
        else:
            S64 = O.commit_gdn(kc, vc, f(rule_inputs[0]), f(rule_inputs[1]), S64)
    t_step = (time.perf_counter() - t0) / steps
    return {
        "value": w.B * w.L / t_step, "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle",
        "sample": f"fp64 oracle, {steps} whole chunk step(s) of {w.name} ({w.passes} full readout passes + 1 commit), "
                  f"{t_step:.2f} s per step",
    }


def stack_report(A, W, torch, dev, layers=30, hybrid_layers=22, chunks=7, reps=5):
    """Attention-only time and memory of a full layer stack over a 7-chunk (21 latent frame) rollout.
    Every layer pass is one arl2_hybrid_attn_fwd call at the Wan-2.1-1.3B layer shape: hybrid layers
    read the fixed-size state; softmax layers attend to a KV cache that holds c chunks at chunk c
    (S = NULL, Lkv = c * 4680).  Layer passes of one kind and one cache length cost the same, so each
    distinct call is timed on its own (median of `reps` batches of back-to-back calls) and the stack total is the
    weighted sum: a cross-check of the executed rollout (stack_execute), which is the measurement.  Inputs are
    synthetic and there is no model between the layers."""
    w = W.WORKLOADS["wan_layer"]
    P = w.passes
    q, k, v, g = (t.to(dev) for t in W.pass_inputs(w, 0, 0))
    kc, vc, gate = (t.to(dev) for t in W.clean_inputs(w, 0))
    out = torch.empty_like(q)
    S = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device=dev)
    ws = A.alloc_workspace(w.B, w.H, w.L, w.D, kc.dtype, device=dev)
    A.arl2_state_commit(kc, vc, gate, S, ws)
    kv_k = W.normal(1, w, (w.B, chunks * w.L, w.H, w.D), 101).to(dev)
    kv_v = W.normal(1, w, (w.B, chunks * w.L, w.H, w.D), 102).to(dev)

    def timed(fn, batch=32):
        """Milliseconds per call: `batch` back-to-back calls between two events (as the calls run in a stack), median of `reps`."""
        for _ in range(batch):
            fn()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(batch):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / batch)
        return sorted(ts)[len(ts) // 2]

    t_hybrid = timed(lambda: A.arl2_hybrid_attn_fwd(q, k, v, S, g, out))
    t_commit = timed(lambda: A.arl2_state_commit(kc, vc, gate, S, ws))
    t_kv = [timed(lambda c=c: A.arl2_hybrid_attn_fwd(q, kv_k[:, :c * w.L], kv_v[:, :c * w.L], None, None, out))
            for c in range(1, chunks + 1)]
    sm_layers = layers - hybrid_layers
    hybrid_ms = sum(P * (hybrid_layers * t_hybrid + sm_layers * t_kv[c]) + hybrid_layers * t_commit for c in range(chunks))
    softmax_ms = sum(P * layers * t_kv[c] for c in range(chunks))
    tok_bytes = w.B * w.H * w.D * 2
    kv_layer_bytes = 2 * chunks * w.L * tok_bytes                      # K and V cache of one softmax layer at full length
    state_bytes = w.B * w.H * w.D * w.D * 4
    return {
        "report": "attention time and memory of a %d-layer stack over %d chunks of %d tokens, %d readout passes per chunk"
                  % (layers, chunks, w.L, P),
        "hybrid_stack": {"layers": "%d hybrid + %d softmax-KV" % (hybrid_layers, sm_layers), "attention_ms": hybrid_ms,
                         "memory_bytes": hybrid_layers * state_bytes + sm_layers * kv_layer_bytes},
        "softmax_stack": {"layers": "%d softmax-KV" % layers, "attention_ms": softmax_ms,
                          "memory_bytes": layers * kv_layer_bytes},
        "speedup": softmax_ms / hybrid_ms,
        "memory_ratio": (hybrid_layers * state_bytes + sm_layers * kv_layer_bytes) / (layers * kv_layer_bytes),
        "per_call_ms": {"hybrid_pass": t_hybrid, "commit": t_commit, "softmax_kv_pass_by_cached_chunks": t_kv},
        "note": "the paper's 2.26x / -54% are end-to-end (denoising + VAE) on another GPU; this is attention only",
    }


def stack_execute(A, W, torch, dev, layers=30, hybrid_layers=22, chunks=7, pool=3):
    """The same stack, executed: for each of `chunks` chunks the chunk's keys and values are appended to the
    KV cache of every softmax layer, then `passes` readout passes run through all layers in order (a hybrid
    layer reads its own fixed-size state, a softmax layer attends to its cache, current chunk included), then
    every hybrid layer commits the chunk.  Both stacks (22 hybrid + 8 softmax-KV, and 30 softmax-KV) run the
    whole rollout back to back on one stream between two events; peak device memory is what torch's allocator
    reports for the caches, states and workspace of the stack (inputs and outputs are allocated before the
    measurement starts and excluded).  Inputs are synthetic: a pool of `pool` pre-drawn (q, k, v, g) sets is
    cycled over layer passes, there is no model between the layers."""
    w = W.WORKLOADS["wan_layer"]
    P, L = w.passes, w.L
    sets = [tuple(t.to(dev) for t in W.pass_inputs(w, 100 + i, 0)) for i in range(pool)]
    cleans = [tuple(t.to(dev) for t in W.clean_inputs(w, 100 + i)) for i in range(pool)]
    out = torch.empty_like(sets[0][0])
    torch.cuda.synchronize()

    def run(n_hybrid):
        n_soft = layers - n_hybrid
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        caches = [(torch.empty((w.B, chunks * L, w.H, w.D), dtype=torch.bfloat16, device=dev),
                   torch.empty((w.B, chunks * L, w.H, w.D), dtype=torch.bfloat16, device=dev)) for _ in range(n_soft)]
        states = [torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device=dev) for _ in range(n_hybrid)]
        ws = A.alloc_workspace(w.B, w.H, L, w.D, torch.bfloat16, device=dev) if n_hybrid else None
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        calls = 0
        e0.record()
        for c in range(chunks):
            kc, vc, gate = cleans[c % pool]
            for (ck, cv) in caches:                                  # cache growth: this chunk's K, V appended
                ck[:, c * L:(c + 1) * L].copy_(kc)
                cv[:, c * L:(c + 1) * L].copy_(vc)
            for p in range(P):
                for l in range(layers):
                    q, k, v, g = sets[(c + p + l) % pool]
                    if l < n_hybrid:
                        A.arl2_hybrid_attn_fwd(q, k, v, states[l], g, out)
                    else:
                        ck, cv = caches[l - n_hybrid]
                        A.arl2_hybrid_attn_fwd(q, ck[:, :(c + 1) * L], cv[:, :(c + 1) * L], None, None, out)
                    calls += 1
            for l in range(n_hybrid):
                A.arl2_state_commit(kc, vc, gate, states[l], ws)
        e1.record()
        torch.cuda.synchronize()
        peak = torch.cuda.max_memory_allocated() - base
        ms = e0.elapsed_time(e1)
        del caches, states, ws
        return ms, peak, calls

    run(hybrid_layers)                                               # warm-up of both code paths and the allocator
    h_ms, h_mem, h_calls = run(hybrid_layers)
    s_ms, s_mem, s_calls = run(0)
    return {"hybrid_stack": {"attention_ms": h_ms, "peak_memory_bytes": h_mem, "readout_calls": h_calls},
            "softmax_stack": {"attention_ms": s_ms, "peak_memory_bytes": s_mem, "readout_calls": s_calls},
            "speedup": s_ms / h_ms, "memory_ratio": h_mem / s_mem}


def rollout_series(A, W, torch, dev, w, pool=4):
    """`w.chunks` consecutive chunk steps (passes readouts + 1 commit each) with the state carried from chunk
    to chunk, every step timed on its own with two events; a pool of `pool` pre-drawn input sets is cycled,
    every chunk has its own forget gate.  Returns the per-chunk latency series and its flatness figures."""
    sets = [[tuple(t.to(dev) for t in W.pass_inputs(w, i, p)) for p in range(w.passes)] for i in range(pool)]
    cleans = [tuple(t.to(dev) for t in W.clean_inputs(w, i)) for i in range(pool)]
    gates = [W.uniform(0, w, (w.B, w.H), w.gate_lo, w.gate_hi, c, 0, W._GATE).to(dev) for c in range(w.chunks)]
    outs = [torch.empty_like(sets[0][p][0]) for p in range(w.passes)]
    S = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device=dev)
    ws = A.alloc_workspace(w.B, w.H, w.L, w.D, torch.bfloat16, device=dev)

    def rollout(timed):
        S.zero_()
        ev = []
        for c in range(w.chunks):
            if timed:
                e0 = torch.cuda.Event(enable_timing=True)
                e0.record()
            for p in range(w.passes):
                q, k, v, g = sets[c % pool][p]
                A.arl2_hybrid_attn_fwd(q, k, v, S, g, outs[p])
            kc, vc, _ = cleans[c % pool]
            A.arl2_state_commit(kc, vc, gates[c], S, ws)
            if timed:
                e1 = torch.cuda.Event(enable_timing=True)
                e1.record()
                ev.append((e0, e1))
        torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in ev]

    rollout(False)                                                   # warm-up: clocks and caches settle
    ms = rollout(True)
    n = len(ms)
    med = sorted(ms)[n // 2]
    xm, ym = (n - 1) / 2.0, sum(ms) / n
    slope = sum((i - xm) * (y - ym) for i, y in enumerate(ms)) / sum((i - xm) ** 2 for i in range(n))
    return {"chunks": n, "ms_per_chunk": [round(x, 4) for x in ms], "median_ms": med, "max_over_median": max(ms) / med,
            "p90_over_median": sorted(ms)[int(0.9 * n)] / med, "drift_over_rollout": slope * n / med}


def source_sha16(path):
    import hashlib
    return hashlib.sha256(open(path, "rb").read()).hexdigest()[:16]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="wan_layer", choices=["wan_layer", "wan_batched", "ragged_small", "wan_rollout"],
                    help="wan_layer is the bench workload; wan_rollout runs its 64 chunk steps one after the other, "
                         "state carried, and reports the per-chunk latency series instead of the bench line")
    ap.add_argument("--commit-rule", default="plain", choices=["plain", "delta", "gdn"],
                    help="state update of the step: plain (the headline: gate * S + K'^T V), delta (Eq. (4) at frame "
                         "level, one learning rate per head), gdn (Eq. (4) token by token, per-token gates)")
    ap.add_argument("--feature-maps", action="store_true",
                    help="put the learned per-head maps of Eq. (3) on the path: every readout pass first computes "
                         "q_lin = RoPE(phi_q(Q)) (arl2_feature_map) and reads the state with it; the commit is preceded by "
                         "RoPE(phi_k(K)) and phi_v(V) of the clean pass.  Not the headline configuration.")
    ap.add_argument("--unfused-maps", action="store_true",
                    help="with --feature-maps: every map as a separate arl2_feature_map launch instead of inside the readout "
                         "and (plain rule) the commit kernel")
    ap.add_argument("--gate-proj", action="store_true",
                    help="compute the mix gate of every readout pass on the path, G = sigmoid(x W_g) (arl2_gate_proj), "
                         "instead of taking it as an input.  Not the headline configuration.")
    ap.add_argument("--gate-granularity", choices=["head", "token", "element"], default="head",
                    help="with --gate-proj: one gate per (token, head) (the paper's choice), per token, or per output "
                         "feature (W_g is d_model x d_model: a dense product), the three rows of the gate ablation")
    ap.add_argument("--clean-readout", action="store_true",
                    help="one more readout pass per step, on the clean pass's inputs before the commit "
                         "(passes + 1 readouts, then the commit).  Not the headline configuration.")
    ap.add_argument("--cpu-steps", type=int, default=3, help="whole chunk steps timed on the CPU oracle")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stack-report", action="store_true",
                    help="instead of the bench line: attention time and memory of a 30-layer stack over a "
                         "21-latent-frame rollout (7 chunks), 22 hybrid + 8 softmax-KV layers vs 30 softmax-KV layers")
    ap.add_argument("--execute", action="store_true",
                    help="with --stack-report: also run the whole rollout of both stacks for real (KV caches allocated and "
                         "appended to per chunk, every layer pass launched), time it end to end and report peak memory")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of 256 MiB (5 times): the reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (heads and streams are independent, so the step "
              "shards without any exchange); --gpus must be 1", file=sys.stderr)
        return 2

    import torch

    import paper_2605_16579_amd as A
    import workloads as W

    A.load_library()   # fails loudly if the HIP library is missing: there is no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        n = 256 << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": n, "copies": 5}))
        return 0
    w = W.WORKLOADS[args.workload]
    io_bytes = 2 if w.io_dtype == "bf16" else 4
    if args.stack_report:
        rep = stack_report(A, W, torch, dev)
        if args.execute:
            ex = stack_execute(A, W, torch, dev)
            rep["executed"] = ex
            rep["executed_over_weighted_sum"] = {
                "hybrid_stack": ex["hybrid_stack"]["attention_ms"] / rep["hybrid_stack"]["attention_ms"],
                "softmax_stack": ex["softmax_stack"]["attention_ms"] / rep["softmax_stack"]["attention_ms"]}
        print(json.dumps(rep), flush=True)
        return 0
    if args.workload == "wan_rollout":
        ser = rollout_series(A, W, torch, dev, w)
        total_ms = sum(ser["ms_per_chunk"])
        print(json.dumps({"metric": "per-chunk latency over a 64-chunk rollout (4 readout passes + 1 commit per chunk, state carried)",
                          "value": w.B * w.L * ser["chunks"] / (total_ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
                          "higher_is_better": True, "dtype": w.io_dtype, "data": "synthetic",
                          "config": {"workload": f"{w.name}: B={w.B} H={w.H} D={w.D} L={w.L}, {w.chunks} chunks"},
                          "rollout": ser}), flush=True)
        return 0

    # ---- inputs, resident in HBM
    passes_cpu = [W.pass_inputs(w, 0, p) for p in range(w.passes)]
    clean_cpu = W.clean_inputs(w, 0)
    passes = [tuple(t.to(dev) for t in pi) for pi in passes_cpu]
    kc, vc, gate = (t.to(dev) for t in clean_cpu)
    outs = [torch.empty_like(passes[p][0]) for p in range(w.passes)]
    S = torch.zeros((w.B, w.H, w.D, w.D), dtype=torch.float32, device=dev)
    ws = A.alloc_workspace(w.B, w.H, w.L, w.D, kc.dtype, device=dev)
    rule = args.commit_rule
    rule_cpu = None
    if rule == "delta":       # learning rate in the range where the frame-level rule is a contraction (below 2 D / L)
        rule_cpu = (W.uniform(0, w, (w.B, w.H), 0.2 * w.D / w.L, 1.0 * w.D / w.L, 0, 0, 77),)
    elif rule == "gdn":
        rule_cpu = W.token_gates(w, 0)
        ws_gdn = torch.empty(A.arl2_gdn_workspace_bytes(w.B, w.H, w.L, w.D), dtype=torch.uint8, device=dev)
    rule_dev = None if rule_cpu is None else tuple(t.to(dev) for t in rule_cpu)

    gp = None
    if args.gate_proj:
        if w.io_dtype != "bf16":
            print("bench.py: --gate-proj needs a bf16 workload", file=sys.stderr)
            return 2
        n_gate = {"head": w.H, "token": 1, "element": w.H * w.D}[args.gate_granularity]
        g_shape = {"head": (w.B, w.L, w.H), "token": (w.B, w.L), "element": (w.B, w.L, w.H, w.D)}[args.gate_granularity]
        gp = [tuple(t.to(dev) for t in W.gate_inputs(w, 0, p, n_out=n_gate)) +
              (torch.empty(g_shape, dtype=torch.float32, device=dev),) for p in range(w.passes)]
    n_read = w.passes + (1 if args.clean_readout else 0)
    fm = None
    if args.feature_maps:
        if w.io_dtype != "bf16":
            print("bench.py: --feature-maps needs a bf16 workload", file=sys.stderr)
            return 2
        Wq, Wk, Wv = (t.to(dev) for t in W.feature_weights(w))
        cs, sn = (t.to(dev) for t in W.rope_tables(w))
        fm = {"Wq": Wq, "Wk": Wk, "Wv": Wv, "cs": cs, "sn": sn, "ql": torch.empty_like(kc),
              "kl": torch.empty_like(kc), "vl": torch.empty_like(kc)}

    def commit():
        if fm is not None and rule == "plain" and not args.unfused_maps:
            # the key and value maps run inside the commit kernel: no intermediate arrays, no extra launches
            A.arl2_state_commit_fm(kc, fm["Wk"], fm["cs"], fm["sn"], vc, fm["Wv"], gate, S, ws)
            return
        if fm is not None:
            A.arl2_feature_map(kc, fm["Wk"], fm["cs"], fm["sn"], fm["kl"])
            A.arl2_feature_map(vc, fm["Wv"], None, None, fm["vl"])
            kk, vv = fm["kl"], fm["vl"]
        else:
            kk, vv = kc, vc
        _commit(kk, vv)

    def _commit(kc, vc):
        if rule == "plain":
            A.arl2_state_commit(kc, vc, gate, S, ws)
        elif rule == "delta":
            A.arl2_state_commit_delta(kc, vc, gate, rule_dev[0], S, ws)
        else:
            A.arl2_state_commit_gdn(kc, vc, rule_dev[0], rule_dev[1], S, ws_gdn)
    for j in range(w.prefill):     # input preparation: the state the chunk starts from
        pk, pv, pg = (t.to(dev) for t in W.prefill_inputs(w, j))
        A.arl2_state_commit(pk, pv, pg, S, ws)
    torch.cuda.synchronize()
    S0 = S.detach().cpu().numpy().copy()

    # Two events per step on the launch stream: before the first readout pass and after the last one
    # (a record between every pair of launches costs ~15 % of the step on this machine).
    def step(events=None):
        if events is not None:
            e0 = torch.cuda.Event(enable_timing=True)
            e0.record()
        for p in range(n_read):
            q, k, v, g = passes[p % w.passes]
            if gp is not None:
                xg, Wg, g = gp[p % w.passes]
                A.arl2_gate_proj(xg, Wg, g, heads=w.H)
            if fm is not None:
                if args.unfused_maps:
                    A.arl2_feature_map(q, fm["Wq"], fm["cs"], fm["sn"], fm["ql"])
                    A.arl2_hybrid_attn_fwd_ex(q, k, v, fm["ql"], S, g, outs[p % w.passes])
                else:      # the query map fused into the readout kernel: no intermediate array, one launch
                    A.arl2_hybrid_attn_fwd_fm(q, k, v, q, fm["Wq"], fm["cs"], fm["sn"], S, g, outs[p % w.passes])
            else:
                A.arl2_hybrid_attn_fwd(q, k, v, S, g, outs[p % w.passes])
        if events is not None:
            e1 = torch.cuda.Event(enable_timing=True)
            e1.record()
            events.append((e0, e1))
        commit()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    end = torch.cuda.Event(enable_timing=True)
    end.record()
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0

    ms_per_step = 1e3 * t_total / args.steps
    # readout launch time: span of the `passes` back-to-back launches of a step / passes;
    # commit time: from the end of a step's last readout pass to the start of the next step
    fwd_ms = [e0.elapsed_time(e1) / n_read for (e0, e1) in events]
    nxt = [e[0] for e in events[1:]] + [end]
    com_ms = [events[i][1].elapsed_time(nxt[i]) for i in range(len(events))]
    fwd_avg_ms = sum(fwd_ms) / len(fwd_ms)
    com_avg_ms = sum(com_ms) / len(com_ms)

    ff, cf = fwd_flops(w.B, w.H, w.L, w.D), commit_flops(w.B, w.H, w.L, w.D)
    step_flops = n_read * ff + cf
    fwd_tflops = ff / (fwd_avg_ms * 1e-3) / 1e12
    step_tflops = step_flops / (ms_per_step * 1e-3) / 1e12
    result = {
        "metric": "hybrid-attn tokens/s + TFLOP/s (% bf16 MFMA peak) per chunk step, 4680 tok",
        "value": w.B * w.L / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.io_dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} D={w.D} L={w.L}, {w.passes} readout passes + 1 commit per step",
                   "passes": w.passes, "commit_rule": rule, "feature_maps": (("query map fused into the readout" + (", key and value maps fused into the commit" if rule == "plain" else ""))
                                    if not args.unfused_maps else "separate launches") if args.feature_maps else False, "gate_proj": args.gate_granularity if args.gate_proj else False,
                   "readouts_per_step": n_read, "state": "fp32 [B,H,D,D], pre-filled by %d commits" % w.prefill},
        "step_tflops": step_tflops,
        "step_frac_bf16_peak": step_tflops / PEAK_BF16_TFLOPS,
        "token_passes_per_s": w.B * w.L * n_read / (ms_per_step * 1e-3),
        "fwd_ms": fwd_avg_ms, "fwd_ms_min": min(fwd_ms),
        "commit_ms": com_avg_ms, "commit_ms_min": min(com_ms),
        "commit_gbs": commit_bytes(w.B, w.H, w.L, w.D, io_bytes, rule) / (com_avg_ms * 1e-3) / 1e9,
        "commit_frac_hbm_peak": commit_bytes(w.B, w.H, w.L, w.D, io_bytes, rule) / (com_avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "fwd_gbs": fwd_bytes(w.B, w.H, w.L, w.D, io_bytes) / (fwd_avg_ms * 1e-3) / 1e9,
        "roofline": {"kernel": "fwd_bf16_kernel (flash softmax + fused state readout)",
                     "bound": "mfma", "achieved": fwd_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": fwd_tflops / PEAK_BF16_TFLOPS, "traffic": None},
    }
    # HBM bytes per launch come from a committed rocprofv3 counter run; they are only quoted while the kernel
    # source is the one that run profiled
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        t = json.load(open(traffic_file)).get(w.name)
        src = os.path.join(ROOT, "paper_2605_16579_amd", "csrc", "arl2_fwd_bf16.hip")
        if t and t.get("fwd_kernel_source_sha16") == source_sha16(src):
            result["roofline"]["traffic"] = t.get("fwd_hbm_bytes_per_launch")
            result["roofline"]["traffic_source"] = "profiles/traffic.json (%s), kernel source %s" % (
                t.get("profile", "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE"), t.get("fwd_kernel_source_sha16"))
        elif t:
            result["roofline"]["traffic_source"] = "profiles/traffic.json is for another version of the kernel source: not quoted"
    if not args.no_cpu_baseline and fm is None and gp is None and not args.clean_readout:
        result["cpu_baseline"] = cpu_baseline(w, passes_cpu, clean_cpu, S0, args.cpu_steps, rule, rule_cpu)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
