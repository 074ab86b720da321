#!/usr/bin/env python3
"""Benchmark of the BP-Transformer graph self-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload lm] [--no-cpu-baseline]

A step is one forward + backward of graph self-attention (paper Sec. 3.1 eq. 6,
Sec. 3.4 eq. 8) over one synthetic batch, on a graph built once beforehand by the
GPU graph builder (Sec. 3.2) -- the graph depends only on (n, k, causal) and is
shared by every layer, head and batch, so its build time is reported separately
(`graph_build_ms`, and `edges_per_s_incl_build` charges one build to every step).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
# HBM bytes per launch of a kernel, from rocprofv3 FETCH_SIZE (x2.0: the counter reads half the bytes of a
# plain device copy of known size, `--calibrate-copy-mib`) + WRITE_SIZE on this
# workload; the runs and their commands are in profiles/.  None where not measured.
MEASURED_TRAFFIC = {
    "lm": {  # profiles/lm_n8192_k8_causal_bf16_kernels.md
        "bwd_kv_tile_kernel": int((212833.0 * 2.0 + 279937.0) * 1024),
        "bwd_q_tile_kernel": int((132667.0 * 2.0 + 77826.0) * 1024),
        "fwd_tile_kernel": int((116273.0 * 2.0 + 36091.0) * 1024),
        "bwd_q_span_tile_kernel": int((67596.0 * 2.0 + 105082.0) * 1024),
        "fwd_span_tile_kernel": int((49609.0 * 2.0 + 59992.0) * 1024),
    },
}
# HBM bytes of one whole step (all kernels, same counters and scaling)
MEASURED_STEP_TRAFFIC = {"lm": 1852491634}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="lm")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout rate on the attention weights (the mask is formed inside the kernels); 0 = the "
                         "headline configuration")
    ap.add_argument("--layer", action="store_true",
                    help="time the forward of one whole graph layer (projections, attention, FFN, normalisations; "
                         "d_ff = 4 d) of the workload's shape instead of the attention path")
    ap.add_argument("--layers", type=int, default=1,
                    help="with --layer: the update of the graph over this many layers, from the embeddings to the "
                         "token rows (causal workloads) or the root's row of the last layer, forward + backward")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="only run a plain device-to-device copy of this many MiB (10 times) and exit: the known "
                         "traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    return ap.parse_args()


def layer_params(torch, rnd, d, d_ff):
    p = {k_: rnd(d, d, s=d ** -0.5).to(torch.bfloat16) for k_ in ("Wq", "Wk", "Wv", "Wo")}
    p["W1"] = rnd(d, d_ff, s=d ** -0.5).to(torch.bfloat16)
    p["W2"] = rnd(d_ff, d, s=d_ff ** -0.5).to(torch.bfloat16)
    p.update(b1=rnd(d_ff, s=0.1), b2=rnd(d, s=0.1), g1=1 + rnd(d, s=0.1), beta1=rnd(d, s=0.1), g2=1 + rnd(d, s=0.1),
             beta2=rnd(d, s=0.1))
    return p


def bench_stack(args, w, bpt, torch, np):
    """Forward + backward of the update of the graph (Sec. 3.3) over --layers layers on the workload's shape: from
    the embeddings [B, n, d] to the token rows (causal workloads: language modelling) or the root's row
    (classification) of the last layer and back; d = heads * 64, d_ff = 4 d, random bf16 weights."""
    from paper_1911_04070_amd.workloads import make_lengths
    d, d_ff, layers = w.H * w.D, 4 * w.H * w.D, args.layers
    g = bpt.bpt_build_graph(w.n, w.k, w.causal)
    gen = torch.Generator(device="cuda").manual_seed(1911 + w.index)
    rnd = lambda *shape, s=1.0: (s * torch.randn(*shape, device="cuda", generator=gen))
    E = rnd(w.B, w.n, d).to(torch.bfloat16)
    rels = [rnd(g.num_levels, g.rel_width, w.D, s=0.02).to(torch.bfloat16) for _ in range(layers)]
    params = [layer_params(torch, rnd, d, d_ff) for _ in range(layers)]
    lens_d = torch.from_numpy(make_lengths(w)).cuda() if w.length_mix else None
    tokens_out = bool(w.causal)
    d_root = None if tokens_out else rnd(w.B, d).to(torch.bfloat16)
    d_tokens = rnd(w.B, w.n, d).to(torch.bfloat16) if tokens_out else None
    fws, bws = bpt.stack_workspace_bytes(g, w.B, w.H, d_ff, layers)
    ws = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")
    fwd = lambda: bpt.bpt_stack_fwd(g, E, rels, params, w.H, scale=w.scale, seq_len=lens_d, want_root=not tokens_out,
                                    want_tokens=tokens_out, workspace=ws)
    bwd = lambda: bpt.bpt_stack_bwd(g, E, rels, params, w.H, ws, d_root, d_tokens, scale=w.scale, seq_len=lens_d,
                                    workspace=ws_b)

    def wall_ms(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    for _ in range(args.warmup + 2):
        fwd()
        bwd()
    ms = wall_ms(lambda: (fwd(), bwd()))
    ms_fwd = wall_ms(fwd)
    rows = w.B * g.num_nodes
    tokens = int(make_lengths(w).sum()) if w.length_mix else w.B * w.n   # the tokens that exist, not the padding
    flops = layers * 3 * 2.0 * rows * (4 * d * d + 2 * d * d_ff)
    print(json.dumps({
        "metric": "BPT graph update fwd+bwd tokens/sec", "value": round(tokens / (ms * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "dtype": "bf16", "data": "synthetic", "vs_baseline": None, "forward_ms": round(ms_fwd, 4),
        "config": {"workload": "%s+%d layers" % (w.name, layers), "n": w.n, "k": w.k, "causal": w.causal, "batch": w.B,
                   "heads": w.H, "d_model": d, "d_ff": d_ff, "layers": layers, "node_rows": rows, "tokens": tokens,
                   "output": "tokens" if tokens_out else "root"},
        "dense_TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1),
        "workspace_GB": round((fws + bws) / 1e9, 2),
    }), flush=True)


def bench_layer(args, w, bpt, torch, np):
    """Forward + backward of one graph layer (Sec. 3.3) on the workload's shape: d = heads * 64, d_ff = 4 d, random
    bf16 weights."""
    from paper_1911_04070_amd.workloads import make_lengths
    d, d_ff = w.H * w.D, 4 * w.H * w.D
    g = bpt.bpt_build_graph(w.n, w.k, w.causal)
    gen = torch.Generator(device="cuda").manual_seed(1911 + w.index)
    rnd = lambda *shape, s=1.0: (s * torch.randn(*shape, device="cuda", generator=gen))
    X = rnd(w.B, g.num_nodes, d).to(torch.bfloat16)
    X[:, w.n:] = 0                                            # span nodes start from zero
    R = rnd(g.num_levels, g.rel_width, w.D, s=0.02).to(torch.bfloat16)
    p = layer_params(torch, rnd, d, d_ff)
    lens_d = torch.from_numpy(make_lengths(w)).cuda() if w.length_mix else None
    Y = torch.empty_like(X)
    dY = rnd(w.B, g.num_nodes, d).to(torch.bfloat16)
    dX = torch.empty_like(X)
    d_rel = torch.empty(R.shape, dtype=torch.float32, device="cuda")
    grads = {"d" + k_: torch.empty(v.shape, dtype=torch.float32, device="cuda") for k_, v in p.items()}
    fws, bws = bpt.layer_workspace_bytes(g, w.B, w.H, d_ff)
    ws = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")
    fwd = lambda: bpt.bpt_layer_fwd(g, X, R, p, w.H, scale=w.scale, seq_len=lens_d, out=Y, workspace=ws)
    bwd = lambda: bpt.bpt_layer_bwd(g, X, R, p, w.H, ws, dY, scale=w.scale, seq_len=lens_d, dX=dX, grads=grads, d_rel=d_rel,
                                    workspace=ws_b)

    def step():
        fwd()
        bwd()

    def wall_ms(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    for _ in range(args.warmup + 2):                         # the first GEMM calls load the library's kernels
        step()
    ms = wall_ms(step)
    ms_fwd = wall_ms(fwd)
    bpt.bpt_profile_enable(True)
    for _ in range(5):
        step()
    torch.cuda.synchronize()
    own = {name: total / 5 for name, (calls, total) in bpt.bpt_profile_report().items()}   # ms per step, all its launches
    bpt.bpt_profile_enable(False)
    rows = w.B * g.num_nodes
    flops = 3 * 2.0 * rows * (4 * d * d + 2 * d * d_ff)       # the backward has two products per forward product
    print(json.dumps({
        "metric": "BPT graph layer fwd+bwd node rows/sec", "value": round(rows / (ms * 1e-3), 1), "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "dtype": "bf16", "data": "synthetic", "vs_baseline": None, "forward_ms": round(ms_fwd, 4),
        "config": {"workload": w.name + "+layer", "n": w.n, "k": w.k, "causal": w.causal, "batch": w.B, "heads": w.H,
                   "d_model": d, "d_ff": d_ff, "node_rows": rows},
        "dense_TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1),
        "own_kernel_ms": {k_: round(v, 4) for k_, v in sorted(own.items(), key=lambda kv: -kv[1])},
        "gemm_and_gaps_ms": round(ms - sum(own.values()), 4),
    }), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); the path shards over (batch, head) "
              "without communication (one all-reduce of d_rel in the backward)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.calibrate_copy_mib > 0:
        torch.cuda.set_device(0)
        src = torch.ones(args.calibrate_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_mib": args.calibrate_copy_mib, "copies": 10}), flush=True)
        return

    from paper_1911_04070_amd import binding as bpt
    from paper_1911_04070_amd.workloads import WORKLOADS, make_inputs, make_lengths

    if not os.path.exists(bpt.LIB_PATH):
        from paper_1911_04070_amd.build import build_library
        build_library()
    w = WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    if args.layer:
        return (bench_stack if args.layers > 1 else bench_layer)(args, w, bpt, torch, np)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    bytes_scale = 1.0 if w.dtype == "bf16" else 2.0

    x = make_inputs(w)
    dev = {k: torch.from_numpy(v).to(tdt).cuda() for k, v in x.items()}

    # graph build (GPU kernels + host schedule), timed on its own
    torch.cuda.synchronize()
    g = bpt.bpt_build_graph(w.n, w.k, w.causal)
    g.destroy()
    t0 = time.perf_counter()
    g = bpt.bpt_build_graph(w.n, w.k, w.causal)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) * 1e3
    # sequences of different lengths: only the edges a sequence keeps count as work
    lengths = make_lengths(w) if w.length_mix else None
    lens_d = torch.from_numpy(lengths).cuda() if lengths is not None else None
    if lengths is None:
        edge_inst = w.B * w.H * g.num_edges
    else:
        edge_inst = w.H * sum(bpt.bpt_count_edges(w.n, w.k, w.causal, int(x)) for x in lengths)

    Q, K, V, R, dO = dev["Q"], dev["K"], dev["V"], dev["Rel"], dev["dO"]
    out = torch.empty_like(Q)
    lse = torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty(Q.shape, dtype=torch.float32, device="cuda") for _ in range(3)) + (
        torch.empty(R.shape, dtype=torch.float32, device="cuda"),)
    fws, bws = bpt.workspace_bytes(g, Q, w.scale)
    ws_f = torch.empty(max(fws, 256), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(bws, 256), dtype=torch.uint8, device="cuda")

    drop = (args.dropout, 1911) if args.dropout > 0 else None

    def step():
        bpt.bpt_attn_fwd(g, Q, K, V, R, scale=w.scale, out=out, lse=lse, workspace=ws_f, seq_len=lens_d, dropout=drop)
        if w.backward:
            bpt.bpt_attn_bwd(g, Q, K, V, R, lse, dO, scale=w.scale, grads=grads, workspace=ws_b, seq_len=lens_d,
                             dropout=drop)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-stage device time with events on the stream the library launches on
    def timed(fn, reps):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in evs]))

    reps = max(5, min(args.steps, 30))
    stage_ms = {"fwd": timed(lambda: bpt.bpt_attn_fwd(g, Q, K, V, R, scale=w.scale, out=out, lse=lse,
                                                      workspace=ws_f, seq_len=lens_d, dropout=drop), reps)}
    if w.backward:
        stage_ms["bwd_query_side"] = timed(
            lambda: bpt.bpt_attn_bwd_query_side(g, Q, K, V, R, lse, dO, grads[0], grads[3], ws_b, scale=w.scale,
                                                seq_len=lens_d, dropout=drop), reps)
        stage_ms["bwd_key_side"] = timed(
            lambda: bpt.bpt_attn_bwd_key_side(g, Q, K, V, R, lse, dO, grads[1], grads[2], ws_b, scale=w.scale,
                                              seq_len=lens_d, dropout=drop), reps)

    # per-kernel device time, live: the library brackets each of its launches with HIP events on the launch stream
    bpt.bpt_profile_enable(True)
    for _ in range(reps):
        step()
    torch.cuda.synchronize()
    prof = bpt.bpt_profile_report()
    bpt.bpt_profile_enable(False)
    kernel_ms = {name: total / calls for name, (calls, total) in prof.items()}

    # what a plain device-to-device copy of 256 MiB reaches on this machine (read + write), beside the published peak
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    copy_ms = timed(lambda: dst.copy_(src), 10)
    copy_gbs = 2.0 * src.numel() / (copy_ms * 1e-3) / 1e9
    del src, dst

    # algorithmic bytes per launch: every edge-instance a gather kernel handles counts one
    # key row + one value row (or one query row + one dout row): 256 B in bf16, 512 B in fp32
    bh = w.B * w.H
    if lengths is None:
        tok_inst = int(g.csr_to_host()[0][w.n]) * bh
    else:   # every level above the tokens holds each token of a sequence once
        tok_inst = edge_inst - w.H * int(lengths.sum()) * (g.num_levels - 1)
    span_inst = edge_inst - tok_inst
    gather = 256.0 * bytes_scale
    alg_bytes = {
        "fwd_tile_kernel": gather * tok_inst, "bwd_q_tile_kernel": gather * tok_inst,
        "fwd_span_tile_kernel": gather * span_inst, "bwd_q_span_tile_kernel": gather * span_inst,
        "bwd_kv_tile_kernel": gather * edge_inst, "bwd_kv_kernel": gather * edge_inst,
    }
    # the gather kernels take whatever rows the tile kernels of this launch did not
    alg_bytes["fwd_kernel"] = gather * (edge_inst - (tok_inst if "fwd_tile_kernel" in kernel_ms else 0) - (
        span_inst if "fwd_span_tile_kernel" in kernel_ms else 0))
    alg_bytes["bwd_q_kernel"] = gather * (edge_inst - (tok_inst if "bwd_q_tile_kernel" in kernel_ms else 0) - (
        span_inst if "bwd_q_span_tile_kernel" in kernel_ms else 0))
    main = {k: v for k, v in kernel_ms.items() if k in alg_bytes}
    dominant = max(main, key=main.get)
    achieved = alg_bytes[dominant] / (kernel_ms[dominant] * 1e-3) / 1e9
    step_alg_bytes = gather * (3 if w.backward else 1) * edge_inst
    esz = 2 if w.dtype == "bf16" else 4
    tensor = bh * g.num_nodes * w.D
    # the tensors of the boundary, each moved once per stage that needs it: the forward reads Q, K, V and
    # writes out, lse; the backward reads Q, K, V, dout, lse and writes dQ, dK, dV (fp32) -- no workspace traffic
    compulsory = tensor * esz * 4 + bh * g.num_nodes * 4
    if w.backward:
        compulsory += tensor * esz * 4 + bh * g.num_nodes * 4 + 3 * tensor * 4
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "device_copy_GBs": round(copy_gbs, 1),
        "traffic": MEASURED_TRAFFIC.get(w.name, {}).get(dominant),
        "launch_ms": round(kernel_ms[dominant], 4),
        "algorithmic_bytes_per_edge_instance": gather,
        "kernel_ms": {k: round(v, 4) for k, v in sorted(kernel_ms.items(), key=lambda kv: -kv[1])},
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "step_algorithmic_GBs": round(step_alg_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_measured_hbm_bytes": MEASURED_STEP_TRAFFIC.get(w.name),
        "step_measured_hbm_frac_of_peak": (round(MEASURED_STEP_TRAFFIC[w.name] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                                           if w.name in MEASURED_STEP_TRAFFIC else None),
        "step_compulsory_bytes": int(compulsory),
        "step_compulsory_frac_of_hbm_peak": round(compulsory / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "note": "achieved counts one gathered row pair per edge-instance (the algorithmic bytes of the method); the "
                "tile kernels fetch a row once per 16-row tile and re-use it on chip, so achieved can exceed the HBM "
                "peak while the measured HBM traffic (traffic, profiles/) stays far below it",
    }

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        og = oracle.build_graph(w.n, w.k, w.causal)
        passes, dt, used = 0, 0.0, 1
        while passes < 1 or (dt < 5.0 and passes < 50):      # a few seconds of wall time on all cores
            t0 = time.perf_counter()
            if lengths is not None:
                oracle.attn_fwd_lengths(w.n, w.k, w.causal, lengths, x["Q"], x["K"], x["V"], x["Rel"], w.scale)
                if w.backward:
                    oracle.attn_bwd_lengths(w.n, w.k, w.causal, lengths, x["Q"], x["K"], x["V"], x["Rel"], x["dO"], w.scale)
                used = min(os.cpu_count() or 1, w.H)
            else:
                _, _, used = oracle.attn_fwd(og, x["Q"], x["K"], x["V"], x["Rel"], w.scale)
            if w.backward and lengths is None:
                oracle.attn_bwd(og, x["Q"], x["K"], x["V"], x["Rel"], x["dO"], w.scale)
            dt += time.perf_counter() - t0
            passes += 1
        # the same oracle on one thread, on the first (batch, head) of the workload
        one = {k_: np.ascontiguousarray(v[:1, :1]) for k_, v in x.items() if k_ != "Rel"}
        len0 = int(lengths[0]) if lengths is not None else w.n
        g1 = og if lengths is None else oracle.build_graph_len(w.n, len0, w.k, w.causal)
        t0 = time.perf_counter()
        oracle.attn_fwd(g1, one["Q"], one["K"], one["V"], x["Rel"], w.scale, threads=1)
        if w.backward:
            oracle.attn_bwd(g1, one["Q"], one["K"], one["V"], x["Rel"], one["dO"], w.scale, threads=1)
        dt1 = time.perf_counter() - t0
        cpu = {"value": round(edge_inst * passes / dt, 1), "unit": "edges/s", "cores": used, "kind": "oracle",
               "sample": "the whole workload, %d pass(es) of forward%s in fp64, %.1f s wall" % (
                   passes, " + backward" if w.backward else "", dt),
               "one_thread_value": round(g1.num_edges / dt1, 1),
               "one_thread_sample": "one (batch, head) of the workload, %.2f s" % dt1}

    res = {
        "metric": "BPT graph-attention fwd+bwd edges/sec" if w.backward else "BPT graph-attention fwd edges/sec",
        "value": round(edge_inst / (ms_per_step * 1e-3), 1),
        "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "k": w.k, "causal": w.causal, "batch": w.B, "heads": w.H,
                   "head_dim": w.D, "nodes": g.num_nodes, "edges": g.num_edges, "edge_instances": edge_inst,
                   "backward": w.backward, "dropout": args.dropout,
                   "lengths": ([int(v) for v in lengths] if lengths is not None else None)},
        "graph_build_ms": round(build_ms, 3),
        "edges_per_s_incl_build": round(edge_inst / ((ms_per_step + build_ms) * 1e-3), 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
