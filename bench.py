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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
KERNEL_SOURCES = os.path.join(ROOT, "paper_1911_04070_amd", "csrc")


def kernel_source_hash():
    """sha256 over the sources of the graph and attention kernels (not the layer around them, whose kernels are not
    in that file): the counter figures in profiles/ belong to one build of the kernels."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(KERNEL_SOURCES)):
        if name.endswith((".h", ".hip")) and name != "bpt_layer.hip":
            with open(os.path.join(KERNEL_SOURCES, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per launch of every kernel of `workload` from profiles/hbm_traffic.txt (rocprofv3 FETCH_SIZE and
    WRITE_SIZE runs, scaled as that file says), with the hash of the kernel sources they were taken on.
    Returns ({kernel: (bytes read, bytes written, launches per step)}, sources hash or None)."""
    per_kernel, src, fetch_scale, write_scale = {}, None, 1.0, 1.0
    if not os.path.exists(TRAFFIC_FILE):
        return per_kernel, src
    with open(TRAFFIC_FILE) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "sources":
                src = t[1]
            elif t[0] == "scale":                       # scale FETCH_SIZE x  WRITE_SIZE y   (bytes per counted KiB / 1024)
                fetch_scale, write_scale = float(t[2]), float(t[4])
            elif t[0] == workload:                      # workload kernel FETCH_SIZE WRITE_SIZE launches_per_step
                per_kernel[t[1]] = (float(t[2]) * fetch_scale * 1024.0, float(t[3]) * write_scale * 1024.0, float(t[4]))
    return per_kernel, src


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
    ap.add_argument("--calibrate-gather-mib", type=int, default=0,
                    help="only run the library's calibration gather over this many MiB of 128-byte rows (10 times) and "
                         "exit: known traffic of the attention kernels' request shape for scaling the same counters")
    ap.add_argument("--zero-unkept", action="store_true",
                    help="workloads with sequences of different lengths: zero-fill the rows of nodes a sequence does not "
                         "keep (the default leaves them unwritten, bpt_shape_t.leave_unkept)")
    ap.add_argument("--bf16-grads", action="store_true",
                    help="dQ, dK, dV rounded to bf16 by the backward (bpt_shape_t.grad_dtype) instead of fp32")
    ap.add_argument("--memory", choices=("heads", "nodes", "qkvo"), default="heads",
                    help="heads: tensors in [B][H][N][D] memory; nodes: [B][N][H][D], what a projection of node rows writes; "
                         "qkvo: rows of [Q | K | V | out][H][D] and [dQ | dK | dV | dout][H][D], the graph layer's buffers "
                         "(gradients bf16)")
    ap.add_argument("--packed", action="store_true",
                    help="workloads with sequences of different lengths: one graph for the whole batch with rows only for "
                         "the nodes that exist (bpt_build_batch_graph) instead of the padded trees")
    ap.add_argument("--regions", type=int, default=5,
                    help="the timed steps are run as this many back-to-back regions (each synchronised on both sides); "
                         "ms_per_step is the median region, the spread is reported beside it")
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
    packed = args.packed and bool(w.length_mix)   # one graph for the batch: E is [1][tokens of all sequences][d]
    g = bpt.bpt_build_batch_graph(w.n, w.k, w.causal, make_lengths(w)) if packed else bpt.bpt_build_graph(w.n, w.k, w.causal)
    B = 1 if packed else w.B
    gen = torch.Generator(device="cuda").manual_seed(1911 + w.index)
    rnd = lambda *shape, s=1.0: (s * torch.randn(*shape, device="cuda", generator=gen))
    E = rnd(B, g.n_tokens, d).to(torch.bfloat16)
    rels = [rnd(g.num_levels, g.rel_width, w.D, s=0.02).to(torch.bfloat16) for _ in range(layers)]
    params = [layer_params(torch, rnd, d, d_ff) for _ in range(layers)]
    lens_d = torch.from_numpy(make_lengths(w)).cuda() if w.length_mix and not packed else None
    tokens_out = bool(w.causal)
    d_root = None if tokens_out else rnd(w.B, d).to(torch.bfloat16)
    d_tokens = rnd(B, g.n_tokens, d).to(torch.bfloat16) if tokens_out else None
    fws, bws = bpt.stack_workspace_bytes(g, B, w.H, d_ff, layers)
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
    rows = B * g.num_nodes
    tokens = int(make_lengths(w).sum()) if w.length_mix else w.B * w.n   # the tokens that exist, not the padding
    flops = layers * 3 * 2.0 * rows * (4 * d * d + 2 * d * d_ff)
    print(json.dumps({
        "metric": "BPT graph update fwd+bwd tokens/sec", "value": round(tokens / (ms * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "dtype": "bf16", "data": "synthetic", "vs_baseline": None, "forward_ms": round(ms_fwd, 4),
        "config": {"workload": "%s+%d layers%s" % (w.name, layers, "+packed" if packed else ""), "n": w.n, "k": w.k, "causal": w.causal, "batch": w.B,
                   "heads": w.H, "d_model": d, "d_ff": d_ff, "layers": layers, "node_rows": rows, "tokens": tokens,
                   "output": "tokens" if tokens_out else "root"},
        "dense_TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1),
        "workspace_GB": round((fws + bws) / 1e9, 2),
    }), flush=True)


def bench_packed(args, w, bpt, torch, np):
    """Attention forward + backward of a workload whose sequences have different lengths, on ONE graph for the batch
    with rows only for the nodes that exist (bpt_build_batch_graph): tensors [1, H, rows, 64], no padding anywhere."""
    from paper_1911_04070_amd.workloads import make_lengths
    lengths = make_lengths(w)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g = bpt.bpt_build_batch_graph(w.n, w.k, w.causal, lengths)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) * 1e3
    gen = torch.Generator(device="cuda").manual_seed(1911 + w.index)
    rnd = lambda *shape, s=1.0: (s * torch.randn(*shape, device="cuda", generator=gen)).to(tdt)
    Q, K, V, dO = (rnd(1, w.H, g.num_nodes, w.D) for _ in range(4))
    R = rnd(g.num_levels, g.rel_width, w.D, s=0.02)
    out = torch.empty_like(Q)
    lse = torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty(Q.shape, dtype=torch.float32, device="cuda") for _ in range(3)) + (
        torch.empty(R.shape, dtype=torch.float32, device="cuda"),)
    fws, bws = bpt.workspace_bytes(g, Q, w.scale)
    ws_f = torch.empty(max(fws, 256), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(bws, 256), dtype=torch.uint8, device="cuda")

    def step():
        bpt.bpt_attn_fwd(g, Q, K, V, R, scale=w.scale, out=out, lse=lse, workspace=ws_f)
        if w.backward:
            bpt.bpt_attn_bwd(g, Q, K, V, R, lse, dO, scale=w.scale, grads=grads, workspace=ws_b)

    for _ in range(args.warmup):
        step()
    regions = max(1, min(args.regions, args.steps))
    sizes = [args.steps // regions + (1 if r < args.steps % regions else 0) for r in range(regions)]
    region_ms = []
    torch.cuda.synchronize()
    for count in sizes:
        t0 = time.perf_counter()
        for _ in range(count):
            step()
        torch.cuda.synchronize()
        region_ms.append((time.perf_counter() - t0) * 1e3 / count)
    ms = float(np.median(region_ms))
    bpt.bpt_profile_enable(True)
    for _ in range(10):
        step()
    torch.cuda.synchronize()
    prof = bpt.bpt_profile_report()
    bpt.bpt_profile_enable(False)
    edge_inst = w.H * g.num_edges
    es = 2 if w.dtype == "bf16" else 4
    padded_rows = w.B * (2 * w.n - 1)
    print(json.dumps({
        "metric": "BPT graph-attention fwd+bwd edges/sec" if w.backward else "BPT graph-attention fwd edges/sec",
        "value": round(edge_inst / (ms * 1e-3), 1), "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "ms_per_step_min": round(min(region_ms), 4), "ms_per_step_max": round(max(region_ms), 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "+packed", "n": w.n, "k": w.k, "causal": w.causal, "batch": w.B, "heads": w.H,
                   "layout": "one graph for the batch, rows of kept nodes only", "rows": g.num_nodes,
                   "padded_rows": padded_rows, "tokens": g.n_tokens, "edges_per_head": g.num_edges,
                   "lengths": [int(v) for v in lengths]},
        "graph_build_ms": round(build_ms, 3),
        "tensor_MB": {"packed_per_tensor": round(w.H * g.num_nodes * w.D * es / 1e6, 2),
                      "padded_per_tensor": round(w.H * padded_rows * w.D * es / 1e6, 2),
                      "workspace": round((fws + bws) / 1e6, 2)},
        "kernel_ms": {name: round(total / calls, 5) for name, (calls, total) in prof.items()},
    }), flush=True)


def bench_layer(args, w, bpt, torch, np):
    """Forward + backward of one graph layer (Sec. 3.3) on the workload's shape: d = heads * 64, d_ff = 4 d, random
    bf16 weights."""
    from paper_1911_04070_amd.workloads import make_lengths
    d, d_ff = w.H * w.D, 4 * w.H * w.D
    packed = args.packed and bool(w.length_mix)   # one graph for the batch, rows of kept nodes only: X is [1][rows][d]
    g = bpt.bpt_build_batch_graph(w.n, w.k, w.causal, make_lengths(w)) if packed else bpt.bpt_build_graph(w.n, w.k, w.causal)
    B = 1 if packed else w.B
    gen = torch.Generator(device="cuda").manual_seed(1911 + w.index)
    rnd = lambda *shape, s=1.0: (s * torch.randn(*shape, device="cuda", generator=gen))
    X = rnd(B, g.num_nodes, d).to(torch.bfloat16)
    X[:, g.n_tokens:] = 0                                     # span nodes start from zero
    R = rnd(g.num_levels, g.rel_width, w.D, s=0.02).to(torch.bfloat16)
    p = layer_params(torch, rnd, d, d_ff)
    lens_d = torch.from_numpy(make_lengths(w)).cuda() if w.length_mix and not packed else None
    Y = torch.empty_like(X)
    dY = rnd(B, g.num_nodes, d).to(torch.bfloat16)
    dX = torch.empty_like(X)
    d_rel = torch.empty(R.shape, dtype=torch.float32, device="cuda")
    grads = {"d" + k_: torch.empty(v.shape, dtype=torch.float32, device="cuda") for k_, v in p.items()}
    fws, bws = bpt.layer_workspace_bytes(g, B, w.H, d_ff)
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
    rows = B * g.num_nodes
    flops = 3 * 2.0 * rows * (4 * d * d + 2 * d * d_ff)       # the backward has two products per forward product
    print(json.dumps({
        "metric": "BPT graph layer fwd+bwd node rows/sec", "value": round(rows / (ms * 1e-3), 1), "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "dtype": "bf16", "data": "synthetic", "vs_baseline": None, "forward_ms": round(ms_fwd, 4),
        "config": {"workload": w.name + "+layer" + ("+packed" if packed else ""), "n": w.n, "k": w.k, "causal": w.causal, "batch": w.B,
                   "heads": w.H, "d_model": d, "d_ff": d_ff, "node_rows": rows, "workspace_MB": round((fws + bws) / 1e6, 1)},
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
    if args.calibrate_gather_mib > 0:
        # rows of 128 bytes of a tensor far larger than the caches, each read once through a random permutation
        from paper_1911_04070_amd import binding as bpt
        torch.cuda.set_device(0)
        rows = (args.calibrate_gather_mib << 20) // 128
        src = torch.ones(rows * 128, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        perm = torch.from_numpy(np.random.Generator(np.random.PCG64(1911)).permutation(rows).astype(np.int32)).cuda()
        for _ in range(10):
            bpt.bpt_calibrate_gather(src, perm, dst)
        torch.cuda.synchronize()
        print(json.dumps({"gather_mib": args.calibrate_gather_mib, "rows": rows, "launches": 10,
                          "bytes_read_per_launch": rows * 132, "bytes_written_per_launch": rows * 128}), flush=True)
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
    if args.packed:
        if not w.length_mix:
            sys.exit("--packed is for the workloads with sequences of different lengths (lm_lengths, cls_lengths)")
        return bench_packed(args, w, bpt, torch, np)
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
    out = None
    if args.memory == "nodes":   # the same values, the heads of a node side by side in memory
        Q, K, V, dO = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (Q, K, V, dO))
    elif args.memory == "qkvo":
        args.bf16_grads = True
        rows = torch.empty((w.B, Q.shape[2], 4, w.H, w.D), dtype=tdt, device="cuda")
        grows = torch.empty_like(rows)
        for slot, t in enumerate((Q, K, V)):
            rows[:, :, slot] = t.permute(0, 2, 1, 3)
        grows[:, :, 3] = dO.permute(0, 2, 1, 3)
        Q, K, V, out = (rows[:, :, slot].permute(0, 2, 1, 3) for slot in range(4))
        dO = grows[:, :, 3].permute(0, 2, 1, 3)
    if out is None:
        out = torch.empty_like(Q)
    lse = torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda")
    if args.bf16_grads and w.dtype != "bf16":
        sys.exit("--bf16-grads is for the bf16 workloads")
    gdt = torch.bfloat16 if args.bf16_grads else torch.float32
    grads = (tuple(grows[:, :, slot].permute(0, 2, 1, 3) for slot in range(3)) if args.memory == "qkvo" else
             tuple(torch.empty_like(Q, dtype=gdt) for _ in range(3))) + (
        torch.empty(R.shape, dtype=torch.float32, device="cuda"),)
    fws, bws = bpt.workspace_bytes(g, Q, w.scale)
    ws_f = torch.empty(max(fws, 256), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(bws, 256), dtype=torch.uint8, device="cuda")

    drop = (args.dropout, 1911) if args.dropout > 0 else None
    leave = lengths is not None and not args.zero_unkept

    def step():
        bpt.bpt_attn_fwd(g, Q, K, V, R, scale=w.scale, out=out, lse=lse, workspace=ws_f, seq_len=lens_d, dropout=drop,
                         leave_unkept=leave)
        if w.backward:
            bpt.bpt_attn_bwd(g, Q, K, V, R, lse, dO, scale=w.scale, grads=grads, workspace=ws_b, seq_len=lens_d,
                             dropout=drop, leave_unkept=leave)

    for _ in range(args.warmup):
        step()
    # exactly --steps timed steps, as back-to-back regions with a synchronisation on both sides of each
    regions = max(1, min(args.regions, args.steps))
    sizes = [args.steps // regions + (1 if r < args.steps % regions else 0) for r in range(regions)]
    region_ms = []
    torch.cuda.synchronize()
    t_all = time.perf_counter()
    for count in sizes:
        t0 = time.perf_counter()
        for _ in range(count):
            step()
        torch.cuda.synchronize()
        region_ms.append((time.perf_counter() - t0) * 1e3 / count)
    ms_mean = (time.perf_counter() - t_all) * 1e3 / args.steps
    ms_per_step = float(np.median(region_ms))

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
    stage_ms = {"fwd": timed(lambda: bpt.bpt_attn_fwd(g, Q, K, V, R, scale=w.scale, out=out, lse=lse, workspace=ws_f,
                                                      seq_len=lens_d, dropout=drop, leave_unkept=leave), reps)}
    if w.backward:
        stage_ms["bwd_query_side"] = timed(
            lambda: bpt.bpt_attn_bwd_query_side(g, Q, K, V, R, lse, dO, grads[0], grads[3], ws_b, scale=w.scale,
                                                seq_len=lens_d, dropout=drop, leave_unkept=leave), reps)
        stage_ms["bwd_key_side"] = timed(
            lambda: bpt.bpt_attn_bwd_key_side(g, Q, K, V, R, lse, dO, grads[1], grads[2], ws_b, scale=w.scale,
                                              seq_len=lens_d, dropout=drop, leave_unkept=leave), reps)

    # the same step with nothing of its tensors left in the caches (the 256 MB memory-side cache included): 1 GiB is
    # overwritten before every step, events around the step alone.  In the timed loop above the step's inputs are
    # re-read every step and partly stay in that cache; behind other work (a layer's GEMMs) they do not.
    scrub = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cold = []
    for rep in range(10):
        scrub.fill_(rep)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        step()
        b.record()
        torch.cuda.synchronize()
        cold.append(a.elapsed_time(b))
    cold_ms = float(np.median(cold))
    del scrub

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

    # ---- roofline of the dominant kernel --------------------------------------------------------------------
    # Two byte counts per launch, never conflated:
    #  * gathered bytes: one key row + one value row (or one query row + one dout row) per edge-instance the kernel
    #    handles, 256 B in bf16 -- the method's per-edge work at the load level.  The tile kernels fetch a row
    #    once per 16-row tile and re-use it on chip, so this is NOT a lower bound on memory traffic;
    #  * compulsory bytes: every row the kernel must read or write, once -- a lower bound on its HBM traffic whatever
    #    the blocking, so compulsory bytes / time / HBM peak is a fraction of a roof (<= 1 by construction).
    bh = w.B * w.H
    row_ptr_h, col_h, _ = g.csr_to_host()
    e_tok_graph = int(row_ptr_h[w.n])
    if lengths is None:
        tok_inst = e_tok_graph * bh
        fill = 1.0
    else:   # every level above the tokens holds each token of a sequence once
        tok_inst = edge_inst - w.H * int(lengths.sum()) * (g.num_levels - 1)
        fill = float(lengths.sum()) / float(w.B * w.n)
    span_inst = edge_inst - tok_inst
    gather = 256.0 * bytes_scale
    alg_bytes = {
        "fwd_tile_kernel": gather * tok_inst, "bwd_q_tile_kernel": gather * tok_inst,
        "fwd_span_tile_kernel": gather * span_inst, "bwd_q_span_tile_kernel": gather * span_inst,
        "bwd_kv_tile_kernel": gather * edge_inst, "bwd_kv_chain_kernel": gather * edge_inst, "bwd_kv_kernel": gather * edge_inst,
    }
    # the gather kernels take whatever rows the tile kernels of this launch did not
    alg_bytes["fwd_kernel"] = gather * (edge_inst - (tok_inst if "fwd_tile_kernel" in kernel_ms else 0) - (
        span_inst if "fwd_span_tile_kernel" in kernel_ms else 0))
    alg_bytes["bwd_q_kernel"] = gather * (edge_inst - (tok_inst if "bwd_q_tile_kernel" in kernel_ms else 0) - (
        span_inst if "bwd_q_span_tile_kernel" in kernel_ms else 0))
    esz = 2 if w.dtype == "bf16" else 4
    gsz = 2 if args.bf16_grads else 4
    row, frow = w.D * esz, w.D * gsz                          # a row of a tensor; a row of a gradient (fp32 unless --bf16-grads)
    # node rows per (batch, head), scaled by the fill of a batch of different lengths (the kept nodes)
    n_tok, n_span, n_all = w.n * fill, (w.n - 1) * fill, g.num_nodes * fill
    keys_tok = len(np.unique(col_h[:e_tok_graph])) * fill     # nodes some token row attends to
    keyed = len(np.unique(col_h)) * fill                      # nodes with at least one in-edge
    compulsory_kernel = {
        # Q rows, K and V rows, out rows, lse
        "fwd_tile_kernel": bh * (n_tok * row + keys_tok * 2 * row + n_tok * row + n_tok * 4),
        "fwd_span_tile_kernel": bh * (n_span * row + n_tok * 2 * row + n_span * row + n_span * 4),
        # Q and dout rows, K and V rows, lse; dQ rows (fp32) and (lse, delta) out
        "bwd_q_tile_kernel": bh * (n_tok * 2 * row + keys_tok * 2 * row + n_tok * 4 + n_tok * frow + n_tok * 8),
        "bwd_q_span_tile_kernel": bh * (n_span * 2 * row + n_tok * 2 * row + n_span * 4 + n_span * frow + n_span * 8),
        # Q and dout rows of every query node with (lse, delta), K and V rows of the keys; dK and dV rows (fp32) out
        "bwd_kv_tile_kernel": bh * (n_all * 2 * row + n_all * 8 + keyed * 2 * row + keyed * 2 * frow),
    }
    compulsory_kernel["bwd_kv_kernel"] = compulsory_kernel["bwd_kv_chain_kernel"] = compulsory_kernel["bwd_kv_tile_kernel"]
    rows_fwd = n_all - (n_tok if "fwd_tile_kernel" in kernel_ms else 0) - (n_span if "fwd_span_tile_kernel" in kernel_ms else 0)
    rows_bq = n_all - (n_tok if "bwd_q_tile_kernel" in kernel_ms else 0) - (n_span if "bwd_q_span_tile_kernel" in kernel_ms else 0)
    keys_of = lambda rows: keyed if rows > n_span else n_tok   # all rows: every keyed node; span rows only: the tokens
    compulsory_kernel["fwd_kernel"] = bh * (rows_fwd * 2 * row + keys_of(rows_fwd) * 2 * row + rows_fwd * 4)
    compulsory_kernel["bwd_q_kernel"] = bh * (rows_bq * 2 * row + keys_of(rows_bq) * 2 * row + rows_bq * (12 + frow))
    main = {k: v for k, v in kernel_ms.items() if k in alg_bytes}
    dominant = max(main, key=main.get)
    dom_s = kernel_ms[dominant] * 1e-3
    achieved = compulsory_kernel[dominant] / dom_s / 1e9
    step_alg_bytes = gather * (3 if w.backward else 1) * edge_inst
    tensor = bh * n_all * w.D
    # the tensors of the boundary, each moved once per stage that needs it: the forward reads Q, K, V and
    # writes out, lse; the backward reads Q, K, V, dout, lse and writes dQ, dK, dV (fp32) -- no workspace traffic
    compulsory = tensor * esz * 4 + bh * n_all * 4
    if w.backward:
        compulsory += tensor * esz * 4 + bh * n_all * 4 + 3 * tensor * gsz
    # measured HBM traffic (rocprofv3 counters, profiles/hbm_traffic.txt) -- only if taken on these kernel sources
    per_kernel, measured_on = measured_traffic(w.name)
    sources = kernel_source_hash()
    fresh = bool(per_kernel) and measured_on == sources and args.dropout == 0 and not args.bf16_grads and args.memory == "heads"
    traffic = step_traffic = None
    if fresh:
        if dominant in per_kernel:
            traffic = int(per_kernel[dominant][0] + per_kernel[dominant][1])
        step_traffic = int(sum((r + wr) * launches for r, wr, launches in per_kernel.values()))
    # matrix-core work of the dominant kernel if its tiles were full: 2 * 64 flops per edge-instance and product
    products = {"fwd_tile_kernel": 3, "fwd_span_tile_kernel": 2, "bwd_q_tile_kernel": 6, "bwd_q_span_tile_kernel": 4,
                "bwd_kv_tile_kernel": 5, "bwd_kv_chain_kernel": 5}.get(dominant)
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "bytes": "compulsory: every row the kernel has to read or write, once (a lower bound on its HBM traffic)",
        "compulsory_bytes": int(compulsory_kernel[dominant]),
        "traffic": traffic,
        "wasted_traffic_ratio": round(traffic / compulsory_kernel[dominant], 3) if traffic else None,
        "traffic_GBs": round(traffic / dom_s / 1e9, 1) if traffic else None,
        "traffic_frac_of_peak": round(traffic / dom_s / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
        "traffic_source": ("profiles/hbm_traffic.txt" if fresh else
                           "none for this workload" if not per_kernel else
                           "stale: profiles/hbm_traffic.txt was taken on kernel sources %s, these are %s" % (measured_on, sources)
                           if measured_on != sources else "not measured with these options"),
        "launch_ms": round(kernel_ms[dominant], 4),
        "limiter": "latency of the chain row gather -> LDS -> matrix products -> exp -> matrix products inside a "
                   "wavefront at two wavefronts per SIMD (counters in profiles/): neither HBM nor the matrix cores are "
                   "saturated; hbm is the nearer of the two roofs",
        "mfma_frac_if_tiles_were_full": (round(products * 128.0 * (alg_bytes[dominant] / gather) / dom_s / 1e12 /
                                               MFMA_BF16_PEAK_TFLOPS, 4) if products and w.dtype == "bf16" else None),
        "gathered_bytes_per_edge_instance": gather,
        "gathered_GBs": round(alg_bytes[dominant] / dom_s / 1e9, 1),
        "device_copy_GBs": round(copy_gbs, 1),
        "kernel_ms": {k: round(v, 4) for k, v in sorted(kernel_ms.items(), key=lambda kv: -kv[1])},
        "kernel_compulsory_frac_of_hbm_peak": {k: round(compulsory_kernel[k] / (v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                                               for k, v in sorted(main.items(), key=lambda kv: -kv[1])},
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "step_ms_behind_1GiB_of_other_writes": round(cold_ms, 4),
        "step_gathered_GBs": round(step_alg_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_compulsory_bytes": int(compulsory),
        "step_compulsory_frac_of_hbm_peak": round(compulsory / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "step_traffic": step_traffic,
        "step_traffic_frac_of_hbm_peak": (round(step_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                                          if step_traffic else None),
        "step_wasted_traffic_ratio": round(step_traffic / compulsory, 3) if step_traffic else None,
        "target_50pct_of_hbm_peak_met": (bool(step_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS >= 0.5)
                                         if step_traffic else None),
    }

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        og = oracle.build_graph(w.n, w.k, w.causal)
        passes, dt, used = 0, 0.0, 1
        while passes < 1 or (dt < 10.0 and passes < 50):     # about ten seconds of wall time on all cores
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
        "ms_per_step_min": round(min(region_ms), 4), "ms_per_step_max": round(max(region_ms), 4),
        "ms_per_step_mean": round(ms_mean, 4), "timed_regions": sizes,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "k": w.k, "causal": w.causal, "batch": w.B, "heads": w.H,
                   "head_dim": w.D, "nodes": g.num_nodes, "edges": g.num_edges, "edge_instances": edge_inst,
                   "backward": w.backward, "dropout": args.dropout, "gradients": "bf16" if args.bf16_grads else "fp32",
                   "memory": {"heads": "[B][H][N][D]", "nodes": "[B][N][H][D]", "qkvo": "[B][N][Q|K|V|out][H][D]"}[args.memory], "unkept_rows": ("unwritten" if leave else "zero-filled") if lengths is not None else None,
                   "lengths": ([int(v) for v in lengths] if lengths is not None else None)},
        "graph_build_ms": round(build_ms, 3),
        "edges_per_s_incl_build": round(edge_inst / ((ms_per_step + build_ms) * 1e-3), 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
