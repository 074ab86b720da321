"""CPU oracle for BP-Transformer graph self-attention (test infrastructure only).

This package wraps ``bpt_oracle.c`` -- a plain double-precision restatement of
the paper's graph construction (Sec. 3.2), tree relative positions (Sec. 3.4)
and graph self-attention (Sec. 3.1 eq. 6, Sec. 3.4 eq. 8) with its gradient.
It exists to check the GPU library and to time a CPU baseline.  It shares no
code with the HIP path and is never imported by the product package; only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bpt_oracle.c")
_LIB = os.path.join(_HERE, "libbpt_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over batch*heads / rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i32, i64, f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        p = ctypes.c_void_p
        L.bpto_num_levels.restype = i32
        L.bpto_num_levels.argtypes = [i32]
        L.bpto_level_offset.restype = i64
        L.bpto_level_offset.argtypes = [i32, i32]
        L.bpto_rel_width.restype = i32
        L.bpto_rel_width.argtypes = [i32]
        L.bpto_count_edges.restype = i64
        L.bpto_count_edges.argtypes = [i32, i32, i32, p]
        L.bpto_build_graph.restype = i32
        L.bpto_build_graph.argtypes = [i32, i32, i32, p, p, p]
        L.bpto_count_edges_len.restype = i64
        L.bpto_count_edges_len.argtypes = [i32, i32, i32, i32, p]
        L.bpto_build_graph_len.restype = i32
        L.bpto_build_graph_len.argtypes = [i32, i32, i32, i32, p, p, p]
        L.bpto_transpose.restype = None
        L.bpto_transpose.argtypes = [i32, p, p, p, p, p]
        L.bpto_attn_fwd.restype = i32
        L.bpto_attn_fwd.argtypes = [i32, p, p, p, i32, i32, p, p, p, p, f64, p, p, i32, f64, ctypes.c_uint32, i32]
        L.bpto_attn_bwd.restype = i32
        L.bpto_attn_bwd.argtypes = [i32, p, p, p, i32, i32, i32, p, p, p, p, p, f64, p, p, p, p, i32, f64, ctypes.c_uint32, i32]
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class Graph:
    """Binary-partition graph in CSR by query node (Sec. 3.2)."""
    n: int
    k: int
    causal: bool
    num_nodes: int          # 2n-1
    num_levels: int         # log2(n)+1, tokens are level 0
    rel_width: int          # W = 2(k+1)+1 slots per level in the r table
    row_ptr: np.ndarray     # int32 [num_nodes+1]
    col: np.ndarray         # int32 [E]  key node id
    rel: np.ndarray         # int32 [E]  level*W + (offset + k+1)

    @property
    def num_edges(self) -> int:
        return int(self.row_ptr[-1])

    def level_offset(self, level: int) -> int:
        return int(_load().bpto_level_offset(self.n, level))


def num_levels(n: int) -> int:
    return int(_load().bpto_num_levels(n))


def level_offset(n: int, level: int) -> int:
    return int(_load().bpto_level_offset(n, level))


def degrees(n: int, k: int, causal: bool) -> np.ndarray:
    L = _load()
    deg = np.zeros(2 * n - 1, dtype=np.int64)
    E = L.bpto_count_edges(n, k, int(causal), _ptr(deg))
    if E < 0:
        raise ValueError("n must be a power of two >= 2 and k >= 1")
    return deg


def build_graph(n: int, k: int, causal: bool) -> Graph:
    L = _load()
    E = L.bpto_count_edges(n, k, int(causal), None)
    if E < 0:
        raise ValueError("n must be a power of two >= 2 and k >= 1")
    N = 2 * n - 1
    row_ptr = np.zeros(N + 1, dtype=np.int32)
    col = np.zeros(E, dtype=np.int32)
    rel = np.zeros(E, dtype=np.int32)
    rc = L.bpto_build_graph(n, k, int(causal), _ptr(row_ptr), _ptr(col), _ptr(rel))
    if rc != 0:
        raise RuntimeError("oracle graph build failed (edge count overflow?)")
    return Graph(n, k, bool(causal), N, num_levels(n), int(L.bpto_rel_width(k)), row_ptr, col, rel)


def build_graph_len(n: int, length: int, k: int, causal: bool) -> Graph:
    """Graph of a sequence of ``length`` <= n tokens on the node ids of the tree over n:
    only nodes that hold a token are kept, the other rows are empty."""
    L = _load()
    E = L.bpto_count_edges_len(n, length, k, int(causal), None)
    if E < 0:
        raise ValueError("n must be a power of two >= 2, k >= 1 and 1 <= length <= n")
    N = 2 * n - 1
    row_ptr = np.zeros(N + 1, dtype=np.int32)
    col = np.zeros(E, dtype=np.int32)
    rel = np.zeros(E, dtype=np.int32)
    rc = L.bpto_build_graph_len(n, length, k, int(causal), _ptr(row_ptr), _ptr(col), _ptr(rel))
    if rc != 0:
        raise RuntimeError("oracle graph build failed")
    return Graph(n, k, bool(causal), N, num_levels(n), int(L.bpto_rel_width(k)), row_ptr, col, rel)


def transpose(g: Graph):
    """(t_ptr, t_src, t_eid): for each key node its edges in ascending edge index."""
    L = _load()
    t_ptr = np.zeros(g.num_nodes + 1, dtype=np.int32)
    t_src = np.zeros(g.num_edges, dtype=np.int32)
    t_eid = np.zeros(g.num_edges, dtype=np.int32)
    L.bpto_transpose(g.num_nodes, _ptr(g.row_ptr), _ptr(g.col), _ptr(t_ptr), _ptr(t_src), _ptr(t_eid))
    return t_ptr, t_src, t_eid


def _as_bhnd(x: np.ndarray, N: int):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim != 4 or x.shape[2] != N:
        raise ValueError("expected [B,H,N,D] with N=%d, got %r" % (N, x.shape))
    return x


def attn_fwd(g: Graph, Q, K, V, Rel, scale: float, threads: int = 0, dropout=0.0, seed=0, bh0=0):
    """Eq. (8) per node in float64.  Q,K,V: [B,H,N,D]; Rel: [levels,W,D].  dropout, seed: inverted dropout on the
    attention weights with the counter-based mask of the C source; bh0: index of this call's first (batch, head).

    Returns (out [B,H,N,D] f64, lse [B,H,N] f64, threads_used)."""
    L = _load()
    Q = _as_bhnd(Q, g.num_nodes)
    K = _as_bhnd(K, g.num_nodes)
    V = _as_bhnd(V, g.num_nodes)
    B, H, N, D = Q.shape
    Rel = np.ascontiguousarray(Rel, dtype=np.float32)
    assert Rel.shape == (g.num_levels, g.rel_width, D), Rel.shape
    out = np.zeros((B, H, N, D), dtype=np.float64)
    lse = np.zeros((B, H, N), dtype=np.float64)
    used = L.bpto_attn_fwd(N, _ptr(g.row_ptr), _ptr(g.col), _ptr(g.rel), B * H, D, _ptr(Q), _ptr(K),
                           _ptr(V), _ptr(Rel), float(scale), _ptr(out), _ptr(lse), int(threads), float(dropout),
                           int(seed) & 0xFFFFFFFF, int(bh0))
    return out, lse, int(used)


def attn_bwd(g: Graph, Q, K, V, Rel, dO, scale: float, threads: int = 0, dropout=0.0, seed=0, bh0=0):
    """Gradient of eq. (8) in float64.  Returns (dQ, dK, dV, dRel, threads_used)."""
    L = _load()
    Q = _as_bhnd(Q, g.num_nodes)
    K = _as_bhnd(K, g.num_nodes)
    V = _as_bhnd(V, g.num_nodes)
    dO = _as_bhnd(dO, g.num_nodes)
    B, H, N, D = Q.shape
    Rel = np.ascontiguousarray(Rel, dtype=np.float32)
    assert Rel.shape == (g.num_levels, g.rel_width, D), Rel.shape
    dQ = np.zeros((B, H, N, D), dtype=np.float64)
    dK = np.zeros_like(dQ)
    dV = np.zeros_like(dQ)
    dRel = np.zeros((g.num_levels, g.rel_width, D), dtype=np.float64)
    used = L.bpto_attn_bwd(N, _ptr(g.row_ptr), _ptr(g.col), _ptr(g.rel), B * H, D,
                           g.num_levels * g.rel_width, _ptr(Q), _ptr(K), _ptr(V), _ptr(Rel), _ptr(dO),
                           float(scale), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dRel), int(threads), float(dropout),
                           int(seed) & 0xFFFFFFFF, int(bh0))
    return dQ, dK, dV, dRel, int(used)


def attn_fwd_lengths(n, k, causal, lengths, Q, K, V, Rel, scale: float, threads: int = 0, dropout=0.0, seed=0):
    """Forward of a batch whose b-th sequence has lengths[b] tokens: every batch entry runs
    on the graph of its own length.  Returns (out, lse, edges) with edges = edge count of
    the whole batch per head."""
    out = np.zeros(np.shape(Q), dtype=np.float64)
    lse = np.zeros(np.shape(Q)[:3], dtype=np.float64)
    edges = 0
    for b, length in enumerate(lengths):
        g = build_graph_len(n, int(length), k, causal)
        edges += g.num_edges
        out[b:b + 1], lse[b:b + 1], _ = attn_fwd(g, Q[b:b + 1], K[b:b + 1], V[b:b + 1], Rel, scale, threads, dropout, seed,
                                                 b * np.shape(Q)[1])
    return out, lse, edges


def attn_bwd_lengths(n, k, causal, lengths, Q, K, V, Rel, dO, scale: float, threads: int = 0, dropout=0.0, seed=0):
    """Gradient of a batch of sequences of different lengths; dRel is summed over the batch."""
    dQ = np.zeros(np.shape(Q), dtype=np.float64)
    dK = np.zeros_like(dQ)
    dV = np.zeros_like(dQ)
    dRel = None
    for b, length in enumerate(lengths):
        g = build_graph_len(n, int(length), k, causal)
        q, kk, v, r, _ = attn_bwd(g, Q[b:b + 1], K[b:b + 1], V[b:b + 1], Rel, dO[b:b + 1], scale, threads, dropout, seed,
                                  b * np.shape(Q)[1])
        dQ[b:b + 1], dK[b:b + 1], dV[b:b + 1] = q, kk, v
        dRel = r if dRel is None else dRel + r
    return dQ, dK, dV, dRel


def batch_layout(n: int, lengths):
    """Rows of a batch of sequences joined into one graph, only kept nodes getting a row: level-major over the
    batch (all tokens first, sequence by sequence, then the level-1 nodes, ...).  Level l of a sequence of
    len tokens keeps ceil(len / 2^l) nodes.  Returns (first_row[l][b], row_count[l][b], rows)."""
    L = num_levels(n)
    first = np.zeros((L, len(lengths)), dtype=np.int64)
    count = np.zeros((L, len(lengths)), dtype=np.int64)
    row = 0
    for l in range(L):
        for b, length in enumerate(lengths):
            count[l, b] = -(-int(length) // (1 << l))
            first[l, b] = row
            row += int(count[l, b])
    return first, count, row


def batch_rows(n: int, lengths):
    """(row_of[b][node of the tree over n] or -1, sequence of every row, tree node of every row) of batch_layout."""
    first, count, rows = batch_layout(n, lengths)
    row_of = -np.ones((len(lengths), 2 * n - 1), dtype=np.int64)
    b_of = np.zeros(rows, dtype=np.int64)
    node_of = np.zeros(rows, dtype=np.int64)
    for l in range(first.shape[0]):
        off = level_offset(n, l)
        for b in range(len(lengths)):
            c, r0 = int(count[l, b]), int(first[l, b])
            row_of[b, off:off + c] = r0 + np.arange(c)
            b_of[r0:r0 + c] = b
            node_of[r0:r0 + c] = off + np.arange(c)
    return row_of, b_of, node_of


def build_batch_graph(n: int, k: int, causal: bool, lengths) -> Graph:
    """The graphs of a batch of sequences (build_graph_len of every length, Sec. 3.2 on the kept nodes) joined
    into one graph over the rows of batch_layout: the disjoint union, every row keeping its edges in their
    order with the key nodes renumbered.  (The paper batches the graphs of its sentences in the same way,
    Sec. 4.1 and the appendix on implementation details.)  Graph.num_nodes is the row count."""
    row_of, b_of, node_of = batch_rows(n, lengths)
    rows = len(b_of)
    per = [build_graph_len(n, int(length), k, causal) if length >= 1 else None for length in lengths]
    row_ptr = np.zeros(rows + 1, dtype=np.int32)
    cols, rels = [np.zeros(0, dtype=np.int32)], [np.zeros(0, dtype=np.int32)]
    for r in range(rows):
        g, u = per[b_of[r]], node_of[r]
        e0, e1 = int(g.row_ptr[u]), int(g.row_ptr[u + 1])
        c = row_of[b_of[r], g.col[e0:e1]]
        if e1 <= e0 or (c < 0).any():
            raise RuntimeError("a kept node without edges, or an edge to a node that is not kept")
        cols.append(c.astype(np.int32))
        rels.append(g.rel[e0:e1].astype(np.int32))
        row_ptr[r + 1] = row_ptr[r] + (e1 - e0)
    return Graph(n, k, bool(causal), rows, num_levels(n), int(_load().bpto_rel_width(k)), row_ptr,
                 np.concatenate(cols), np.concatenate(rels))
