"""Pins for the oracle's graph of a packed batch (oracle.build_batch_graph, CPU only).

A batch joined into one graph is the disjoint union of the per-sequence graphs, so everything is fixed by the
per-length oracle (pinned in test_oracle_graph.py / test_oracle_attention.py): attention over the joined graph
must give, row for row, what every sequence gives on its own graph, the table gradient must be the sum over
the sequences, and no edge may join two sequences.
"""
import numpy as np
import pytest

import oracle

CASES = [
    (8, 1, False, [8, 1, 5, 3]), (16, 2, False, [16, 9, 1, 0, 7]), (16, 3, True, [0, 0, 5]),
    (64, 2, False, [64, 1, 37, 17, 64, 2]), (64, 70, False, [33, 64, 50]), (128, 3, True, [100, 128, 2, 127]),
]


@pytest.mark.parametrize("n,k,causal,lengths", CASES)
def test_layout_counts_the_kept_nodes(n, k, causal, lengths):
    first, count, rows = oracle.batch_layout(n, lengths)
    row_of, b_of, node_of = oracle.batch_rows(n, lengths)
    # a sequence keeps exactly the nodes that have an edge in its own graph
    for b, length in enumerate(lengths):
        kept = np.flatnonzero(row_of[b] >= 0)
        if length >= 1:
            deg = np.diff(oracle.build_graph_len(n, length, k, causal).row_ptr)
            assert np.array_equal(kept, np.flatnonzero(deg > 0))
        else:
            assert kept.size == 0
    assert rows == sum(int((row_of[b] >= 0).sum()) for b in range(len(lengths)))
    # rows are a bijection onto (sequence, node) pairs, level-major: tokens first, sequence by sequence
    assert np.array_equal(row_of[b_of, node_of], np.arange(rows))
    T = int(sum(lengths))
    assert (node_of[:T] < n).all() and (node_of[T:] >= n).all()
    assert np.array_equal(b_of[:T], np.repeat(np.arange(len(lengths)), lengths))
    assert first[0, 0] == 0 and int(count.sum()) == rows


@pytest.mark.parametrize("n,k,causal,lengths", CASES)
def test_joined_graph_is_the_disjoint_union(n, k, causal, lengths):
    g = oracle.build_batch_graph(n, k, causal, lengths)
    _, b_of, node_of = oracle.batch_rows(n, lengths)
    assert g.num_nodes == len(b_of)
    assert g.num_edges == sum(oracle.build_graph_len(n, length, k, causal).num_edges for length in lengths if length >= 1)
    src = np.repeat(np.arange(g.num_nodes), np.diff(g.row_ptr))
    assert np.array_equal(b_of[src], b_of[g.col])                 # no edge between two sequences
    # every row lists what the sequence's own graph lists, translated back
    for r in range(g.num_nodes):
        own = oracle.build_graph_len(n, lengths[b_of[r]], k, causal)
        e0, e1 = own.row_ptr[node_of[r]], own.row_ptr[node_of[r] + 1]
        assert np.array_equal(node_of[g.col[g.row_ptr[r]:g.row_ptr[r + 1]]], own.col[e0:e1])
        assert np.array_equal(g.rel[g.row_ptr[r]:g.row_ptr[r + 1]], own.rel[e0:e1])


@pytest.mark.parametrize("n,k,causal,lengths", CASES)
def test_attention_over_the_joined_graph_equals_the_sequences_on_their_own(n, k, causal, lengths):
    H, D = 2, 16
    g = oracle.build_batch_graph(n, k, causal, lengths)
    _, b_of, node_of = oracle.batch_rows(n, lengths)
    rows = g.num_nodes
    rng = np.random.default_rng(n + k)
    Q, K, V, dO = (rng.standard_normal((1, H, rows, D)).astype(np.float32) for _ in range(4))
    Rel = (0.5 * rng.standard_normal((g.num_levels, g.rel_width, D))).astype(np.float32)
    out, lse, _ = oracle.attn_fwd(g, Q, K, V, Rel, 0.25)
    dQ, dK, dV, dRel, _ = oracle.attn_bwd(g, Q, K, V, Rel, dO, 0.25)

    live = [b for b, length in enumerate(lengths) if length >= 1]
    pos = {b: i for i, b in enumerate(live)}
    bi = np.array([pos[b] for b in b_of])
    padded = []
    for x in (Q, K, V, dO):
        p = np.zeros((len(live), H, 2 * n - 1, D), dtype=np.float32)
        p[bi, :, node_of] = np.transpose(x[0], (1, 0, 2))
        padded.append(p)
    ll = [lengths[b] for b in live]
    o, l, _ = oracle.attn_fwd_lengths(n, k, causal, ll, padded[0], padded[1], padded[2], Rel, 0.25)
    dq, dk, dv, dr = oracle.attn_bwd_lengths(n, k, causal, ll, padded[0], padded[1], padded[2], Rel, padded[3], 0.25)
    for got, want in ((out, o), (dQ, dq), (dK, dk), (dV, dv)):
        np.testing.assert_allclose(got[0], np.transpose(want[bi, :, node_of], (1, 0, 2)), rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse[0], np.transpose(l[bi, :, node_of], (1, 0)), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dRel, dr, rtol=0, atol=1e-11)


def test_a_batch_of_full_sequences_repeats_the_single_graph():
    n, k = 32, 2
    one = oracle.build_graph(n, k, False)
    g = oracle.build_batch_graph(n, k, False, [n])
    assert np.array_equal(g.row_ptr, one.row_ptr) and np.array_equal(g.col, one.col) and np.array_equal(g.rel, one.rel)
