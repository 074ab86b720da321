"""Pins for the oracle's graph builder (CPU only).

Every check here rests on something other than the builder itself: closed
forms and invariants the paper states (Sec. 3.2), an exhaustive declarative
search over tilings, and a hand-derived example.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

SMALL = [(n, k, c) for n in (2, 4, 8, 16, 32) for k in (1, 2, 3, 4, 5, 40) for c in (False, True)]
MEDIUM = [(64, 1, False), (64, 3, True), (128, 4, False), (256, 2, True), (512, 4, False), (1024, 8, True)]


def node_span(n, node):
    """(level, index, first token, one-past-last token) of a node id, from the
    level-major numbering: level l holds n/2^l nodes."""
    level, base, cnt = 0, 0, n
    while node >= base + cnt:
        base += cnt
        cnt //= 2
        level += 1
    m = node - base
    return level, m, m << level, (m + 1) << level


def unpack(g, r):
    level, slot = divmod(int(r), g.rel_width)
    return level, slot - (g.k + 1)


def row(g, u):
    b, e = int(g.row_ptr[u]), int(g.row_ptr[u + 1])
    return g.col[b:e], g.rel[b:e]


# ---------------------------------------------------------------- node set
@pytest.mark.parametrize("n", [2, 4, 16, 512, 4096])
def test_node_count_and_levels(n):
    # Sec. 3.2.1: 2n-1 partitions; perfect binary tree; level l has n/2^l nodes
    g = oracle.build_graph(n, 2, False)
    assert g.num_nodes == 2 * n - 1
    assert g.num_levels == int(np.log2(n)) + 1
    acc = 0
    for l in range(g.num_levels):
        assert oracle.level_offset(n, l) == acc
        acc += n >> l
    assert acc == 2 * n - 1
    assert oracle.level_offset(n, g.num_levels - 1) == 2 * n - 2        # root is the last id


def test_rejects_bad_arguments():
    for n in (0, 1, 3, 6, 100):
        with pytest.raises(ValueError):
            oracle.build_graph(n, 2, False)
    with pytest.raises(ValueError):
        oracle.build_graph(8, 0, False)


# ---------------------------------------------------------- affiliated edges
@pytest.mark.parametrize("n,k,causal", SMALL + MEDIUM)
def test_affiliated_edges(n, k, causal):
    # Sec. 3.2.2: span u_{l,m} receives an edge from each of its 2^l tokens
    g = oracle.build_graph(n, k, causal)
    total = 0
    for u in range(n, g.num_nodes):
        level, m, lo, hi = node_span(n, u)
        c, r = row(g, u)
        assert len(c) == 1 << level
        assert np.array_equal(c, np.arange(lo, hi))
        assert all(unpack(g, x) == (level, 0) for x in r)               # r_anc(level)
        total += len(c)
    assert total == n * int(np.log2(n))


# ------------------------------------------- contextual edges: declarative pin
def tilings(n, k, start):
    """All ways to cover tokens [start, n) by runs of aligned nodes, one run per
    consecutive level 0,1,2,..., run length k or k+1 (Sec. 3.2.2: k per level,
    plus the extra node), except the last run which only has to be 1..k+1 long
    and must end exactly at n.  Returns a list of solutions, each a list of
    (level, first_index, count)."""
    sols = []

    def rec(level, pos, acc):
        size = 1 << level
        if pos % size:
            return                        # run would not start on a node of this level
        for cnt in range(1, k + 2):
            end = pos + cnt * size
            if end == n:
                sols.append(acc + [(level, pos // size, cnt)])
            elif end < n and cnt in (k, k + 1):
                rec(level + 1, end, acc + [(level, pos // size, cnt)])

    if start < n:
        rec(0, start, [])
    else:
        sols.append([])
    return sols


@pytest.mark.parametrize("n,k", [(n, k) for n in (2, 4, 8, 16, 32) for k in (1, 2, 3, 4, 5, 40)])
def test_contextual_edges_are_the_unique_tiling(n, k):
    g = oracle.build_graph(n, k, False)
    gc = oracle.build_graph(n, k, True)
    for i in range(n):
        right = tilings(n, k, i + 1)
        # the left context is the mirror image: token i has n-1-i ... reversed
        left_m = tilings(n, k, n - i)       # mirror: tokens [0,i) <-> [n-i, n)
        assert len(right) == 1 and len(left_m) == 1, (n, k, i, right, left_m)
        expect = {(0, i, 0, 0)}             # (level, index, side, order) ; self
        for level, first, cnt in right[0]:
            for t in range(cnt):
                expect.add((level, first + t, +1, t + 1))
        for level, first, cnt in left_m[0]:
            cnt_nodes = n >> level
            for t in range(cnt):
                expect.add((level, cnt_nodes - 1 - (first + t), -1, t + 1))
        for graph, keep in ((g, lambda s: True), (gc, lambda s: s <= 0)):
            c, r = row(graph, i)
            got = set()
            for node, rid in zip(c, r):
                level, m, lo, hi = node_span(n, int(node))
                lv, off = unpack(graph, rid)
                assert lv == level
                got.add((level, m, int(np.sign(off)), abs(off)))
            assert got == {x for x in expect if keep(x[2])}, (n, k, i)
            assert len(c) == len(got)


@pytest.mark.parametrize("n,k,causal", SMALL + MEDIUM)
def test_token_rows_tile_the_sequence(n, k, causal):
    # Sec. 3: context grouped into non-overlapping spans whose scale grows with
    # distance;  Sec. 3.2.2: distance between two tokens is at most 2 hops, i.e.
    # every other token lies in exactly one attended span.
    g = oracle.build_graph(n, k, causal)
    for i in range(n):
        c, r = row(g, i)
        cover = np.zeros(n, dtype=np.int64)
        per_level = {}
        for node, rid in zip(c, r):
            level, m, lo, hi = node_span(n, int(node))
            cover[lo:hi] += 1
            lv, off = unpack(g, rid)
            assert lv == level
            if off == 0:
                assert node == i and level == 0
            else:
                assert (off > 0) == (lo > i) and (off < 0) == (hi <= i)
                assert not (lo <= i < hi)           # never an ancestor of itself
                per_level.setdefault((level, off > 0), []).append((abs(off), lo))
        want = np.ones(n, dtype=np.int64)
        if causal:
            want[i + 1:] = 0
        assert np.array_equal(cover, want), (n, k, causal, i)
        for (level, right), lst in per_level.items():
            lst.sort()
            offs = [o for o, _ in lst]
            assert offs == list(range(1, len(lst) + 1))         # i-th node to join, nearest first
            assert len(lst) <= k + 1                            # k regular + at most one extra
            starts = [lo for _, lo in lst]
            step = (1 << level) if right else -(1 << level)
            assert all(b - a == step for a, b in zip(starts, starts[1:]))
        for right in (False, True):
            levels = sorted(l for (l, rr) in per_level if rr == right)
            assert levels == list(range(len(levels)))           # consecutive levels from 0
            for l in levels[:-1]:
                assert len(per_level[(l, right)]) in (k, k + 1)


@pytest.mark.parametrize("n,k", [(16, 1), (32, 2), (64, 3), (256, 4), (512, 9)])
def test_mirror_symmetry_and_causal_subset(n, k):
    g = oracle.build_graph(n, k, False)
    gc = oracle.build_graph(n, k, True)
    for i in range(n):
        c, r = row(g, i)
        cm, rm = row(g, n - 1 - i)
        a = set()
        for node, rid in zip(c, r):
            level, m, _, _ = node_span(n, int(node))
            a.add((level, m, unpack(g, rid)[1]))
        b = set()
        for node, rid in zip(cm, rm):
            level, m, _, _ = node_span(n, int(node))
            b.add((level, (n >> level) - 1 - m, -unpack(g, rid)[1]))
        assert a == b
        cc, rc = row(gc, i)
        keep = np.array([unpack(g, x)[1] <= 0 for x in r])
        assert np.array_equal(cc, c[keep]) and np.array_equal(rc, r[keep])
    # span rows are identical in both graphs
    for u in range(n, g.num_nodes):
        assert np.array_equal(row(g, u)[0], row(gc, u)[0])


@pytest.mark.parametrize("n", [2, 8, 64, 256])
def test_k_at_least_n_is_the_complete_token_graph(n):
    # Sec. 3.4 last paragraph: k >= sentence length degenerates to the vanilla Transformer
    for k in (n, n + 3):
        g = oracle.build_graph(n, k, False)
        for i in range(n):
            c, r = row(g, i)
            assert np.array_equal(c, np.arange(n))
            assert [unpack(g, x) for x in r] == [(0, j - i) for j in range(n)]
        assert g.num_edges == n * n + n * int(np.log2(n))
        gc = oracle.build_graph(n, k, True)
        for i in range(n):
            assert np.array_equal(row(gc, i)[0], np.arange(i + 1))


@pytest.mark.parametrize("n,k,causal", [(512, 4, False), (8192, 8, True), (4096, 2, False), (4096, 32, False),
                                        (1024, 1, True), (2048, 16, False)])
def test_edge_count_growth(n, k, causal):
    # Sec. 3.2.2: O(k n log(n/k)) edges.  Band implied by "k or k+1 nodes per
    # side per level over about log2(n/k) levels".
    s = 1 if causal else 2
    deg = oracle.degrees(n, k, causal)
    ctx = int(deg[:n].sum()) - n
    lg = np.log2(n / k)
    assert n * s * k * (np.floor(lg) - 2) <= ctx <= n * s * (k + 1) * (np.ceil(lg) + 1)
    ctx2 = int(oracle.degrees(2 * n, k, causal)[:2 * n].sum()) - 2 * n
    assert abs(ctx2 / ctx - 2 * (1 + 1 / lg)) < 0.25


def test_csr_is_canonical():
    for n, k, causal in SMALL + MEDIUM:
        g = oracle.build_graph(n, k, causal)
        assert g.row_ptr[0] == 0 and np.all(np.diff(g.row_ptr) > 0)     # no empty row
        assert np.array_equal(np.diff(g.row_ptr), oracle.degrees(n, k, causal))
        for u in range(g.num_nodes):
            c, r = row(g, u)
            assert np.all(np.diff(r) > 0) if u < n else np.all(np.diff(r) == 0)
            assert np.all(np.diff(c) > 0)
            assert c.min() >= 0 and c.max() < g.num_nodes
            assert r.min() >= 0 and r.max() < g.num_levels * g.rel_width


def test_hand_derived_example():
    """n=16, k=2, bidirectional, token 5, worked by hand from Sec. 3.2.2's rule
    (fixture: tests/golden/toy_n16_k2_token5.txt).  Not printed in the paper."""
    rows = []
    with open(os.path.join(GOLDEN, "toy_n16_k2_token5.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(tuple(int(x) for x in line.split()))
    g = oracle.build_graph(16, 2, False)
    c, r = row(g, 5)
    got = []
    for node, rid in zip(c, r):
        level, m, lo, hi = node_span(16, int(node))
        got.append((level, lo, hi, unpack(g, rid)[1]))
    assert got == rows


def test_golden_edge_counts():
    """Edge counts of the benchmark graphs, written by tests/golden/make_edge_counts.py
    (oracle only) -- a regression pin, cross-checked there against the closed
    form for the affiliated part."""
    with open(os.path.join(GOLDEN, "edge_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            n, k, causal, E = (int(x) for x in line.split())
            assert int(oracle.degrees(n, k, bool(causal)).sum()) == E


# ------------------------------------------------------------ transposed CSR
@pytest.mark.parametrize("n,k,causal", [(2, 1, False), (8, 1, True), (32, 2, False), (64, 3, True),
                                        (512, 4, False), (1024, 8, True)])
def test_transpose_matches_definition(n, k, causal):
    g = oracle.build_graph(n, k, causal)
    t_ptr, t_src, t_eid = oracle.transpose(g)
    order = np.argsort(g.col, kind="stable")                 # edges grouped by key, edge index ascending
    src_of_edge = np.repeat(np.arange(g.num_nodes), np.diff(g.row_ptr))
    assert np.array_equal(t_eid, order)
    assert np.array_equal(t_src, src_of_edge[order])
    assert np.array_equal(t_ptr, np.concatenate([[0], np.cumsum(np.bincount(g.col, minlength=g.num_nodes))]))


@pytest.mark.parametrize("n,k,causal", [(32, 2, False), (64, 3, True), (512, 4, False), (2048, 8, True)])
def test_in_neighbours_are_contiguous_token_ranges(n, k, causal):
    """Monotonicity of the run boundaries in the token index makes the set of
    tokens attending to a node, on either side of it, one contiguous range."""
    g = oracle.build_graph(n, k, causal)
    t_ptr, t_src, _ = oracle.transpose(g)
    for v in range(g.num_nodes):
        level, m, lo, hi = node_span(n, v)
        src = t_src[t_ptr[v]:t_ptr[v + 1]]
        tok = src[src < n]
        left, right = tok[tok < lo], tok[tok >= hi]
        for part in (left, right):
            if len(part):
                assert np.array_equal(part, np.arange(part[0], part[0] + len(part)))
        anc = src[src >= n]
        if level == 0:
            assert len(anc) == g.num_levels - 1          # one affiliated edge per ancestor
            assert np.sum(tok == v) == 1
        else:
            assert len(anc) == 0 and not np.any((tok >= lo) & (tok < hi))


# ------------------------------------------- sequences of any length on the tree over n
# The paper states the tree for n a power of two (Sec. 3.2.1).  The oracle's reading for a
# sequence of `length` <= n tokens keeps the nodes that hold a token; the checks below pin it
# to the pinned power-of-two builder (as a sub-graph, and as the smaller tree when the length
# is itself a power of two), to a declarative search, and to the covering invariant.
LEN_CASES = [(n, k, c) for n in (2, 4, 8, 16, 32) for k in (1, 2, 3, 5, 40) for c in (False, True)]


@pytest.mark.parametrize("n,k,causal", LEN_CASES + [(256, 3, False), (512, 4, True)])
def test_length_n_is_the_graph_of_the_paper(n, k, causal):
    a, b = oracle.build_graph_len(n, n, k, causal), oracle.build_graph(n, k, causal)
    assert np.array_equal(a.row_ptr, b.row_ptr) and np.array_equal(a.col, b.col) and np.array_equal(a.rel, b.rel)


def test_length_arguments():
    for n, length in ((8, 0), (8, 9), (6, 3), (8, -1)):
        with pytest.raises(ValueError):
            oracle.build_graph_len(n, length, 2, False)


@pytest.mark.parametrize("n,k,causal", LEN_CASES + [(128, 3, False), (256, 2, True), (512, 7, False)])
def test_length_graph_is_the_sub_graph_of_kept_nodes(n, k, causal):
    # a node is kept iff its first token exists; an edge iff both ends are kept; packed ids and
    # the order of a row's edges are those of the full graph
    full = oracle.build_graph(n, k, causal)
    keep = np.array([node_span(n, v)[2] for v in range(full.num_nodes)])
    lengths = range(1, n + 1) if n <= 32 else (1, 2, 3, n // 2 - 1, n // 2, n // 2 + 1, n - 5, n - 1)
    for length in lengths:
        g = oracle.build_graph_len(n, length, k, causal)
        ok = keep < length
        for u in range(full.num_nodes):
            c, r = row(full, u)
            sel = ok[c] & ok[u]
            gc, gr = row(g, u)
            assert np.array_equal(gc, c[sel]) and np.array_equal(gr, r[sel]), (n, k, causal, length, u)


def tilings_len(length, k, start):
    """As tilings(), for a sequence whose levels end with a node that may be cut short: the
    last run is 1..k+1 nodes long, its last node holds a token and reaches the end.  With cut
    nodes the end of the sequence no longer forces alignment, so the rule for the extra node
    (Sec. 3.2.2: only when k nodes do not end on a parent boundary) is stated as a constraint."""
    sols = []

    def rec(level, pos, acc):
        size = 1 << level
        if pos % size:
            return
        for cnt in range(1, k + 2):
            last_lo, end = pos + (cnt - 1) * size, pos + cnt * size
            if last_lo >= length:
                break
            if cnt == k + 1 and (pos + k * size) % (2 * size) == 0:
                continue
            if end >= length:
                sols.append(acc + [(level, pos // size, cnt)])
            elif cnt in (k, k + 1):
                rec(level + 1, end, acc + [(level, pos // size, cnt)])

    if start < length:
        rec(0, start, [])
    else:
        sols.append([])
    return sols


@pytest.mark.parametrize("n,k", [(n, k) for n in (4, 8, 16, 32) for k in (1, 2, 3, 5, 40)])
def test_length_right_context_is_the_unique_tiling(n, k):
    full = oracle.build_graph(n, k, False)
    for length in range(1, n + 1):
        g = oracle.build_graph_len(n, length, k, False)
        for i in range(length):
            sols = tilings_len(length, k, i + 1)
            assert len(sols) == 1, (n, k, length, i, sols)
            expect = {(level, first + t, t + 1) for level, first, cnt in sols[0] for t in range(cnt)}
            c, r = row(g, i)
            got, left = set(), []
            for node, rid in zip(c, r):
                level, m, lo, hi = node_span(n, int(node))
                lv, off = unpack(g, rid)
                assert lv == level
                if off > 0:
                    got.add((level, m, off))
                elif off < 0:
                    left.append((int(node), int(rid)))
            assert got == expect, (n, k, length, i)
            # the left context does not depend on what follows the token
            fc, fr = row(full, i)
            assert left == [(int(a), int(b)) for a, b in zip(fc, fr) if unpack(full, b)[1] < 0]


@pytest.mark.parametrize("n,k,causal", LEN_CASES + [(64, 3, False), (128, 2, True)])
def test_length_rows_tile_the_sequence(n, k, causal):
    lengths = range(1, n + 1) if n <= 32 else (1, 5, 31, 33, 47, 64, 100, n - 1)
    for length in lengths:
        if length > n:
            continue
        g = oracle.build_graph_len(n, length, k, causal)
        for i in range(length):
            c, _ = row(g, i)
            cover = np.zeros(n, dtype=np.int64)
            for node in c:
                _, _, lo, hi = node_span(n, int(node))
                assert lo < length
                cover[lo:min(hi, length)] += 1
            want = np.zeros(n, dtype=np.int64)
            want[:(i + 1 if causal else length)] = 1
            assert np.array_equal(cover, want), (n, k, causal, length, i)
        for u in range(n, g.num_nodes):          # span rows: the tokens they hold, r_anc(level)
            level, m, lo, hi = node_span(n, u)
            c, r = row(g, u)
            assert list(c) == list(range(lo, min(hi, length)))
            assert all(unpack(g, x) == (level, 0) for x in r)
        assert g.row_ptr[length] == g.row_ptr[n]                 # tokens beyond the end: empty rows


@pytest.mark.parametrize("n,p,k,causal", [(8, 2, 1, False), (16, 4, 2, True), (32, 8, 3, False), (64, 16, 1, True),
                                           (256, 64, 4, False), (512, 128, 9, True), (64, 32, 40, False)])
def test_power_of_two_length_is_the_smaller_tree(n, p, k, causal):
    # a sequence of p = 2^a tokens padded to n: levels 0..a are the tree over p of the paper;
    # each higher level keeps one node, which holds all p tokens
    g = oracle.build_graph_len(n, p, k, causal)
    small = oracle.build_graph(p, k, causal)
    to_big = np.zeros(small.num_nodes, dtype=np.int64)
    for v in range(small.num_nodes):
        level, m, _, _ = node_span(p, v)
        to_big[v] = oracle.level_offset(n, level) + m
    for v in range(small.num_nodes):
        c, r = row(small, v)
        gc, gr = row(g, int(to_big[v]))
        assert np.array_equal(gc, to_big[c]) and np.array_equal(gr, r), (v,)
    top = small.num_levels
    for level in range(top, g.num_levels):
        c, r = row(g, oracle.level_offset(n, level))
        assert list(c) == list(range(p)) and all(unpack(g, x) == (level, 0) for x in r)
    used = set(int(x) for x in to_big) | {oracle.level_offset(n, l) for l in range(top, g.num_levels)}
    deg = np.diff(g.row_ptr)
    assert all(deg[u] == 0 for u in range(g.num_nodes) if u not in used)
