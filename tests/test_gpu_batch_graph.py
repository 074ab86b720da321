"""GPU parity of the packed batch graph (bpt_build_batch_graph): one graph for a batch of sequences of different
lengths, rows only for the nodes that exist.

The expected graph is oracle.build_batch_graph (the oracle's per-length graph of every sequence, renumbered into
the packed rows and joined); the expected attention results are the oracle's per-length results
(oracle.attn_*_lengths on padded arrays), read at the rows of the kept nodes.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1911_04070_amd import binding as bpt

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def say(*a):
    print(*a, flush=True)


BATCHES = [
    (2, 1, False, [2]), (2, 1, True, [1, 2, 1]), (8, 1, False, [8, 1, 5, 3]), (16, 2, False, [16, 9, 1, 0, 7]),
    (16, 3, True, [0, 0, 5]), (64, 2, False, [64, 1, 37, 17, 64, 2]), (64, 70, False, [33, 64, 50]),
    (256, 3, True, [100, 256, 2, 255]), (512, 4, False, [512, 300, 33, 1, 0, 511, 257]), (1024, 1, False, [1000, 17, 1024, 3]),
    (2048, 16, False, [2047, 1025, 3]), (4096, 8, True, [3000, 4096, 129]), (8192, 4, False, [5000, 8192, 1, 4097]),
]


@pytest.mark.parametrize("n,k,causal,lengths", BATCHES)
def test_batch_graph_is_bit_exact(n, k, causal, lengths):
    say("batch graph", n, k, causal, lengths)
    want = oracle.build_batch_graph(n, k, causal, lengths)
    g = bpt.bpt_build_batch_graph(n, k, causal, lengths)
    first, count, rows = oracle.batch_layout(n, lengths)
    assert (g.batch, g.n_tokens, g.num_nodes) == (len(lengths), int(sum(lengths)), rows)
    assert np.array_equal(g.first_row, first) and np.array_equal(g.row_count, count)
    assert g.num_edges == want.num_edges
    assert g.num_edges == sum(bpt.bpt_count_edges(n, k, causal, int(length)) for length in lengths)
    row_ptr, col, rel = g.csr_to_host()
    assert np.array_equal(row_ptr, want.row_ptr)
    assert np.array_equal(col, want.col)
    assert np.array_equal(rel, want.rel)
    t_ptr, t_src, t_eid = g.transposed_to_host()
    w_ptr, w_src, w_eid = oracle.transpose(want)
    assert np.array_equal(t_ptr, w_ptr)
    assert np.array_equal(t_src, w_src)
    assert np.array_equal(t_eid, w_eid)
    g.destroy()


def test_random_batch_graphs_are_bit_exact():
    rng = np.random.default_rng(2024)
    for case in range(40):
        n = int(2 ** rng.integers(1, 12))
        k = int(rng.integers(1, 24))
        causal = bool(rng.integers(0, 2))
        B = int(rng.integers(1, 40))
        lengths = [int(v) for v in rng.integers(0, n + 1, size=B)]
        if sum(lengths) == 0:
            lengths[-1] = 1
        say("random batch graph", case, n, k, causal, lengths[:8], "..." if B > 8 else "")
        want = oracle.build_batch_graph(n, k, causal, lengths)
        g = bpt.bpt_build_batch_graph(n, k, causal, lengths)
        row_ptr, col, rel = g.csr_to_host()
        assert np.array_equal(row_ptr, want.row_ptr) and np.array_equal(col, want.col) and np.array_equal(rel, want.rel)
        t_ptr, t_src, t_eid = g.transposed_to_host()
        w_ptr, w_src, w_eid = oracle.transpose(want)
        assert np.array_equal(t_ptr, w_ptr) and np.array_equal(t_src, w_src) and np.array_equal(t_eid, w_eid)
        g.destroy()


def test_batch_graph_of_full_sequences_is_the_single_graph_repeated():
    n, k = 256, 3
    one = bpt.bpt_build_graph(n, k, False)
    rp, col, rel = one.csr_to_host()
    g = bpt.bpt_build_batch_graph(n, k, False, [n])
    rp1, col1, rel1 = g.csr_to_host()
    assert np.array_equal(rp, rp1) and np.array_equal(col, col1) and np.array_equal(rel, rel1)
    assert np.array_equal(g.first_row[:, 0], one.first_row[:, 0]) and np.array_equal(g.row_count, one.row_count)
    assert (one.batch, one.n_tokens) == (1, n)
    one.destroy()
    g.destroy()


def test_batch_graph_errors():
    with pytest.raises(bpt.BptError):
        bpt.bpt_build_batch_graph(64, 2, False, [0, 0])          # no token at all
    with pytest.raises(bpt.BptError):
        bpt.bpt_build_batch_graph(64, 2, False, [65])            # longer than n
    with pytest.raises(bpt.BptError):
        bpt.bpt_build_batch_graph(64, 2, False, [-1, 4])
    with pytest.raises(bpt.BptError):
        bpt.bpt_build_batch_graph(48, 2, False, [4])             # n not a power of two
    g = bpt.bpt_build_batch_graph(64, 2, False, [10, 64])
    x = torch.zeros(1, 1, g.num_nodes, 64, device="cuda")
    r = torch.zeros(g.num_levels, g.rel_width, 64, device="cuda")
    with pytest.raises(bpt.BptError):                            # the graph carries the lengths itself
        bpt.bpt_attn_fwd(g, x, x, x, r, seq_len=torch.tensor([10], dtype=torch.int32, device="cuda"))
    with pytest.raises(bpt.BptError):                            # dropout masks are defined on one tree's nodes
        bpt.bpt_attn_fwd(g, x, x, x, r, dropout=(0.1, 3))
    g.destroy()


def bf16_round(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).float().numpy()


def to_dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def run_attention_case(dtype, n, k, causal, H, lengths, node_major=False, seed=5):
    say("batch attention", dtype, n, k, causal, H, lengths, "node-major" if node_major else "head-major")
    _, b_of, node_of = oracle.batch_rows(n, lengths)
    rows = len(b_of)
    B, N, D = len(lengths), 2 * n - 1, 64
    L, W = oracle.num_levels(n), 2 * (k + 1) + 1
    rng = np.random.default_rng(seed)
    packed = {key: rng.standard_normal((1, H, rows, D)).astype(np.float32) for key in ("Q", "K", "V", "dO")}
    Rel = (0.5 * rng.standard_normal((L, W, D))).astype(np.float32)
    if dtype == "bf16":
        packed = {key: bf16_round(v) for key, v in packed.items()}
        Rel = bf16_round(Rel)
    # the same rows on the padded trees, one batch entry per sequence (other rows: anything -- the oracle's
    # per-length graph has no edge to them)
    padded = {key: np.full((B, H, N, D), 7.0, dtype=np.float32) for key in packed}
    for key in packed:
        padded[key][b_of, :, node_of] = np.transpose(packed[key][0], (1, 0, 2))
    live = [b for b, length in enumerate(lengths) if length >= 1]
    ll = [lengths[b] for b in live]
    sub = {key: np.ascontiguousarray(v[live]) for key, v in padded.items()}
    scale = 0.125
    o, l, _ = oracle.attn_fwd_lengths(n, k, causal, ll, sub["Q"], sub["K"], sub["V"], Rel, scale)
    dq, dk, dv, dr = oracle.attn_bwd_lengths(n, k, causal, ll, sub["Q"], sub["K"], sub["V"], Rel, sub["dO"], scale)
    pos = {b: i for i, b in enumerate(live)}
    bi = np.array([pos[b] for b in b_of])
    ref = {"out": o[bi, :, node_of], "dQ": dq[bi, :, node_of], "dK": dk[bi, :, node_of], "dV": dv[bi, :, node_of]}
    ref = {key: np.transpose(v, (1, 0, 2))[None] for key, v in ref.items()}          # [1, H, rows, D]
    ref["lse"] = np.transpose(l[bi, :, node_of], (1, 0))[None]
    ref["d_rel"] = dr

    g = bpt.bpt_build_batch_graph(n, k, causal, lengths)
    assert g.num_nodes == rows
    if node_major:   # [1, rows, H, D] memory seen as [1, H, rows, D]
        Q, K, V, dO = (to_dev(np.transpose(packed[key], (0, 2, 1, 3)), dtype).transpose(1, 2) for key in ("Q", "K", "V", "dO"))
    else:
        Q, K, V, dO = (to_dev(packed[key], dtype) for key in ("Q", "K", "V", "dO"))
    R = to_dev(Rel, dtype)
    bpt.bpt_profile_enable(True)
    out_d, lse_d = bpt.bpt_attn_fwd(g, Q, K, V, R, scale=scale)
    grads = bpt.bpt_attn_bwd(g, Q, K, V, R, lse_d, dO, scale=scale)
    torch.cuda.synchronize()
    ran = set(bpt.bpt_profile_report())
    bpt.bpt_profile_enable(False)
    say("   kernels", sorted(ran))
    # bf16 tensors on trees of at least 32 tokens: the matrix-core kernels on the packed rows, not the gather kernels
    tiles = dtype == "bf16" and n >= 32
    assert ("fwd_tile_kernel" in ran) == tiles and ("bwd_q_tile_kernel" in ran) == tiles, ran
    assert ("bwd_kv_tile_kernel" in ran or "bwd_kv_chain_kernel" in ran) == tiles, ran
    assert ("fwd_kernel" in ran or "bwd_q_kernel" in ran or "bwd_kv_kernel" in ran) == (not tiles), ran
    res = {}
    for name, got_t in zip(("out", "lse", "dQ", "dK", "dV", "d_rel"), (out_d, lse_d) + tuple(grads)):
        got = host(got_t)
        assert got.shape == ref[name].shape, (name, got.shape, ref[name].shape)
        assert np.isfinite(got).all(), name
        res[name] = float(np.abs(got - ref[name]).max())
        assert res[name] <= TOL[dtype], (name, res[name])
    say("   max-abs errors", {key: float("%.3g" % v) for key, v in res.items()})
    if dtype == "bf16":   # gradients rounded to bf16: the same sums, rounded once
        g16 = bpt.bpt_attn_bwd(g, Q, K, V, R, lse_d, dO, scale=scale, bf16_grads=True)
        torch.cuda.synchronize()
        for name, a32, a16 in zip(("dQ", "dK", "dV"), grads[:3], g16[:3]):
            want = a32.to(torch.bfloat16)
            if name == "dQ":   # rounded twice where a second kernel adds the relative-position part (many ids in use)
                bound = want.float().abs() * 2.0 ** -7 + float(want.float().abs().max()) * 2.0 ** -8
                assert bool(((a16.float() - want.float()).abs() <= bound).all())
            else:
                assert torch.equal(want, a16), name
        assert torch.equal(grads[3], g16[3])
    g.destroy()


ATTENTION = [
    ("f32", 8, 1, False, 1, [8, 1, 5, 3]), ("f32", 64, 2, False, 2, [64, 1, 37, 17, 0]), ("f32", 256, 3, True, 1, [100, 256, 2]),
    ("f32", 2048, 5, False, 1, [1500, 700, 3]), ("f32", 64, 70, False, 1, [33, 64, 50]),
    ("bf16", 16, 1, False, 2, [16, 9, 1]), ("bf16", 64, 2, False, 1, [33, 64, 2, 48]),
    ("bf16", 512, 4, False, 2, [512, 300, 33, 1, 0]), ("bf16", 1024, 3, True, 2, [1000, 17, 1024]),
    ("bf16", 2048, 16, False, 1, [2047, 1025]), ("bf16", 4096, 8, True, 1, [3000, 4096, 129]),
    ("bf16", 1024, 40, False, 1, [700, 90]),
    # eight sequences of three tokens: eight consecutive span rows of degree 3 (no power of two)
    ("f32", 16, 1, False, 1, [3] * 9), ("bf16", 16, 2, False, 1, [3] * 9 + [6] * 8),
]


@pytest.mark.parametrize("dtype,n,k,causal,H,lengths", ATTENTION)
def test_attention_on_a_batch_graph(dtype, n, k, causal, H, lengths):
    run_attention_case(dtype, n, k, causal, H, lengths)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_on_a_batch_graph_with_node_major_memory(dtype):
    run_attention_case(dtype, 512, 4, False, 4, [400, 512, 77, 1], node_major=True)


def test_a_batch_of_300_sequences_and_the_language_model_shape():
    # more sequences than the token-tile kernels number in closed form (256): their walk over all (sequence, head,
    # tile) triples takes over; and two long sequences at the language-modelling density
    rng = np.random.default_rng(300)
    run_attention_case("bf16", 64, 2, False, 1, [int(v) for v in rng.integers(0, 65, size=300)])
    run_attention_case("bf16", 8192, 8, True, 2, [1332, 7532])


def test_nothing_is_written_outside_the_rows_of_a_batch_graph():
    # the tensors are views of larger buffers: the rows before and after them keep their pattern
    n, k, H, lengths = 512, 4, 2, [300, 33, 512, 1, 77]
    g = bpt.bpt_build_batch_graph(n, k, False, lengths)
    rows, pad, mark = g.num_nodes, 64, 5.0
    gen = torch.Generator(device="cuda").manual_seed(7)
    rnd = lambda: torch.randn(1, H, rows, 64, device="cuda", generator=gen).to(torch.bfloat16)
    Q, K, V, dO = rnd(), rnd(), rnd(), rnd()
    R = (0.1 * torch.randn(g.num_levels, g.rel_width, 64, device="cuda", generator=gen)).to(torch.bfloat16)

    def framed(dtype):   # [1, H, pad + rows + pad, 64] full of the mark; the middle rows are the tensor
        buf = torch.full((1, H, rows + 2 * pad, 64), mark, dtype=dtype, device="cuda")
        return buf, buf[:, :, pad:pad + rows]

    obuf, out = framed(torch.bfloat16)
    lse_c = torch.empty(1, H, rows, dtype=torch.float32, device="cuda")
    Qb, Qv = framed(torch.bfloat16)
    Qv.copy_(Q)
    K2, V2 = framed(torch.bfloat16)[1], framed(torch.bfloat16)[1]
    K2.copy_(K)
    V2.copy_(V)
    bpt.bpt_attn_fwd(g, Qv, K2, V2, R, out=out, lse=lse_c)
    dbufs = [framed(torch.float32) for _ in range(3)]
    dOv = framed(torch.bfloat16)[1]
    dOv.copy_(dO)
    d_rel = torch.empty_like(R, dtype=torch.float32)
    bpt.bpt_attn_bwd(g, Qv, K2, V2, R, lse_c, dOv, grads=tuple(v for _, v in dbufs) + (d_rel,))
    torch.cuda.synchronize()
    for buf in [obuf] + [b for b, _ in dbufs]:
        assert bool((buf[:, :, :pad] == mark).all()) and bool((buf[:, :, pad + rows:] == mark).all())
    # and the framed call gives the bits of the plain one
    out0, lse0 = bpt.bpt_attn_fwd(g, Q, K, V, R)
    g0 = bpt.bpt_attn_bwd(g, Q, K, V, R, lse0, dO)
    torch.cuda.synchronize()
    assert torch.equal(out0, out) and torch.equal(lse0, lse_c)
    for (_, v), w in zip(dbufs, g0[:3]):
        assert torch.equal(v, w)
    g.destroy()


def test_long_sequences_in_a_batch_graph():
    run_attention_case("bf16", 16384, 4, True, 1, [16384, 9000, 33])


def test_the_forward_that_allocates_nothing_takes_a_batch_graph():
    g = bpt.bpt_build_batch_graph(2048, 4, False, [2048, 700, 1, 1300])
    gen = torch.Generator(device="cuda").manual_seed(11)
    Q, K, V = (torch.randn(1, 2, g.num_nodes, 64, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(3))
    R = (0.1 * torch.randn(g.num_levels, g.rel_width, 64, device="cuda", generator=gen)).to(torch.bfloat16)
    out0, lse0 = bpt.bpt_attn_fwd(g, Q, K, V, R)
    out1, lse1 = torch.full_like(Q, 7.0), torch.full(Q.shape[:3], 7.0, dtype=torch.float32, device="cuda")
    bpt.bpt_attn_fwd_static(g, Q, K, V, R, out1, lse1)
    torch.cuda.synchronize()
    assert torch.equal(out0, out1) and torch.equal(lse0, lse1)
    g.destroy()


def test_batch_graphs_on_a_shared_tree():
    # bpt_build_batch_graph_on: the tree of (n, k, causal) is built once and shared by the graphs of many batches; without
    # edge lists such a graph is a few small tables, serves the matrix-core kernels and refuses the rest
    n, k, causal, H = 1024, 4, False, 2
    tree = bpt.bpt_build_graph(n, k, causal)
    gen = torch.Generator(device="cuda").manual_seed(3)
    for lengths in ([1024, 300, 33, 1, 0], [7, 900], [512] * 5):
        full = bpt.bpt_build_batch_graph(n, k, causal, lengths)
        with_e = bpt.bpt_build_batch_graph_on(tree, lengths, with_edges=True)
        light = bpt.bpt_build_batch_graph_on(tree, lengths)
        for g in (with_e, light):
            assert (g.num_nodes, g.n_tokens, g.batch) == (full.num_nodes, full.n_tokens, full.batch)
            assert np.array_equal(g.first_row, full.first_row) and np.array_equal(g.row_count, full.row_count)
        for a, b in zip(full.csr_to_host() + full.transposed_to_host(), with_e.csr_to_host() + with_e.transposed_to_host()):
            assert np.array_equal(a, b)
        assert light.num_edges == 0
        with pytest.raises(bpt.BptError):
            light.csr_to_host()
        Q, K, V, dO = (torch.randn(1, H, full.num_nodes, 64, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(4))
        R = (0.1 * torch.randn(full.num_levels, full.rel_width, 64, device="cuda", generator=gen)).to(torch.bfloat16)
        out0, lse0 = bpt.bpt_attn_fwd(full, Q, K, V, R)
        g0 = bpt.bpt_attn_bwd(full, Q, K, V, R, lse0, dO)
        for g in (with_e, light):
            out1, lse1 = bpt.bpt_attn_fwd(g, Q, K, V, R)
            g1 = bpt.bpt_attn_bwd(g, Q, K, V, R, lse1, dO)
            torch.cuda.synchronize()
            assert torch.equal(out0, out1) and torch.equal(lse0, lse1)
            for x, y in zip(g0, g1):
                assert torch.equal(x, y)
        # fp32 tensors run the gather kernels, which need the edge lists
        Qf = Q.float()
        bpt.bpt_attn_fwd(with_e, Qf, Qf, Qf, R.float())
        with pytest.raises(bpt.BptError) as e:
            bpt.bpt_attn_fwd(light, Qf, Qf, Qf, R.float())
        assert e.value.status == bpt.BPT_ERR_UNSUPPORTED
        for g in (full, with_e, light):
            g.destroy()
    with pytest.raises(bpt.BptError):       # a batch graph is no tree
        b = bpt.bpt_build_batch_graph(n, k, causal, [5, 6])
        bpt.bpt_build_batch_graph_on(b, [3])
    tree.destroy()


def test_a_batch_of_32_sentences():
    # the classification workload's batch: 32 sentences of very different lengths on trees over 512 tokens
    rng = np.random.default_rng(32)
    lengths = [int(v) for v in np.clip(rng.lognormal(5.2, 0.7, size=32), 5, 512)]
    run_attention_case("bf16", 512, 4, False, 2, lengths)
