"""Pins for the oracle's attention forward and backward (CPU only).

The graph attention of Sec. 3.1 eq. (6) / Sec. 3.4 eq. (8) is by definition
dense softmax attention over all 2n-1 nodes with non-edges masked out, so the
pins are: that dense definition written with numpy, torch's SDPA and autograd
on the dense form, central finite differences, and closed-form invariants.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1911_04070_amd.workloads import WORKLOADS, make_inputs, shrink


def rand_inputs(g, B, H, D, seed, rel_std=0.5):
    rng = np.random.default_rng(seed)
    shp = (B, H, g.num_nodes, D)
    Q, K, V, dO = (rng.standard_normal(shp).astype(np.float32) for _ in range(4))
    Rel = (rel_std * rng.standard_normal((g.num_levels, g.rel_width, D))).astype(np.float32)
    return Q, K, V, Rel, dO


def dense_mask_and_ids(g):
    N = g.num_nodes
    mask = np.zeros((N, N), dtype=bool)
    ids = np.zeros((N, N), dtype=np.int64)
    for u in range(N):
        b, e = g.row_ptr[u], g.row_ptr[u + 1]
        mask[u, g.col[b:e]] = True
        ids[u, g.col[b:e]] = g.rel[b:e]
    return mask, ids


def dense_forward(g, Q, K, V, Rel, scale):
    """eq. (8) on the full N x N score matrix, float64."""
    mask, ids = dense_mask_and_ids(g)
    Q, K, V = (x.astype(np.float64) for x in (Q, K, V))
    R = Rel.astype(np.float64).reshape(-1, Rel.shape[-1])
    S = np.einsum("bhud,bhvd->bhuv", Q, K)
    S = S + np.einsum("bhud,uvd->bhuv", Q, R[ids])
    S = np.where(mask, S * scale, -np.inf)
    m = S.max(-1, keepdims=True)
    P = np.exp(S - m)
    Z = P.sum(-1, keepdims=True)
    return np.einsum("bhuv,bhvd->bhud", P / Z, V), (m + np.log(Z))[..., 0]


GRAPHS = [(2, 1, False), (4, 1, True), (8, 2, False), (16, 2, False), (32, 3, True), (64, 4, False), (64, 1, True)]


@pytest.mark.parametrize("n,k,causal", GRAPHS)
def test_forward_equals_dense_masked_attention(n, k, causal):
    g = oracle.build_graph(n, k, causal)
    Q, K, V, Rel, _ = rand_inputs(g, 2, 2, 8, seed=n * 10 + k)
    scale = 0.37
    out, lse, _ = oracle.attn_fwd(g, Q, K, V, Rel, scale)
    ref_out, ref_lse = dense_forward(g, Q, K, V, Rel, scale)
    assert np.abs(out - ref_out).max() < 1e-12
    assert np.abs(lse - ref_lse).max() < 1e-12


def test_forward_tiny_config_equals_dense():
    # the first benchmark configuration: n=512, k=4, bidirectional, 1 head of 64, fp32
    w = WORKLOADS["tiny"]
    g = oracle.build_graph(w.n, w.k, w.causal)
    x = make_inputs(w, with_dO=False)
    out, lse, _ = oracle.attn_fwd(g, x["Q"], x["K"], x["V"], x["Rel"], w.scale)
    ref_out, ref_lse = dense_forward(g, x["Q"], x["K"], x["V"], x["Rel"], w.scale)
    assert np.abs(out - ref_out).max() < 1e-12
    assert np.abs(lse - ref_lse).max() < 1e-12


def torch_dense(g, Q, K, V, Rel, scale):
    """SDPA (library routine) with the relative-position term as an additive bias."""
    mask, ids = dense_mask_and_ids(g)
    Qt, Kt, Vt = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    Rt = torch.tensor(Rel, dtype=torch.float64, requires_grad=True)
    R = Rt.reshape(-1, Rt.shape[-1])[torch.tensor(ids)]                    # [N,N,D]
    bias = scale * torch.einsum("bhud,uvd->bhuv", Qt, R)
    bias = bias.masked_fill(~torch.tensor(mask), float("-inf"))
    out = torch.nn.functional.scaled_dot_product_attention(Qt, Kt, Vt, attn_mask=bias, scale=scale)
    return out, (Qt, Kt, Vt, Rt)


@pytest.mark.parametrize("n,k,causal", GRAPHS)
def test_forward_and_backward_equal_torch_autograd(n, k, causal):
    g = oracle.build_graph(n, k, causal)
    Q, K, V, Rel, dO = rand_inputs(g, 2, 3, 8, seed=77 + n + k)
    scale = 1.0 / np.sqrt(8)
    out_t, leaves = torch_dense(g, Q, K, V, Rel, scale)
    out_t.backward(torch.tensor(dO, dtype=torch.float64))
    out, _, _ = oracle.attn_fwd(g, Q, K, V, Rel, scale)
    dQ, dK, dV, dRel, _ = oracle.attn_bwd(g, Q, K, V, Rel, dO, scale)
    assert np.abs(out - out_t.detach().numpy()).max() < 1e-12
    for got, leaf in zip((dQ, dK, dV, dRel), leaves):
        assert np.abs(got - leaf.grad.numpy()).max() < 1e-11


def test_backward_matches_finite_differences():
    g = oracle.build_graph(16, 2, False)
    Q, K, V, Rel, dO = rand_inputs(g, 1, 2, 4, seed=5)
    scale = 0.5
    dQ, dK, dV, dRel, _ = oracle.attn_bwd(g, Q, K, V, Rel, dO, scale)

    def loss(Q_, K_, V_, R_):
        o, _, _ = oracle.attn_fwd(g, Q_, K_, V_, R_, scale)
        return float((o * dO.astype(np.float64)).sum())

    rng = np.random.default_rng(0)
    h = 2.0 ** -7                       # exactly representable step: inputs stay float32-exact
    for name, grad, idx in (("Q", dQ, 0), ("K", dK, 1), ("V", dV, 2), ("Rel", dRel, 3)):
        args = [Q, K, V, Rel]
        for _ in range(25):
            pos = tuple(int(rng.integers(0, s)) for s in args[idx].shape)
            base = np.float32(np.round(args[idx][pos] * 128) / 128)     # keep x +/- h exact in float32
            hi, lo = [a.copy() for a in args], [a.copy() for a in args]
            hi[idx][pos] = base + np.float32(h)
            lo[idx][pos] = base - np.float32(h)
            mid = [a.copy() for a in args]
            mid[idx][pos] = base
            g_mid = oracle.attn_bwd(g, mid[0], mid[1], mid[2], mid[3], dO, scale)[idx][pos]
            fd = (loss(*hi) - loss(*lo)) / (2 * h)
            assert abs(fd - g_mid) < 5e-4 * max(1.0, abs(g_mid)), (name, pos, fd, g_mid)


@pytest.mark.parametrize("n", [4, 16, 64])
def test_k_at_least_n_without_rel_is_vanilla_attention(n):
    # Sec. 3.3 / Sec. 3.4: attending to all token nodes recovers the Transformer
    g = oracle.build_graph(n, n, False)
    Q, K, V, Rel, _ = rand_inputs(g, 1, 2, 16, seed=n)
    Rel[:] = 0
    scale = 0.25
    out, lse, _ = oracle.attn_fwd(g, Q, K, V, Rel, scale)
    Qt, Kt, Vt = (torch.tensor(x[:, :, :n], dtype=torch.float64) for x in (Q, K, V))
    ref = torch.softmax(Qt @ Kt.transpose(-1, -2) * scale, -1) @ Vt
    assert np.abs(out[:, :, :n] - ref.numpy()).max() < 1e-12
    # causal variant = lower-triangular attention
    gc = oracle.build_graph(n, n, True)
    outc, _, _ = oracle.attn_fwd(gc, Q, K, V, Rel, scale)
    refc = torch.nn.functional.scaled_dot_product_attention(Qt, Kt, Vt, is_causal=True, scale=scale)
    assert np.abs(outc[:, :, :n] - refc.numpy()).max() < 1e-12


def test_invariants_constant_values_and_row_shift():
    g = oracle.build_graph(64, 3, False)
    Q, K, V, Rel, dO = rand_inputs(g, 1, 2, 8, seed=3)
    scale = 0.3
    # all V rows equal -> every output row equals that vector (weights sum to 1)
    Vc = np.broadcast_to(V[:, :, :1], V.shape).copy()
    out, _, _ = oracle.attn_fwd(g, Q, K, Vc, Rel, scale)
    assert np.abs(out - Vc).max() < 1e-13
    # r_anc adds the same constant to every score of a span row: out unchanged,
    # lse moves by exactly scale * q_u . r_anc(level)
    out0, lse0, _ = oracle.attn_fwd(g, Q, K, V, Rel, scale)
    Rel2 = Rel.copy()
    Rel2[1:, g.k + 1, :] = 0
    out1, lse1, _ = oracle.attn_fwd(g, Q, K, V, Rel2, scale)
    assert np.abs(out0 - out1).max() < 1e-13
    for level in range(1, g.num_levels):
        lo = oracle.level_offset(64, level)
        cnt = 64 >> level
        shift = scale * np.einsum("bhud,d->bhu", Q[:, :, lo:lo + cnt].astype(np.float64),
                                  Rel[level, g.k + 1].astype(np.float64))
        assert np.abs((lse0 - lse1)[:, :, lo:lo + cnt] - shift).max() < 1e-12
    assert np.abs((lse0 - lse1)[:, :, :64]).max() == 0
    # backward identities: d r_anc = 0; column sums of dV equal those of dO
    dQ, dK, dV, dRel, _ = oracle.attn_bwd(g, Q, K, V, Rel, dO, scale)
    assert np.abs(dRel[1:, g.k + 1]).max() < 1e-12
    assert np.abs(dV.sum(2) - dO.astype(np.float64).sum(2)).max() < 1e-11
    # slots the graph never uses receive no gradient
    used = np.zeros(g.num_levels * g.rel_width, dtype=bool)
    used[g.rel] = True
    assert np.all(dRel.reshape(-1, 8)[~used] == 0)


@pytest.mark.parametrize("n,k,causal", [(32, 2, False), (64, 3, True)])
def test_zero_queries_give_uniform_attention_in_closed_form(n, k, causal):
    # with q_u = 0 every score is 0: lse_u = ln deg(u), out_u = the mean of the neighbours' values, and by the
    # chain rule dV_v = sum over the rows u that read v of dO_u / deg(u), dS_e = (dO_u . v_e - dO_u . out_u) / deg(u),
    # dQ_u = scale * sum_e dS_e (k_e + r_e), dK = 0 and d_rel = 0 (both carry a factor q_u)
    g = oracle.build_graph(n, k, causal)
    Q, K, V, Rel, dO = rand_inputs(g, 1, 2, 8, seed=12)
    Q[:] = 0
    scale = 0.25
    out, lse, _ = oracle.attn_fwd(g, Q, K, V, Rel, scale)
    dQ, dK, dV, dRel, _ = oracle.attn_bwd(g, Q, K, V, Rel, dO, scale)
    deg = np.diff(g.row_ptr)
    assert np.abs(lse - np.log(deg)[None, None, :]).max() < 1e-13
    V64, K64, dO64, R64 = (a.astype(np.float64) for a in (V, K, dO, Rel.reshape(-1, Rel.shape[-1])))
    want_out, want_dV, want_dQ = np.zeros_like(V64), np.zeros_like(V64), np.zeros_like(V64)
    for u in range(g.num_nodes):
        e = slice(g.row_ptr[u], g.row_ptr[u + 1])
        cols = g.col[e]
        want_out[:, :, u] = V64[:, :, cols].mean(2)
        np.add.at(want_dV, (slice(None), slice(None), cols), dO64[:, :, u:u + 1] / deg[u])
        dS = (np.einsum("bhd,bhed->bhe", dO64[:, :, u], V64[:, :, cols])
              - np.einsum("bhd,bhd->bh", dO64[:, :, u], want_out[:, :, u])[..., None]) / deg[u]
        want_dQ[:, :, u] = scale * np.einsum("bhe,bhed->bhd", dS, K64[:, :, cols] + R64[g.rel[e]][None, None])
    assert np.abs(out - want_out).max() < 1e-13
    assert np.abs(dV - want_dV).max() < 1e-12 and np.abs(dQ - want_dQ).max() < 1e-12
    assert np.abs(dK).max() == 0 and np.abs(dRel).max() == 0


def test_threads_do_not_change_the_result():
    w = shrink(WORKLOADS["cls"], B=2, H=2, n=64)
    g = oracle.build_graph(w.n, w.k, w.causal)
    x = make_inputs(w)
    a = oracle.attn_fwd(g, x["Q"], x["K"], x["V"], x["Rel"], w.scale, threads=1)
    b = oracle.attn_fwd(g, x["Q"], x["K"], x["V"], x["Rel"], w.scale, threads=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    ga = oracle.attn_bwd(g, x["Q"], x["K"], x["V"], x["Rel"], x["dO"], w.scale, threads=1)
    gb = oracle.attn_bwd(g, x["Q"], x["K"], x["V"], x["Rel"], x["dO"], w.scale, threads=4)
    for p, q in zip(ga[:4], gb[:4]):
        assert np.array_equal(p, q)


def test_workload_inputs_are_seeded_and_bf16_exact():
    w = shrink(WORKLOADS["lm"], B=1, H=1, n=32)
    a, b = make_inputs(w), make_inputs(w)
    for key in a:
        assert np.array_equal(a[key], b[key])
        bits = a[key].view(np.uint32)
        assert np.all(bits & 0xFFFF == 0)                   # representable in bfloat16
    t = torch.tensor(a["Q"]).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t, a["Q"])
    assert abs(a["Rel"].std() - 0.02) < 0.005 and abs(a["Q"].std() - 1.0) < 0.05


# ------------------------------------------------ batches of sequences of different lengths
def test_lengths_batch_equals_dense_attention_over_kept_nodes():
    # every batch entry: plain softmax attention (library routine) over the kept nodes of its own
    # length, forward and gradient; rows of nodes that are not kept give zeros everywhere
    n, k, D, scale = 32, 2, 8, 0.4
    lengths = [32, 1, 5, 17, 24]
    for causal in (False, True):
        g0 = oracle.build_graph(n, k, causal)
        Q, K, V, Rel, dO = rand_inputs(g0, len(lengths), 2, D, seed=91 + causal)
        out, lse, edges = oracle.attn_fwd_lengths(n, k, causal, lengths, Q, K, V, Rel, scale)
        dQ, dK, dV, dRel = oracle.attn_bwd_lengths(n, k, causal, lengths, Q, K, V, Rel, dO, scale)
        dRel_ref = np.zeros_like(dRel)
        assert edges == sum(oracle.build_graph_len(n, x, k, causal).num_edges for x in lengths)
        for b, length in enumerate(lengths):
            g = oracle.build_graph_len(n, length, k, causal)
            rows = np.flatnonzero(np.diff(g.row_ptr) > 0)
            gone = np.flatnonzero(np.diff(g.row_ptr) == 0)
            mask, ids = dense_mask_and_ids(g)
            Qt, Kt, Vt = (torch.tensor(x[b:b + 1], dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
            Rt = torch.tensor(Rel, dtype=torch.float64, requires_grad=True)
            R = Rt.reshape(-1, D)[torch.tensor(ids[rows])]
            bias = scale * torch.einsum("bhud,uvd->bhuv", Qt[:, :, rows], R)
            bias = bias.masked_fill(~torch.tensor(mask[rows]), float("-inf"))
            o = torch.nn.functional.scaled_dot_product_attention(Qt[:, :, rows], Kt, Vt, attn_mask=bias, scale=scale)
            o.backward(torch.tensor(dO[b:b + 1, :, rows], dtype=torch.float64))
            assert np.abs(out[b:b + 1, :, rows] - o.detach().numpy()).max() < 1e-12
            for got, leaf in zip((dQ, dK, dV), (Qt, Kt, Vt)):
                assert np.abs(got[b:b + 1] - leaf.grad.numpy()).max() < 1e-11
            dRel_ref += Rt.grad.numpy()
            for t in (out, lse, dQ, dK, dV):
                assert np.all(t[b][:, gone] == 0)
        assert np.abs(dRel - dRel_ref).max() < 1e-11


def test_power_of_two_length_runs_the_smaller_tree():
    # a sequence of p = 2^a tokens padded to n gives, on the nodes of the tree over p, exactly
    # what the graph of the paper over p gives (oracle functions already pinned above)
    n, p, k, D, scale = 64, 16, 2, 8, 0.3
    for causal in (False, True):
        small = oracle.build_graph(p, k, causal)
        big0 = oracle.build_graph(n, k, causal)
        Q, K, V, Rel, dO = rand_inputs(big0, 1, 2, D, seed=13)
        idx = np.concatenate([oracle.level_offset(n, l) + np.arange(p >> l) for l in range(small.num_levels)])
        sub = lambda x: np.ascontiguousarray(x[:, :, idx])
        Rs = np.ascontiguousarray(Rel[:small.num_levels])
        o_s, l_s, _ = oracle.attn_fwd(small, sub(Q), sub(K), sub(V), Rs, scale)
        g_s = oracle.attn_bwd(small, sub(Q), sub(K), sub(V), Rs, sub(dO), scale)
        o_b, l_b, _ = oracle.attn_fwd_lengths(n, k, causal, [p], Q, K, V, Rel, scale)
        # gradient of the nodes of the smaller tree only: the chain above its root gets no dO
        dO2 = np.zeros_like(dO)
        dO2[:, :, idx] = dO[:, :, idx]
        g_b = oracle.attn_bwd_lengths(n, k, causal, [p], Q, K, V, Rel, dO2, scale)
        assert np.abs(o_b[:, :, idx] - o_s).max() < 1e-13 and np.abs(l_b[:, :, idx] - l_s).max() < 1e-13
        for a, b in zip(g_b[:3], g_s[:3]):
            assert np.abs(a[:, :, idx] - b).max() < 1e-12
        assert np.abs(g_b[3][:small.num_levels] - g_s[3]).max() < 1e-12
        # each node of the chain above sees the same tokens as the root of the smaller tree
        root = oracle.level_offset(n, small.num_levels - 1)
        for level in range(small.num_levels, big0.num_levels):
            u = oracle.level_offset(n, level)
            Q2 = Q.copy()
            Q2[:, :, u] = Q[:, :, root]
            o2, _, _ = oracle.attn_fwd_lengths(n, k, causal, [p], Q2, K, V, Rel, scale)
            assert np.abs(o2[:, :, u] - o_b[:, :, root]).max() < 1e-13


def test_rows_that_are_not_kept_have_no_influence():
    n, k, D, scale = 64, 3, 8, 0.25
    lengths = [37, 64, 2]
    g0 = oracle.build_graph(n, k, False)
    Q, K, V, Rel, dO = rand_inputs(g0, 3, 1, D, seed=4)
    a = oracle.attn_fwd_lengths(n, k, False, lengths, Q, K, V, Rel, scale)[:2] + \
        oracle.attn_bwd_lengths(n, k, False, lengths, Q, K, V, Rel, dO, scale)
    rng = np.random.default_rng(1)
    Q2, K2, V2, dO2 = (x.copy() for x in (Q, K, V, dO))
    for b, length in enumerate(lengths):
        gone = np.flatnonzero(np.diff(oracle.build_graph_len(n, length, k, False).row_ptr) == 0)
        for x in (Q2, K2, V2, dO2):
            x[b, :, gone] = rng.standard_normal((len(gone), 1, D)).astype(np.float32) * 100
    b2 = oracle.attn_fwd_lengths(n, k, False, lengths, Q2, K2, V2, Rel, scale)[:2] + \
        oracle.attn_bwd_lengths(n, k, False, lengths, Q2, K2, V2, Rel, dO2, scale)
    for x, y in zip(a, b2):
        assert np.array_equal(x, y)


# ------------------------------------------------ dropout on the attention weights
def keep_mask(g, B, H, p, seed):
    """The documented mask, restated with numpy uint32 arithmetic: [B*H, N, N] of 0 / 1/(1-p)."""
    def mix(z):
        z = z ^ (z >> np.uint32(16))
        z = z * np.uint32(0x7FEB352D)
        z = z ^ (z >> np.uint32(15))
        z = z * np.uint32(0x846CA68B)
        return z ^ (z >> np.uint32(16))
    N = g.num_nodes
    thr = np.uint32(min(int(np.floor(p * 2.0 ** 32)), 2 ** 32 - 1))
    M = np.zeros((B * H, N, N))
    with np.errstate(over="ignore"):
        for bh in range(B * H):
            h0 = mix(np.uint32(seed) ^ (np.uint32(0x9E3779B9) * np.uint32(bh)))
            for u in range(N):
                b, e = g.row_ptr[u], g.row_ptr[u + 1]
                cols, rels = g.col[b:e].astype(np.uint32), g.rel[b:e].astype(np.uint32)
                x = rels if u < g.n else np.uint32(0x80000000) + cols
                r = mix(mix(h0 + np.uint32(u)) + x)
                M[bh, u, g.col[b:e]] = np.where(r >= thr, 1.0 / (1.0 - p), 0.0)
    return M.reshape(B, H, N, N)


@pytest.mark.parametrize("n,k,causal,p", [(16, 2, False, 0.1), (32, 3, True, 0.5), (8, 1, False, 0.9)])
def test_dropout_equals_dense_attention_with_the_documented_mask(n, k, causal, p):
    g = oracle.build_graph(n, k, causal)
    B, H, D = 2, 2, 8
    Q, K, V, Rel, dO = rand_inputs(g, B, H, D, seed=n + 3)
    scale, seed = 0.3, 123456789
    M = keep_mask(g, B, H, p, seed)
    mask, ids = dense_mask_and_ids(g)
    Qt, Kt, Vt = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    Rt = torch.tensor(Rel, dtype=torch.float64, requires_grad=True)
    R = Rt.reshape(-1, D)[torch.tensor(ids)]
    S = scale * (torch.einsum("bhud,bhvd->bhuv", Qt, Kt) + torch.einsum("bhud,uvd->bhuv", Qt, R))
    S = S.masked_fill(~torch.tensor(mask), float("-inf"))
    P = torch.softmax(S, -1)
    out_t = (P * torch.tensor(M)) @ Vt
    out_t.backward(torch.tensor(dO, dtype=torch.float64))
    out, lse, _ = oracle.attn_fwd(g, Q, K, V, Rel, scale, dropout=p, seed=seed)
    grads = oracle.attn_bwd(g, Q, K, V, Rel, dO, scale, dropout=p, seed=seed)
    assert np.abs(out - out_t.detach().numpy()).max() < 1e-12
    assert np.abs(lse - torch.logsumexp(S, -1).detach().numpy()).max() < 1e-12      # lse is that of the full softmax
    for got, leaf in zip(grads[:4], (Qt, Kt, Vt, Rt)):
        assert np.abs(got - leaf.grad.numpy()).max() < 1e-11
    # the kept fraction is about 1 - p, and the mask differs between heads and between seeds
    edges = mask.sum() * B * H
    kept = (M > 0).sum() / edges
    assert abs(kept - (1 - p)) < 4 * np.sqrt(p * (1 - p) / edges) + 0.01
    assert not np.array_equal(M[0, 0], M[0, 1])
    assert not np.array_equal(M, keep_mask(g, B, H, p, seed + 1))


def test_dropout_zero_is_no_dropout_and_lengths_use_global_head_indices():
    g = oracle.build_graph(32, 2, False)
    Q, K, V, Rel, dO = rand_inputs(g, 3, 2, 8, seed=8)
    a = oracle.attn_fwd(g, Q, K, V, Rel, 0.2)[0]
    b = oracle.attn_fwd(g, Q, K, V, Rel, 0.2, dropout=0.0, seed=99)[0]
    assert np.array_equal(a, b)
    # a batch of full lengths through the per-entry path draws the same masks as one call
    c = oracle.attn_fwd(g, Q, K, V, Rel, 0.2, dropout=0.3, seed=5)[0]
    d = oracle.attn_fwd_lengths(32, 2, False, [32, 32, 32], Q, K, V, Rel, 0.2, dropout=0.3, seed=5)[0]
    assert np.array_equal(c, d)
    ga = oracle.attn_bwd(g, Q, K, V, Rel, dO, 0.2, dropout=0.3, seed=5)
    gb = oracle.attn_bwd_lengths(32, 2, False, [32, 32, 32], Q, K, V, Rel, dO, 0.2, dropout=0.3, seed=5)
    for x, y in zip(ga[:3], gb[:3]):
        assert np.array_equal(x, y)
    assert np.abs(ga[3] - gb[3]).max() < 1e-12


def test_dropout_is_unbiased_over_seeds():
    # inverted dropout: the mean of `out` over many masks is the `out` without dropout (a wrong scale,
    # or a mask that ignores the seed, fails this without reference to the hash itself)
    g = oracle.build_graph(16, 2, False)
    Q, K, V, Rel, _ = rand_inputs(g, 1, 2, 8, seed=21)
    want = oracle.attn_fwd(g, Q, K, V, Rel, 0.3)[0]
    p, seeds = 0.3, 600
    acc = np.zeros_like(want)
    for s in range(seeds):
        acc += oracle.attn_fwd(g, Q, K, V, Rel, 0.3, dropout=p, seed=1000 + 7 * s)[0]
    err = np.abs(acc / seeds - want)
    # per element: variance <= p/(1-p) * sum_e p_e^2 v_e^2 <= p/(1-p) * max|v|^2; 5 sigma of the mean
    bound = 5 * np.sqrt(p / (1 - p) / seeds) * np.abs(V).max()
    assert err.max() < bound, (err.max(), bound)
    assert err.mean() < bound / 5
