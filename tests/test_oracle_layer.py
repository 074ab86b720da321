"""Pins for the oracle of the graph layer (CPU only): library routines of torch for the dense parts
(linear maps, layer normalisation, ReLU), the already pinned attention oracle in between."""
import numpy as np
import pytest
import torch

import oracle
from oracle.layer import layer_forward, layer_norm


def make_params(rng, d, d_ff):
    s = 1.0 / np.sqrt(d)
    p = {w: (s * rng.standard_normal((d, d))).astype(np.float32) for w in ("Wq", "Wk", "Wv", "Wo")}
    p["W1"] = (s * rng.standard_normal((d, d_ff))).astype(np.float32)
    p["W2"] = (rng.standard_normal((d_ff, d)) / np.sqrt(d_ff)).astype(np.float32)
    p["b1"] = (0.1 * rng.standard_normal(d_ff)).astype(np.float32)
    p["b2"] = (0.1 * rng.standard_normal(d)).astype(np.float32)
    for g, b in (("g1", "beta1"), ("g2", "beta2")):
        p[g] = (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32)
        p[b] = (0.1 * rng.standard_normal(d)).astype(np.float32)
    return p


def test_layer_norm_is_the_library_routine():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 7, 128))
    g, b = rng.standard_normal(128), rng.standard_normal(128)
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (128,), torch.tensor(g), torch.tensor(b), 1e-5).numpy()
    assert np.abs(layer_norm(x, g, b, 1e-5) - ref).max() < 1e-12
    # a zero row (a span node before the first layer, Sec. 3.3) gives the bias
    assert np.abs(layer_norm(np.zeros((1, 128)), g, b, 1e-5) - b).max() == 0


def test_layer_equals_torch_composition():
    n, k, heads, d_ff = 32, 2, 2, 256
    d = heads * 64
    for causal in (False, True):
        rng = np.random.default_rng(5 + causal)
        g = oracle.build_graph(n, k, causal)
        X = rng.standard_normal((2, g.num_nodes, d)).astype(np.float32)
        X[:, n:] = 0                                           # span nodes start from zero
        Rel = (0.02 * rng.standard_normal((g.num_levels, g.rel_width, 64))).astype(np.float32)
        p = make_params(rng, d, d_ff)
        Y = layer_forward(n, k, causal, heads, X, Rel, p, 0.125)
        t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
        Xt = t(X)
        lin = torch.nn.functional.linear
        Q, K, V = (lin(Xt, t(p[w]).T).reshape(2, -1, heads, 64).permute(0, 2, 1, 3) for w in ("Wq", "Wk", "Wv"))
        out, _, _ = oracle.attn_fwd(g, Q.numpy().astype(np.float32), K.numpy().astype(np.float32),
                                    V.numpy().astype(np.float32), Rel, 0.125)
        O = t(out).permute(0, 2, 1, 3).reshape(2, -1, d)
        ln = torch.nn.functional.layer_norm
        Z = ln(Xt + lin(O, t(p["Wo"]).T), (d,), t(p["g1"]), t(p["beta1"]), 1e-5)
        F = lin(torch.relu(lin(Z, t(p["W1"]).T, t(p["b1"]))), t(p["W2"]).T, t(p["b2"]))
        ref = ln(Z + F, (d,), t(p["g2"]), t(p["beta2"]), 1e-5).numpy()
        assert np.abs(Y - ref).max() < 1e-6                    # the attention oracle takes float32 inputs


def test_k_at_least_n_is_a_transformer_encoder_layer_over_the_tokens():
    # Sec. 3.3: attending to all token nodes recovers the vanilla Transformer -- with the relative
    # positions zero, token rows of the layer equal torch's post-norm encoder layer
    n, heads, d_ff = 16, 2, 128
    d = heads * 64
    rng = np.random.default_rng(9)
    g = oracle.build_graph(n, n, False)
    X = rng.standard_normal((1, g.num_nodes, d)).astype(np.float32)
    Rel = np.zeros((g.num_levels, g.rel_width, 64), dtype=np.float32)
    p = make_params(rng, d, d_ff)
    Y = layer_forward(n, n, False, heads, X, Rel, p, 0.125)
    enc = torch.nn.TransformerEncoderLayer(d, heads, d_ff, dropout=0.0, activation="relu", batch_first=True,
                                           norm_first=False, dtype=torch.float64)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        enc.self_attn.in_proj_weight.copy_(torch.cat([t(p["Wq"]).T, t(p["Wk"]).T, t(p["Wv"]).T]))
        enc.self_attn.in_proj_bias.zero_()
        enc.self_attn.out_proj.weight.copy_(t(p["Wo"]).T)
        enc.self_attn.out_proj.bias.zero_()
        enc.linear1.weight.copy_(t(p["W1"]).T)
        enc.linear1.bias.copy_(t(p["b1"]))
        enc.linear2.weight.copy_(t(p["W2"]).T)
        enc.linear2.bias.copy_(t(p["b2"]))
        enc.norm1.weight.copy_(t(p["g1"]))
        enc.norm1.bias.copy_(t(p["beta1"]))
        enc.norm2.weight.copy_(t(p["g2"]))
        enc.norm2.bias.copy_(t(p["beta2"]))
        ref = enc(t(X[:, :n])).numpy()
    assert np.abs(Y[:, :n] - ref).max() < 1e-6


# ------------------------------------------------------------------ backward of the layer
from oracle.layer import kept_rows, layer_backward, layer_norm_backward   # noqa: E402

PARAMS = ("Wq", "Wk", "Wv", "Wo", "W1", "b1", "W2", "b2", "g1", "beta1", "g2", "beta2")


def test_layer_norm_backward_is_autograd_of_the_library_routine():
    rng = np.random.default_rng(1)
    s, dy = rng.standard_normal((4, 5, 128)), rng.standard_normal((4, 5, 128))
    g, b = 1 + 0.3 * rng.standard_normal(128), rng.standard_normal(128)
    st, gt, bt = (torch.tensor(a, requires_grad=True) for a in (s, g, b))
    torch.nn.functional.layer_norm(st, (128,), gt, bt, 1e-5).backward(torch.tensor(dy))
    ds, dg, db = layer_norm_backward(s, g, 1e-5, dy)
    assert np.abs(ds - st.grad.numpy()).max() < 1e-12
    assert np.abs(dg - gt.grad.numpy()).max() < 1e-12
    assert np.abs(db - bt.grad.numpy()).max() < 1e-12


def dense_graph_tables(graphs, N):
    """Per batch entry: [N, N] edge mask and relative-position ids, from the (pinned) graph builder."""
    masks, ids = [], []
    for g in graphs:
        m, i = np.zeros((N, N), dtype=bool), np.zeros((N, N), dtype=np.int64)
        for u in range(N):
            b, e = g.row_ptr[u], g.row_ptr[u + 1]
            m[u, g.col[b:e]] = True
            i[u, g.col[b:e]] = g.rel[b:e]
        masks.append(m)
        ids.append(i)
    return np.stack(masks), np.stack(ids)


def torch_layer(X, Rel, P, masks, ids, heads, scale, eps=1e-5):
    """The layer as a composition of torch routines, attention as a dense masked softmax over all nodes."""
    B, N, d = X.shape
    lin, ln = torch.nn.functional.linear, torch.nn.functional.layer_norm
    Q, K, V = (lin(X, P[w].T).reshape(B, N, heads, 64).permute(0, 2, 1, 3) for w in ("Wq", "Wk", "Wv"))
    R = Rel.reshape(-1, 64)[torch.tensor(ids)]                                   # [B, N, N, 64]
    S = scale * (torch.einsum("bhud,bhvd->bhuv", Q, K) + torch.einsum("bhud,buvd->bhuv", Q, R))
    S = S.masked_fill(~torch.tensor(masks)[:, None], float("-inf"))
    Pm = torch.softmax(S, -1)
    Pm = torch.where(torch.tensor(masks)[:, None], Pm, torch.zeros_like(Pm))   # rows without edges: zeros, not nan
    O = (Pm @ V).permute(0, 2, 1, 3).reshape(B, N, d)
    Z = ln(X + lin(O, P["Wo"].T), (d,), P["g1"], P["beta1"], eps)
    F = lin(torch.relu(lin(Z, P["W1"].T, P["b1"])), P["W2"].T, P["b2"])
    return ln(Z + F, (d,), P["g2"], P["beta2"], eps)


def check_against_autograd(n, k, causal, lengths, seed):
    heads, d_ff, B = 2, 192, 2
    d = heads * 64
    rng = np.random.default_rng(seed)
    g = oracle.build_graph(n, k, causal)
    N = g.num_nodes
    X = rng.standard_normal((B, N, d)).astype(np.float32)
    dY = rng.standard_normal((B, N, d)).astype(np.float32)
    Rel = (0.3 * rng.standard_normal((g.num_levels, g.rel_width, 64))).astype(np.float32)
    p = make_params(rng, d, d_ff)
    got = layer_backward(n, k, causal, heads, X, Rel, p, dY, 0.125, lengths=lengths)
    graphs = [g] * B if lengths is None else [oracle.build_graph_len(n, L, k, causal) for L in lengths]
    masks, ids = dense_graph_tables(graphs, N)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    Xt, Rt, P = t(X), t(Rel), {w: t(p[w]) for w in PARAMS}
    Y = torch_layer(Xt, Rt, P, masks, ids, heads, 0.125)
    dYt = torch.tensor(dY.astype(np.float64))
    if lengths is not None:
        dYt = dYt * torch.tensor(kept_rows(n, lengths))[:, :, None]
    Y.backward(dYt)
    ref = {"dX": Xt.grad, "dRel": Rt.grad}
    ref.update({"d" + w: P[w].grad for w in PARAMS})
    assert sorted(got) == sorted(ref)
    for name, r in ref.items():
        r = r.numpy()
        # the attention oracle rounds its inputs to float32: 1e-7 relative
        assert np.abs(got[name] - r).max() <= 2e-5 * max(1.0, np.abs(r).max()), name
    return got


def test_layer_backward_equals_autograd_through_a_dense_composition():
    check_against_autograd(16, 2, False, None, 3)
    check_against_autograd(32, 3, True, None, 4)


def test_layer_backward_with_lengths():
    got = check_against_autograd(32, 2, False, [32, 11], 5)
    gone = ~kept_rows(32, [32, 11])
    assert gone[1].sum() > 0 and np.abs(got["dX"][gone]).max() == 0      # rows a sequence does not keep get no gradient


def test_layer_backward_for_k_at_least_n_is_the_transformer_encoder_layer():
    # Sec. 3.3 again: with gradients arriving at the token rows only, the token rows and all parameters
    # get the gradients of torch's post-norm encoder layer
    n, heads, d_ff = 16, 2, 128
    d = heads * 64
    rng = np.random.default_rng(10)
    g = oracle.build_graph(n, n, False)
    X = rng.standard_normal((1, g.num_nodes, d)).astype(np.float32)
    dY = rng.standard_normal((1, g.num_nodes, d)).astype(np.float32)
    dY[:, n:] = 0
    Rel = np.zeros((g.num_levels, g.rel_width, 64), dtype=np.float32)
    p = make_params(rng, d, d_ff)
    got = layer_backward(n, n, False, heads, X, Rel, p, dY, 0.125)
    enc = torch.nn.TransformerEncoderLayer(d, heads, d_ff, dropout=0.0, activation="relu", batch_first=True,
                                           norm_first=False, dtype=torch.float64)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        enc.self_attn.in_proj_weight.copy_(torch.cat([t(p["Wq"]).T, t(p["Wk"]).T, t(p["Wv"]).T]))
        enc.self_attn.in_proj_bias.zero_()
        enc.self_attn.out_proj.weight.copy_(t(p["Wo"]).T)
        enc.self_attn.out_proj.bias.zero_()
        enc.linear1.weight.copy_(t(p["W1"]).T)
        enc.linear1.bias.copy_(t(p["b1"]))
        enc.linear2.weight.copy_(t(p["W2"]).T)
        enc.linear2.bias.copy_(t(p["b2"]))
        enc.norm1.weight.copy_(t(p["g1"]))
        enc.norm1.bias.copy_(t(p["beta1"]))
        enc.norm2.weight.copy_(t(p["g2"]))
        enc.norm2.bias.copy_(t(p["beta2"]))
    Xt = t(X[:, :n]).requires_grad_(True)
    enc(Xt).backward(t(dY[:, :n]))
    tol = lambda r: 2e-5 * max(1.0, float(np.abs(r).max()))
    close = lambda a, r: np.abs(a - r).max() <= tol(r)
    assert close(got["dX"][:, :n], Xt.grad.numpy())
    wq, wk, wv = (w.numpy().T for w in enc.self_attn.in_proj_weight.grad.split(d))
    assert close(got["dWq"], wq) and close(got["dWk"], wk) and close(got["dWv"], wv)
    assert close(got["dWo"], enc.self_attn.out_proj.weight.grad.numpy().T)
    assert close(got["dW1"], enc.linear1.weight.grad.numpy().T) and close(got["db1"], enc.linear1.bias.grad.numpy())
    assert close(got["dW2"], enc.linear2.weight.grad.numpy().T) and close(got["db2"], enc.linear2.bias.grad.numpy())
    assert close(got["dg1"], enc.norm1.weight.grad.numpy()) and close(got["dbeta1"], enc.norm1.bias.grad.numpy())
    assert close(got["dg2"], enc.norm2.weight.grad.numpy()) and close(got["dbeta2"], enc.norm2.bias.grad.numpy())


# ------------------------------------------------------------------ the stack of layers (Sec. 3.3, the whole loop)
from oracle.layer import stack_backward, stack_forward   # noqa: E402


def encoder_like(p, d, heads, d_ff):
    """torch's post-norm encoder layer carrying the parameters p (float64)."""
    enc = torch.nn.TransformerEncoderLayer(d, heads, d_ff, dropout=0.0, activation="relu", batch_first=True,
                                           norm_first=False, dtype=torch.float64)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        enc.self_attn.in_proj_weight.copy_(torch.cat([t(p["Wq"]).T, t(p["Wk"]).T, t(p["Wv"]).T]))
        enc.self_attn.in_proj_bias.zero_()
        enc.self_attn.out_proj.weight.copy_(t(p["Wo"]).T)
        enc.self_attn.out_proj.bias.zero_()
        for mod, w, b in ((enc.linear1, "W1", "b1"), (enc.linear2, "W2", "b2")):
            mod.weight.copy_(t(p[w]).T)
            mod.bias.copy_(t(p[b]))
        for mod, w, b in ((enc.norm1, "g1", "beta1"), (enc.norm2, "g2", "beta2")):
            mod.weight.copy_(t(p[w]))
            mod.bias.copy_(t(p[b]))
    return enc


def test_stack_for_k_at_least_n_is_a_stack_of_transformer_encoder_layers():
    # Sec. 3.3: with every token attending to all tokens the token rows are the vanilla Transformer's, layer
    # after layer (the span rows change from layer to layer but no token reads them); forward and backward
    n, heads, d_ff, layers = 16, 2, 128, 3
    d = heads * 64
    rng = np.random.default_rng(21)
    g = oracle.build_graph(n, n, False)
    E = rng.standard_normal((2, n, d)).astype(np.float32)
    d_tokens = rng.standard_normal((2, n, d)).astype(np.float32)
    Rels = [np.zeros((g.num_levels, g.rel_width, 64), dtype=np.float32)] * layers
    params = [make_params(rng, d, d_ff) for _ in range(layers)]
    root, tokens, states = stack_forward(n, n, False, heads, E, Rels, params, 0.125)
    assert len(states) == layers + 1 and np.abs(states[0][:, n:]).max() == 0 and np.array_equal(states[0][:, :n], E)
    encs = [encoder_like(p, d, heads, d_ff) for p in params]
    Et = torch.tensor(E.astype(np.float64), requires_grad=True)
    x = Et
    for enc in encs:
        x = enc(x)
    assert np.abs(tokens - x.detach().numpy()).max() < 1e-5
    x.backward(torch.tensor(d_tokens.astype(np.float64)))
    dE, grads = stack_backward(n, n, False, heads, E, Rels, params, np.zeros((2, d)), d_tokens, 0.125)
    close = lambda a, r: np.abs(a - r).max() <= 5e-5 * max(1.0, float(np.abs(r).max()))
    assert close(dE, Et.grad.numpy())
    for gr, enc in zip(grads, encs):   # every layer's own parameters, first layer first
        wq, wk, wv = (w.numpy().T for w in enc.self_attn.in_proj_weight.grad.split(d))
        assert close(gr["dWq"], wq) and close(gr["dWk"], wk) and close(gr["dWv"], wv)
        assert close(gr["dWo"], enc.self_attn.out_proj.weight.grad.numpy().T)
        assert close(gr["dW1"], enc.linear1.weight.grad.numpy().T) and close(gr["db1"], enc.linear1.bias.grad.numpy())
        assert close(gr["dW2"], enc.linear2.weight.grad.numpy().T) and close(gr["db2"], enc.linear2.bias.grad.numpy())
        assert close(gr["dg1"], enc.norm1.weight.grad.numpy()) and close(gr["dbeta1"], enc.norm1.bias.grad.numpy())
        assert close(gr["dg2"], enc.norm2.weight.grad.numpy()) and close(gr["dbeta2"], enc.norm2.bias.grad.numpy())


@pytest.mark.parametrize("n,k,causal,lengths", [(16, 2, False, None), (16, 1, True, None), (16, 2, False, [16, 7])])
def test_stack_backward_equals_autograd_through_dense_compositions(n, k, causal, lengths):
    # root and token outputs, span rows carried from layer to layer: autograd through the dense composition of
    # every layer (the library routines of torch), from the zero-initialised span rows to both outputs
    heads, d_ff, B, layers = 1, 96, 2, 2
    d = heads * 64
    rng = np.random.default_rng(31 + n + k)
    g = oracle.build_graph(n, k, causal)
    N = g.num_nodes
    E = rng.standard_normal((B, n, d)).astype(np.float32)
    d_root = rng.standard_normal((B, d)).astype(np.float32)
    d_tokens = rng.standard_normal((B, n, d)).astype(np.float32)
    Rels = [(0.3 * rng.standard_normal((g.num_levels, g.rel_width, 64))).astype(np.float32) for _ in range(layers)]
    params = [make_params(rng, d, d_ff) for _ in range(layers)]
    root, tokens, _ = stack_forward(n, k, causal, heads, E, Rels, params, 0.125, lengths=lengths)
    dE, grads = stack_backward(n, k, causal, heads, E, Rels, params, d_root, d_tokens, 0.125, lengths=lengths)

    graphs = [g] * B if lengths is None else [oracle.build_graph_len(n, L, k, causal) for L in lengths]
    masks, ids = dense_graph_tables(graphs, N)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    Et, Rt, Pt = t(E), [t(r) for r in Rels], [{w: t(p[w]) for w in PARAMS} for p in params]
    x = torch.cat([Et, torch.zeros((B, N - n, d), dtype=torch.float64)], 1)
    for R, P in zip(Rt, Pt):
        x = torch_layer(x, R, P, masks, ids, heads, 0.125)
    keep = torch.tensor(kept_rows(n, lengths if lengths is not None else [n] * B))
    assert np.abs(root - x[:, N - 1].detach().numpy()).max() < 1e-5
    assert np.abs((tokens - x[:, :n].detach().numpy())[keep[:, :n].numpy()]).max() < 1e-5
    loss = (x[:, N - 1] * torch.tensor(d_root.astype(np.float64))).sum() + \
           (x[:, :n] * torch.tensor(d_tokens.astype(np.float64)) * keep[:, :n, None]).sum()
    loss.backward()
    close = lambda a, r: np.abs(a - r).max() <= 5e-5 * max(1.0, float(np.abs(r).max()))
    assert close(dE, Et.grad.numpy())
    for gr, R, P in zip(grads, Rt, Pt):
        assert close(gr["dRel"], R.grad.numpy())
        for w in PARAMS:
            assert close(gr["d" + w], P[w].grad.numpy()), w
