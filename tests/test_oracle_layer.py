"""Pins for the oracle of the graph layer (CPU only): library routines of torch for the dense parts
(linear maps, layer normalisation, ReLU), the already pinned attention oracle in between."""
import numpy as np
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
