"""CPU oracle for the graph layer around graph self-attention (test infrastructure only).

Sec. 3.1 and Sec. 3.3 (the update of the graph): for every node,
    Z  = norm(H + GSA(G, H)),      GSA = [head_1 .. head_h] W^O,  head_i from Q = H W_i^Q, K = H W_i^K, V = H W_i^V
    H' = norm(Z + FFN(Z)),         FFN(x) = max(0, x W_1 + b_1) W_2 + b_2   (position-wise, Vaswani et al.)
with layer normalisation (Ba et al.) over the feature dimension.  All nodes, tokens and spans,
are updated synchronously from the same H.  Everything is float64 numpy; the attention itself is
the oracle's per-node attention.  Readings: the projections carry no bias (the paper writes
H W); the normalisation has a gain and a bias per feature and divides by sqrt(var + eps) with the
biased variance; the i-th head uses columns [64 i, 64 i + 64) of the projected features.
"""
from __future__ import annotations

import numpy as np

from . import attn_bwd, attn_bwd_lengths, attn_fwd, attn_fwd_lengths, build_graph, level_offset, num_levels


def layer_norm(x: np.ndarray, gain: np.ndarray, bias: np.ndarray, eps: float) -> np.ndarray:
    x = x.astype(np.float64)
    mean = x.mean(-1, keepdims=True)
    var = ((x - mean) ** 2).mean(-1, keepdims=True)
    return (x - mean) / np.sqrt(var + eps) * gain.astype(np.float64) + bias.astype(np.float64)


def layer_forward(n, k, causal, heads, X, Rel, p, scale, eps=1e-5, lengths=None):
    """X: [B, N, d] with d = heads * 64; p: dict with Wq, Wk, Wv, Wo [d, d], W1 [d, d_ff], b1 [d_ff],
    W2 [d_ff, d], b2 [d], g1, beta1, g2, beta2 [d].  Returns H' [B, N, d] float64 (for a batch of
    sequences of different lengths only the rows of kept nodes mean anything)."""
    X = X.astype(np.float64)
    B, N, d = X.shape
    D = d // heads

    def split(t):   # [B, N, d] -> [B, heads, N, D]
        return np.ascontiguousarray(t.reshape(B, N, heads, D).transpose(0, 2, 1, 3))

    f64 = lambda a: np.asarray(a, dtype=np.float64)
    Q, K, V = (split(X @ f64(p[w])) for w in ("Wq", "Wk", "Wv"))
    # the attention oracle takes float inputs; give it exactly these values
    Q32, K32, V32 = (t.astype(np.float32) for t in (Q, K, V))
    if lengths is None:
        out, _, _ = attn_fwd(build_graph(n, k, causal), Q32, K32, V32, Rel, scale)
    else:
        out, _, _ = attn_fwd_lengths(n, k, causal, lengths, Q32, K32, V32, Rel, scale)
    O = out.transpose(0, 2, 1, 3).reshape(B, N, d)
    Z = layer_norm(X + O @ f64(p["Wo"]), p["g1"], p["beta1"], eps)
    F = np.maximum(Z @ f64(p["W1"]) + f64(p["b1"]), 0.0) @ f64(p["W2"]) + f64(p["b2"])
    return layer_norm(Z + F, p["g2"], p["beta2"], eps)


def kept_rows(n: int, lengths) -> np.ndarray:
    """[B, 2n-1] bool: node (l, m) of entry b holds a token of its sequence, m * 2^l < lengths[b]."""
    first = np.concatenate([np.arange(n >> l, dtype=np.int64) << l for l in range(num_levels(n))])
    assert first.shape[0] == 2 * n - 1 and level_offset(n, 1) == n
    return first[None, :] < np.asarray(lengths, dtype=np.int64)[:, None]


def layer_norm_backward(s, gain, eps, dy):
    """Gradient of y = norm(s) * gain + bias with respect to s, gain and bias (rows = all leading axes)."""
    mean = s.mean(-1, keepdims=True)
    r = 1.0 / np.sqrt(((s - mean) ** 2).mean(-1, keepdims=True) + eps)
    xh = (s - mean) * r
    dxh = dy * gain
    ds = r * (dxh - dxh.mean(-1, keepdims=True) - xh * (dxh * xh).mean(-1, keepdims=True))
    flat = lambda a: a.reshape(-1, a.shape[-1])
    return ds, (flat(dy) * flat(xh)).sum(0), flat(dy).sum(0)


def layer_backward(n, k, causal, heads, X, Rel, p, dY, scale, eps=1e-5, lengths=None):
    """Gradient of sum(H' * dY) of `layer_forward` with respect to X, the relative-position table and every
    parameter, by the chain rule through the steps of the forward in reverse (float64).  With `lengths`, the
    rows of dY of nodes a sequence does not keep are taken as zero.  Returns a dict: dX [B, N, d], dRel, dWq,
    dWk, dWv, dWo, dW1, db1, dW2, db2, dg1, dbeta1, dg2, dbeta2."""
    X = X.astype(np.float64)
    dY = dY.astype(np.float64)
    B, N, d = X.shape
    D = d // heads
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    W = {w: f64(p[w]) for w in ("Wq", "Wk", "Wv", "Wo", "W1", "W2")}
    if lengths is not None:
        dY = dY * kept_rows(n, lengths)[:, :, None]

    def split(t):   # [B, N, d] -> [B, heads, N, D]
        return np.ascontiguousarray(t.reshape(B, N, heads, D).transpose(0, 2, 1, 3))

    def join(t):    # back
        return t.transpose(0, 2, 1, 3).reshape(B, N, d)

    # forward, keeping what the backward needs
    Q32, K32, V32 = (split(X @ W[w]).astype(np.float32) for w in ("Wq", "Wk", "Wv"))
    if lengths is None:
        g = build_graph(n, k, causal)
        out, _, _ = attn_fwd(g, Q32, K32, V32, Rel, scale)
    else:
        out, _, _ = attn_fwd_lengths(n, k, causal, lengths, Q32, K32, V32, Rel, scale)
    O = join(out)
    S1 = X + O @ W["Wo"]
    Z = layer_norm(S1, p["g1"], p["beta1"], eps)
    Hpre = Z @ W["W1"] + f64(p["b1"])
    F = np.maximum(Hpre, 0.0)
    S2 = Z + F @ W["W2"] + f64(p["b2"])

    # backward
    res = {}
    rows = lambda a: a.reshape(-1, a.shape[-1])
    dS2, res["dg2"], res["dbeta2"] = layer_norm_backward(S2, f64(p["g2"]), eps, dY)
    res["db2"] = rows(dS2).sum(0)
    res["dW2"] = rows(F).T @ rows(dS2)
    dH = (dS2 @ W["W2"].T) * (Hpre > 0.0)
    res["db1"] = rows(dH).sum(0)
    res["dW1"] = rows(Z).T @ rows(dH)
    dZ = dS2 + dH @ W["W1"].T
    dS1, res["dg1"], res["dbeta1"] = layer_norm_backward(S1, f64(p["g1"]), eps, dZ)
    res["dWo"] = rows(O).T @ rows(dS1)
    dO = split(dS1 @ W["Wo"].T).astype(np.float32)   # the attention oracle takes float inputs
    if lengths is None:
        dQ, dK, dV, dRel, _ = attn_bwd(g, Q32, K32, V32, Rel, dO, scale)
    else:
        dQ, dK, dV, dRel = attn_bwd_lengths(n, k, causal, lengths, Q32, K32, V32, Rel, dO, scale)[:4]
    res["dRel"] = dRel
    dX = dS1.copy()
    for name, grad in (("Wq", dQ), ("Wk", dK), ("Wv", dV)):
        gj = join(grad)
        res["d" + name] = rows(X).T @ rows(gj)
        dX += gj @ W[name].T
    res["dX"] = dX
    return res


def initial_states(n: int, E: np.ndarray) -> np.ndarray:
    """Sec. 3.3: token nodes start from their embeddings E [B, n, d], span nodes from zero -> [B, 2n-1, d]."""
    B, _, d = E.shape
    H0 = np.zeros((B, 2 * n - 1, d), dtype=np.float64)
    H0[:, :n] = E
    return H0


def stack_forward(n, k, causal, heads, E, Rels, params, scale, eps=1e-5, lengths=None):
    """Sec. 3.3, the update of the graph: H^0 = initial states, H^i = layer_i(H^{i-1}) with each layer's own
    parameters params[i] and relative-position table Rels[i]; the output is the root's row of the last states
    (node 2n-2) and their token rows.  Returns (root [B, d], tokens [B, n, d], [H^0 .. H^layers])."""
    states = [initial_states(n, E)]
    for Rel, p in zip(Rels, params):
        states.append(layer_forward(n, k, causal, heads, states[-1], Rel, p, scale, eps, lengths))
    last = states[-1]
    return last[:, 2 * n - 2], last[:, :n], states


def stack_backward(n, k, causal, heads, E, Rels, params, d_root, d_tokens, scale, eps=1e-5, lengths=None):
    """Gradient of sum(root * d_root) + sum(tokens * d_tokens) of `stack_forward` with respect to the embeddings
    and every layer's table and parameters: `layer_backward` from the last layer to the first.  Returns (dE
    [B, n, d], list of the layers' gradient dicts, first layer first)."""
    _, _, states = stack_forward(n, k, causal, heads, E, Rels, params, scale, eps, lengths)
    dH = np.zeros_like(states[-1])
    dH[:, 2 * n - 2] = d_root
    dH[:, :n] = d_tokens
    grads = [None] * len(params)
    for i in range(len(params) - 1, -1, -1):
        grads[i] = layer_backward(n, k, causal, heads, states[i], Rels[i], params[i], dH, scale, eps, lengths)
        dH = grads[i]["dX"]
    return dH[:, :n], grads
