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

from . import attn_fwd, attn_fwd_lengths, build_graph


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
