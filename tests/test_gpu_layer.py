"""GPU parity of the graph layer forward (Sec. 3.3) against its fp64 oracle.

Tolerance.  Y is a layer-normalised bf16 tensor with entries of magnitude up to about 4, so its own
rounding is up to 2^-8 * 4 / 2 = 8e-3.  Upstream, Q, K, V, the attention output, Z and the hidden FFN
activations are each rounded to bf16 once (relative 2^-9 per value) and enter sums of 128..2048
terms whose rounding errors add in quadrature; the second normalisation divides by a standard
deviation of order 1.  Measured maxima are 2e-2..3e-2; the bound used is 5e-2 absolute.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle.layer import layer_forward
from paper_1911_04070_amd import binding as bpt
from paper_1911_04070_amd.workloads import round_to_bf16

pytestmark = pytest.mark.gpu
TOL = 5e-2


def make_case(n, k, causal, B, heads, d_ff, seed, zero_spans):
    rng = np.random.Generator(np.random.PCG64(seed))
    d = heads * 64
    N = 2 * n - 1
    bf = lambda a: round_to_bf16(a.astype(np.float32))[0]
    X = bf(rng.standard_normal((B, N, d)))
    if zero_spans:
        X[:, n:] = 0                      # span nodes start from zero (Sec. 3.3)
    levels = n.bit_length()
    Rel = bf(0.02 * rng.standard_normal((levels, 2 * (k + 1) + 1, 64)))
    s = 1.0 / np.sqrt(d)
    p = {w: bf(s * rng.standard_normal((d, d))) for w in ("Wq", "Wk", "Wv", "Wo")}
    p["W1"] = bf(s * rng.standard_normal((d, d_ff)))
    p["W2"] = bf(rng.standard_normal((d_ff, d)) / np.sqrt(d_ff))
    p["b1"] = (0.1 * rng.standard_normal(d_ff)).astype(np.float32)
    p["b2"] = (0.1 * rng.standard_normal(d)).astype(np.float32)
    for g_, b_ in (("g1", "beta1"), ("g2", "beta2")):
        p[g_] = (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32)
        p[b_] = (0.1 * rng.standard_normal(d)).astype(np.float32)
    return X, Rel, p


def to_dev(p):
    return {k_: torch.from_numpy(v).to(torch.bfloat16 if k_.startswith("W") else torch.float32).cuda().contiguous()
            for k_, v in p.items()}


@pytest.mark.parametrize("n,k,causal,B,heads,d_ff,zero_spans,lengths", [
    (64, 2, False, 2, 1, 64, False, None), (256, 4, False, 2, 2, 256, True, None),
    (1024, 8, True, 1, 8, 2048, True, None), (512, 4, False, 3, 4, 512, False, [512, 300, 77]),
])
def test_layer_forward(n, k, causal, B, heads, d_ff, zero_spans, lengths):
    print("layer", n, k, causal, B, heads, d_ff, zero_spans, lengths, flush=True)
    X, Rel, p = make_case(n, k, causal, B, heads, d_ff, 100 + n + heads, zero_spans)
    g = bpt.bpt_build_graph(n, k, causal)
    lens_d = torch.tensor(lengths, dtype=torch.int32, device="cuda") if lengths else None
    Y = bpt.bpt_layer_fwd(g, torch.from_numpy(X).to(torch.bfloat16).cuda(), torch.from_numpy(Rel).to(torch.bfloat16).cuda(),
                          to_dev(p), heads, scale=0.125, seq_len=lens_d)
    torch.cuda.synchronize()
    ref = layer_forward(n, k, causal, heads, X, Rel, p, 0.125, lengths=lengths)
    got = Y.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    if lengths is None:
        err = np.abs(got - ref).max()
    else:   # rows of nodes that a shorter sequence does not keep are unspecified
        err = 0.0
        for b, length in enumerate(lengths):
            kept = np.diff(oracle.build_graph_len(n, length, k, causal).row_ptr) > 0
            err = max(err, float(np.abs(got[b][kept] - ref[b][kept]).max()))
    print("   max-abs error %.3g, |Y| max %.3g" % (err, np.abs(ref).max()), flush=True)
    assert err <= TOL, err
    g.destroy()
