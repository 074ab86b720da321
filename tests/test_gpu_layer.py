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


# ---------------------------------------------------------------------------------- backward
# Tolerance of the backward.  Every gradient is compared as max-abs error relative to the largest entry of
# the oracle's tensor: gradients of parameters are sums over all node rows and have no natural absolute
# scale.  Between the dense maps every activation and every gradient is rounded to bf16 once (2^-9
# relative, independent) and the stored activations differ from the oracle's by the forward's error.
#
# The gate of the ReLU is a decision taken from floating-point values: a hidden unit whose pre-activation
# lies within the forward's error of zero can be on in the kernel and off in the oracle.  A flipped unit
# changes its gradient by all of it, not by a rounding error; with a fraction f of flipped units the sums
# over them (db1, dW1, and everything downstream of the FFN branch: dX, the attention's gradients) are off
# by about sqrt(f) of their size -- measured 3..10 % with N(0, 0.1^2) biases, where f is about 0.3 %.
# So the cases come in two kinds:
#  * `decisive`: b1 = +6 or -6 by column, which puts every pre-activation (unit variance) six deviations
#    from zero; both sides then take the same gate, half of the units on, and what remains is rounding:
#    measured 0.1..0.6 % of the largest entry, bound 1.5 %;
#  * ordinary biases: the gradients that do not pass through the gate's derivative (dW2, db2, dg2, dbeta2: they
#    are formed from dY, the stored sums and the hidden activations themselves, which are continuous in the
#    pre-activation) keep the bound of the decisive cases, 1.5 % (measured 0.2..0.4 %); the others get 15 %
#    (measured 2..10 %, the sqrt(f) above), which still separates a correct backward from a wrong operand,
#    transpose or sign (those give errors of the order of the tensor itself).  A bound that holds for every
#    choice of the ambiguous gates (the sum of the absolute contributions of all units within the forward's
#    error of zero) exceeds the tensors themselves for sums over a thousand rows, so it would check nothing.
from oracle.layer import kept_rows, layer_backward   # noqa: E402

BWD_TOL_DECISIVE, BWD_TOL_ORDINARY = 1.5e-2, 15e-2
GATE_FREE = ("dW2", "db2", "dg2", "dbeta2")   # no factor of the ReLU's derivative in them
GRADS = ("dWq", "dWk", "dWv", "dWo", "dW1", "db1", "dW2", "db2", "dg1", "dbeta1", "dg2", "dbeta2")


@pytest.mark.parametrize("n,k,causal,B,heads,d_ff,lengths,decisive", [
    (64, 2, False, 2, 1, 64, None, True), (256, 4, True, 2, 2, 256, None, True), (512, 4, False, 2, 8, 2048, None, True),
    (256, 3, False, 3, 4, 512, [256, 150, 31], True), (1024, 8, True, 1, 8, 1024, None, True),
    (256, 4, True, 2, 2, 256, None, False), (256, 3, False, 3, 4, 512, [256, 150, 31], False),
])
def test_layer_backward(n, k, causal, B, heads, d_ff, lengths, decisive):
    print("layer backward", n, k, causal, B, heads, d_ff, lengths, decisive, flush=True)
    X, Rel, p = make_case(n, k, causal, B, heads, d_ff, 300 + n + heads, False)
    if decisive:
        p["b1"] = np.where(np.arange(d_ff) % 2 == 0, 6.0, -6.0).astype(np.float32)
    rng = np.random.Generator(np.random.PCG64(77 + n))
    dY = round_to_bf16(rng.standard_normal(X.shape).astype(np.float32))[0]
    g = bpt.bpt_build_graph(n, k, causal)
    lens_d = torch.tensor(lengths, dtype=torch.int32, device="cuda") if lengths else None
    fws, bws = bpt.layer_workspace_bytes(g, B, heads, d_ff)
    ws_f = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")
    Xd, Rd, pd = torch.from_numpy(X).to(torch.bfloat16).cuda(), torch.from_numpy(Rel).to(torch.bfloat16).cuda(), to_dev(p)
    bpt.bpt_layer_fwd(g, Xd, Rd, pd, heads, scale=0.125, seq_len=lens_d, workspace=ws_f)
    dX, d_rel, grads = bpt.bpt_layer_bwd(g, Xd, Rd, pd, heads, ws_f, torch.from_numpy(dY).to(torch.bfloat16).cuda(),
                                         scale=0.125, seq_len=lens_d, workspace=ws_b)
    torch.cuda.synchronize()
    ref = layer_backward(n, k, causal, heads, X, Rel, p, dY, 0.125, lengths=lengths)
    got = {"dX": dX, "dRel": d_rel}
    got.update(grads)
    worst = {}
    for name in ("dX", "dRel") + GRADS:
        a = got[name].float().cpu().numpy().astype(np.float64)
        assert np.isfinite(a).all(), name
        top = float(np.abs(ref[name]).max())
        worst[name] = float(np.abs(a - ref[name]).max()) / max(top, 1e-30)
    print("   relative max-abs errors", {k_: float("%.2g" % v) for k_, v in worst.items()}, flush=True)
    for name, v in worst.items():
        tol = BWD_TOL_DECISIVE if decisive or name in GATE_FREE else BWD_TOL_ORDINARY
        assert v <= tol, (name, v)
    if lengths:   # rows of nodes a sequence does not keep get exactly no gradient
        gone = torch.from_numpy(~kept_rows(n, lengths)).cuda()
        assert float(dX.float()[gone].abs().max()) == 0.0
    # a second call with the same arguments gives the same bits (fixed-order sums; no atomics of ours)
    dX2, d_rel2, grads2 = bpt.bpt_layer_bwd(g, Xd, Rd, pd, heads, ws_f, torch.from_numpy(dY).to(torch.bfloat16).cuda(),
                                            scale=0.125, seq_len=lens_d, workspace=ws_b)
    assert torch.equal(dX, dX2) and torch.equal(d_rel, d_rel2)
    for name in ("db1", "db2", "dg1", "dbeta1", "dg2", "dbeta2"):
        assert torch.equal(grads[name], grads2[name]), name
    g.destroy()


def test_layer_on_either_gemm_library(monkeypatch):
    # The dense products run in hipBLASLt (bias + ReLU and the residual adds of the backward in the products' epilogues)
    # or, with BPT_LAYER_BLAS=rocblas, in rocBLAS with the library's own bias + ReLU and add kernels: the fallback for
    # a product hipBLASLt has no algorithm for.  Both against the oracle, forward and backward, and against each other.
    import os
    n, k, causal, B, heads, d_ff = 256, 4, True, 2, 2, 256
    X, Rel, p = make_case(n, k, causal, B, heads, d_ff, 911, False)
    p["b1"] = np.where(np.arange(d_ff) % 2 == 0, 6.0, -6.0).astype(np.float32)   # decided gates (see above)
    rng = np.random.Generator(np.random.PCG64(912))
    dY = round_to_bf16(rng.standard_normal(X.shape).astype(np.float32))[0]
    g = bpt.bpt_build_graph(n, k, causal)
    fws, bws = bpt.layer_workspace_bytes(g, B, heads, d_ff)
    Xd, Rd, pd = torch.from_numpy(X).to(torch.bfloat16).cuda(), torch.from_numpy(Rel).to(torch.bfloat16).cuda(), to_dev(p)
    dYd = torch.from_numpy(dY).to(torch.bfloat16).cuda()
    ref_y = layer_forward(n, k, causal, heads, X, Rel, p, 0.125)
    ref = layer_backward(n, k, causal, heads, X, Rel, p, dY, 0.125)
    results = {}
    for lib in ("hipblaslt", "rocblas"):
        monkeypatch.setenv("BPT_LAYER_BLAS", lib)
        assert os.environ["BPT_LAYER_BLAS"] == lib
        ws_f = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")
        bpt.bpt_profile_enable(True)
        Y = bpt.bpt_layer_fwd(g, Xd, Rd, pd, heads, scale=0.125, workspace=ws_f)
        dX, d_rel, grads = bpt.bpt_layer_bwd(g, Xd, Rd, pd, heads, ws_f, dYd, scale=0.125, workspace=ws_b)
        torch.cuda.synchronize()
        ran = set(bpt.bpt_profile_report())
        bpt.bpt_profile_enable(False)
        # the library's own bias + ReLU and add kernels run exactly when the products' epilogues do not do their work
        assert ("bias_relu_kernel" in ran) == (lib == "rocblas"), ran
        assert ("add_cast_kernel" in ran) == (lib == "rocblas"), ran
        err = np.abs(Y.float().cpu().numpy().astype(np.float64) - ref_y).max()
        assert err <= TOL, (lib, err)
        got = {"dX": dX, "dRel": d_rel}
        got.update(grads)
        for name in ("dX", "dRel") + GRADS:
            a = got[name].float().cpu().numpy().astype(np.float64)
            v = float(np.abs(a - ref[name]).max()) / max(float(np.abs(ref[name]).max()), 1e-30)
            assert np.isfinite(a).all() and v <= BWD_TOL_DECISIVE, (lib, name, v)
        results[lib] = (Y.float().cpu().numpy(), dX.float().cpu().numpy())
    # the two paths differ by roundings only (bias + ReLU on fp32 sums or on bf16 values, one or two roundings of dX)
    assert np.abs(results["hipblaslt"][0] - results["rocblas"][0]).max() <= TOL
    top = np.abs(results["rocblas"][1]).max()
    assert np.abs(results["hipblaslt"][1] - results["rocblas"][1]).max() <= BWD_TOL_DECISIVE * top
    g.destroy()


@pytest.mark.parametrize("n,k,causal,heads,d_ff,lengths", [
    (256, 3, False, 4, 512, [256, 150, 31, 1]), (512, 4, True, 2, 256, [77, 512, 300]),
])
def test_layer_on_the_graph_of_a_packed_batch(n, k, causal, heads, d_ff, lengths):
    # one graph for the batch, rows only for the nodes that exist (bpt_build_batch_graph): X, Y, dY, dX are
    # [1][rows][d]; the oracle runs the padded trees with the lengths and is read at the kept rows
    print("layer on a packed batch", n, k, causal, heads, d_ff, lengths, flush=True)
    B = len(lengths)
    X, Rel, p = make_case(n, k, causal, B, heads, d_ff, 500 + n + heads, False)
    p["b1"] = np.where(np.arange(d_ff) % 2 == 0, 6.0, -6.0).astype(np.float32)
    rng = np.random.Generator(np.random.PCG64(78 + n))
    dY = round_to_bf16(rng.standard_normal(X.shape).astype(np.float32))[0]
    _, b_of, node_of = oracle.batch_rows(n, lengths)
    g = bpt.bpt_build_batch_graph(n, k, causal, lengths)
    assert g.num_nodes == len(b_of)
    Xp = torch.from_numpy(X[b_of, node_of][None]).to(torch.bfloat16).cuda().contiguous()
    dYp = torch.from_numpy(dY[b_of, node_of][None]).to(torch.bfloat16).cuda().contiguous()
    Rd, pd = torch.from_numpy(Rel).to(torch.bfloat16).cuda(), to_dev(p)
    fws, bws = bpt.layer_workspace_bytes(g, 1, heads, d_ff)
    ws_f = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")
    Y = bpt.bpt_layer_fwd(g, Xp, Rd, pd, heads, scale=0.125, workspace=ws_f)
    dX, d_rel, grads = bpt.bpt_layer_bwd(g, Xp, Rd, pd, heads, ws_f, dYp, scale=0.125, workspace=ws_b)
    torch.cuda.synchronize()
    ref_y = layer_forward(n, k, causal, heads, X, Rel, p, 0.125, lengths=lengths)
    err = float(np.abs(Y.float().cpu().numpy()[0].astype(np.float64) - ref_y[b_of, node_of]).max())
    print("   forward max-abs error %.3g" % err, flush=True)
    assert err <= TOL, err
    ref = layer_backward(n, k, causal, heads, X, Rel, p, dY, 0.125, lengths=lengths)
    ref["dX"] = ref["dX"][b_of, node_of][None]
    got = {"dX": dX, "dRel": d_rel}
    got.update(grads)
    worst = {}
    for name in ("dX", "dRel") + GRADS:
        a = got[name].float().cpu().numpy().astype(np.float64)
        assert np.isfinite(a).all() and a.shape == ref[name].shape, name
        worst[name] = float(np.abs(a - ref[name]).max()) / max(float(np.abs(ref[name]).max()), 1e-30)
    print("   relative max-abs errors", {k_: float("%.2g" % v) for k_, v in worst.items()}, flush=True)
    for name, v in worst.items():
        assert v <= BWD_TOL_DECISIVE, (name, v)
    g.destroy()


def test_misaligned_tensors_are_refused():
    # the kernels move 16 bytes per lane: a tensor that starts 2 bytes off is an error, not a fault
    n, k, B, heads, d_ff = 64, 2, 1, 1, 64
    X, Rel, p = make_case(n, k, False, B, heads, d_ff, 5, True)
    g = bpt.bpt_build_graph(n, k, False)
    Rd, pd = torch.from_numpy(Rel).to(torch.bfloat16).cuda(), to_dev(p)
    flat = torch.zeros(X.size + 8, dtype=torch.bfloat16, device="cuda")
    Xd = flat[1:1 + X.size].view(X.shape)
    assert Xd.data_ptr() % 16 == 2 and Xd.is_contiguous()
    with pytest.raises(bpt.BptError):
        bpt.bpt_layer_fwd(g, Xd, Rd, pd, heads)
    bpt.bpt_layer_fwd(g, flat[8:8 + X.size].view(X.shape), Rd, pd, heads)     # 16 bytes off: fine
    torch.cuda.synchronize()
    g.destroy()
