"""GPU parity of the stack of graph layers (Sec. 3.3: the whole update of the graph, from the initial states to the
root's or the tokens' rows of the last layer) against its fp64 oracle, forward and backward.

Tolerances.  The states between layers are bf16 tensors on the GPU and fp64 in the oracle, so every layer adds
the error of one layer call (bounds of the layer's own tests: 5e-2 absolute on its layer-normalised output;
1.5 % / 15 % of the largest entry for gradients, without / with hidden units whose ReLU gate the two sides can
decide differently) to what it inherits; the normalisations keep the inherited part from growing.  The bounds
used are the layer's bounds times the number of layers (measured with three layers: forward 0.027..0.058;
gradients 1.5..2.1 % with decided gates, 7..13 % otherwise).  Next to that comparison the stack is checked bit for
bit against the same layers called one by one through the layer entry points, which is what it is made of.
"""
import numpy as np
import pytest
import torch

from oracle.layer import kept_rows, stack_backward, stack_forward
from paper_1911_04070_amd import binding as bpt
from paper_1911_04070_amd.workloads import round_to_bf16
from test_gpu_layer import BWD_TOL_DECISIVE, BWD_TOL_ORDINARY, GRADS, TOL, make_case, to_dev

pytestmark = pytest.mark.gpu
LAYERS = 3


def make_stack(n, k, causal, B, heads, d_ff, seed, decisive):
    rels, params = [], []
    for layer in range(LAYERS):
        _, Rel, p = make_case(n, k, causal, 1, heads, d_ff, seed + 17 * layer, False)
        if decisive:   # every pre-activation six deviations from zero: both sides take the same gates
            on = np.arange(d_ff) % 2 == layer % 2
            p["b1"] = np.where(on, 6.0, -6.0).astype(np.float32)
            # ... and b2 takes back the constant row 6 * sum of W2's active rows that this adds to every node: left in,
            # it dominates the next layer's input, all rows become nearly equal and gradients that vanish for equal
            # rows (dWq, dWk: the dS of a row sum to zero) are differences of large numbers
            p["b2"] = (p["b2"] - 6.0 * p["W2"][on].astype(np.float64).sum(0)).astype(np.float32)
        rels.append(Rel)
        params.append(p)
    rng = np.random.Generator(np.random.PCG64(seed + 5))
    bf = lambda a: round_to_bf16(a.astype(np.float32))[0]
    d = heads * 64
    return (bf(rng.standard_normal((B, n, d))), rels, params, bf(rng.standard_normal((B, d))),
            bf(rng.standard_normal((B, n, d))))


CASES = [(64, 2, False, 2, 1, 64, None), (256, 4, True, 2, 2, 256, None), (512, 4, False, 3, 4, 512, [512, 300, 77]),
         (1024, 8, True, 1, 8, 2048, None)]


@pytest.mark.parametrize("n,k,causal,B,heads,d_ff,lengths", CASES)
@pytest.mark.parametrize("decisive", [True, False])
def test_stack_forward_and_backward(n, k, causal, B, heads, d_ff, lengths, decisive):
    print("stack", n, k, causal, B, heads, d_ff, lengths, decisive, flush=True)
    E, rels, params, d_root, d_tokens = make_stack(n, k, causal, B, heads, d_ff, 500 + n + heads, decisive)
    g = bpt.bpt_build_graph(n, k, causal)
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    lens_d = torch.tensor(lengths, dtype=torch.int32, device="cuda") if lengths else None
    Ed, Rd, Pd = dev(E), [dev(r) for r in rels], [to_dev(p) for p in params]
    fws, bws = bpt.stack_workspace_bytes(g, B, heads, d_ff, LAYERS)
    ws_f = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")
    root, tokens = bpt.bpt_stack_fwd(g, Ed, Rd, Pd, heads, scale=0.125, seq_len=lens_d, workspace=ws_f)
    dE, d_rels, grads = bpt.bpt_stack_bwd(g, Ed, Rd, Pd, heads, ws_f, dev(d_root), dev(d_tokens), scale=0.125,
                                          seq_len=lens_d, workspace=ws_b)
    torch.cuda.synchronize()

    # ---- against the oracle
    ref_root, ref_tokens, _ = stack_forward(n, k, causal, heads, E, rels, params, 0.125, lengths=lengths)
    keep = kept_rows(n, lengths if lengths else [n] * B)[:, :n]      # token rows past a sequence's end: unspecified
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(f64(root)).all() and np.isfinite(f64(tokens)[keep]).all()
    err = max(float(np.abs(f64(root) - ref_root).max()), float(np.abs((f64(tokens) - ref_tokens)[keep]).max()))
    print("   forward max-abs error %.3g" % err, flush=True)
    assert err <= TOL * LAYERS, err
    ref_dE, ref_grads = stack_backward(n, k, causal, heads, E, rels, params, d_root, d_tokens, 0.125, lengths=lengths)
    rel_err = lambda a, r: float(np.abs(f64(a) - r).max()) / max(float(np.abs(r).max()), 1e-30)
    worst = {"dE": rel_err(dE, ref_dE)}
    for layer in range(LAYERS):
        worst["dRel%d" % layer] = rel_err(d_rels[layer], ref_grads[layer]["dRel"])
        for name in GRADS:
            worst[name + str(layer)] = rel_err(grads[layer][name], ref_grads[layer][name])
    top = sorted(worst.items(), key=lambda kv: -kv[1])[:4]
    print("   backward, largest relative max-abs errors", [(k_, float("%.2g" % v)) for k_, v in top], flush=True)
    tol = (BWD_TOL_DECISIVE if decisive else BWD_TOL_ORDINARY) * LAYERS
    for name, v in worst.items():
        assert np.isfinite(v) and v <= tol, (name, v)
    if lengths:   # embeddings past a sequence's end get exactly no gradient
        assert float(dE.float()[torch.from_numpy(~keep).cuda()].abs().max()) == 0.0

    # ---- against the layer entry points called one by one: the same bits
    N = g.num_nodes
    X = torch.zeros((B, N, heads * 64), dtype=torch.bfloat16, device="cuda")
    X[:, :n] = Ed
    lf, lb = bpt.layer_workspace_bytes(g, B, heads, d_ff)
    states, spaces = [X], []
    for layer in range(LAYERS):
        spaces.append(torch.empty(lf + 256, dtype=torch.uint8, device="cuda"))
        states.append(bpt.bpt_layer_fwd(g, states[-1], Rd[layer], Pd[layer], heads, scale=0.125, seq_len=lens_d,
                                        workspace=spaces[-1]))
    assert torch.equal(root, states[-1][:, N - 1]) and torch.equal(tokens, states[-1][:, :n])
    dH = torch.zeros_like(X)
    dH[:, :n] = dev(d_tokens)
    dH[:, N - 1] = dev(d_root)
    ws_l = torch.empty(lb + 256, dtype=torch.uint8, device="cuda")
    for layer in range(LAYERS - 1, -1, -1):
        dH, d_rel, gr = bpt.bpt_layer_bwd(g, states[layer], Rd[layer], Pd[layer], heads, spaces[layer], dH, scale=0.125,
                                          seq_len=lens_d, workspace=ws_l)
        assert torch.equal(d_rel, d_rels[layer]), layer
        for name in GRADS:
            assert torch.equal(gr[name], grads[layer][name]), (layer, name)
    assert torch.equal(dE, dH[:, :n])
    g.destroy()


@pytest.mark.parametrize("n,k,causal,heads,d_ff,lengths", [
    (256, 3, False, 2, 256, [256, 150, 31, 0, 1]), (512, 4, True, 4, 512, [77, 512, 300]),
])
def test_stack_on_the_graph_of_a_packed_batch(n, k, causal, heads, d_ff, lengths):
    # one graph for the batch (bpt_build_batch_graph): the embeddings and the token outputs are [1][T][d], the tokens of
    # all sequences in row order, and there is one root per sequence (zero for an empty one); the oracle runs the
    # padded trees with the lengths
    print("stack on a packed batch", n, k, causal, heads, d_ff, lengths, flush=True)
    B = len(lengths)
    E, rels, params, d_root, d_tokens = make_stack(n, k, causal, B, heads, d_ff, 700 + n + heads, True)
    tok = np.concatenate([np.stack([np.full(length, b), np.arange(length)]) for b, length in enumerate(lengths)], axis=1)
    live = [b for b, length in enumerate(lengths) if length >= 1]
    g = bpt.bpt_build_batch_graph(n, k, causal, lengths)
    assert g.n_tokens == tok.shape[1]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).cuda()
    Ed, Rd, Pd = dev(E[tok[0], tok[1]][None]), [dev(r) for r in rels], [to_dev(p) for p in params]
    fws, bws = bpt.stack_workspace_bytes(g, 1, heads, d_ff, LAYERS)
    ws_f = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")
    root, tokens = bpt.bpt_stack_fwd(g, Ed, Rd, Pd, heads, scale=0.125, workspace=ws_f)
    dE, d_rels, grads = bpt.bpt_stack_bwd(g, Ed, Rd, Pd, heads, ws_f, dev(d_root), dev(d_tokens[tok[0], tok[1]][None]),
                                          scale=0.125, workspace=ws_b)
    torch.cuda.synchronize()
    assert tuple(root.shape) == (B, heads * 64) and tuple(tokens.shape) == tuple(Ed.shape)
    # the oracle on the sequences that exist (an empty one has no graph), read at the tokens that exist
    sub = lambda a: np.ascontiguousarray(a[live])
    ll = [lengths[b] for b in live]
    ref_root, ref_tokens, _ = stack_forward(n, k, causal, heads, sub(E), rels, params, 0.125, lengths=ll)
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    pos = {b: i for i, b in enumerate(live)}
    tb = np.array([pos[b] for b in tok[0]])
    err = max(float(np.abs(f64(root)[live] - ref_root).max()), float(np.abs(f64(tokens)[0] - ref_tokens[tb, tok[1]]).max()))
    print("   forward max-abs error %.3g" % err, flush=True)
    assert err <= TOL * LAYERS, err
    for b in range(B):
        if b not in live:
            assert float(root[b].float().abs().max()) == 0.0
    ref_dE, ref_grads = stack_backward(n, k, causal, heads, sub(E), rels, params, sub(d_root), sub(d_tokens), 0.125, lengths=ll)
    rel_err = lambda a, r: float(np.abs(a - r).max()) / max(float(np.abs(r).max()), 1e-30)
    worst = {"dE": rel_err(f64(dE)[0], ref_dE[tb, tok[1]])}
    for layer in range(LAYERS):
        worst["dRel%d" % layer] = rel_err(f64(d_rels[layer]), ref_grads[layer]["dRel"])
        for name in GRADS:
            worst[name + str(layer)] = rel_err(f64(grads[layer][name]), ref_grads[layer][name])
    top = sorted(worst.items(), key=lambda kv: -kv[1])[:4]
    print("   backward, largest relative max-abs errors", [(k_, float("%.2g" % v)) for k_, v in top], flush=True)
    for name, v in worst.items():
        assert np.isfinite(v) and v <= BWD_TOL_DECISIVE * LAYERS, (name, v)
    with pytest.raises(Exception):                      # the graph of a packed batch is the whole batch
        bpt.bpt_stack_fwd(g, torch.cat([Ed, Ed]), Rd, Pd, heads)
    g.destroy()


def test_stack_outputs_are_optional():
    n, k, B, heads, d_ff = 128, 2, 2, 1, 64
    E, rels, params, d_root, d_tokens = make_stack(n, k, False, B, heads, d_ff, 900, True)
    g = bpt.bpt_build_graph(n, k, False)
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    Ed, Rd, Pd = dev(E), [dev(r) for r in rels], [to_dev(p) for p in params]
    fws, _ = bpt.stack_workspace_bytes(g, B, heads, d_ff, LAYERS)
    ws_f = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    root, tokens = bpt.bpt_stack_fwd(g, Ed, Rd, Pd, heads, workspace=ws_f)
    only_root, none = bpt.bpt_stack_fwd(g, Ed, Rd, Pd, heads, want_tokens=False)
    none2, only_tokens = bpt.bpt_stack_fwd(g, Ed, Rd, Pd, heads, want_root=False)
    assert none is None and none2 is None and torch.equal(root, only_root) and torch.equal(tokens, only_tokens)
    # a gradient that arrives at one output only is the other one taken as zero
    a = bpt.bpt_stack_bwd(g, Ed, Rd, Pd, heads, ws_f, dev(d_root), None)
    b = bpt.bpt_stack_bwd(g, Ed, Rd, Pd, heads, ws_f, dev(d_root), torch.zeros_like(Ed))
    assert torch.equal(a[0], b[0]) and all(torch.equal(x, y) for x, y in zip(a[1], b[1]))
    # a workspace that is too small is refused
    with pytest.raises(Exception):
        bpt.bpt_stack_fwd(g, Ed, Rd, Pd, heads, workspace=torch.empty(fws - 256, dtype=torch.uint8, device="cuda"))
    g.destroy()


def test_stack_replays_from_a_captured_graph():
    # after a first call outside the capture (it creates the GEMM library's handle and loads its kernels) a whole
    # training step of the stack only launches kernels on the caller's stream: captured once and replayed with new
    # embeddings in the same buffer, with eager work between the replays, it gives the bits of the eager call
    n, k, causal, B, heads, d_ff = 512, 4, True, 2, 2, 256
    E, rels, params, _, d_tokens = make_stack(n, k, causal, B, heads, d_ff, 77, False)
    g = bpt.bpt_build_graph(n, k, causal)
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    Ed, Rd, Pd, dT = dev(E), [dev(r) for r in rels], [to_dev(p) for p in params], dev(d_tokens)
    fws, bws = bpt.stack_workspace_bytes(g, B, heads, d_ff, LAYERS)
    ws_f = torch.empty(fws + 256, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(bws + 256, dtype=torch.uint8, device="cuda")

    def step():
        _, tokens = bpt.bpt_stack_fwd(g, Ed, Rd, Pd, heads, scale=0.125, want_root=False, workspace=ws_f)
        dE, d_rels, grads = bpt.bpt_stack_bwd(g, Ed, Rd, Pd, heads, ws_f, None, dT, scale=0.125, workspace=ws_b)
        return [tokens, dE] + list(d_rels) + [grads[layer][name] for layer in range(LAYERS) for name in GRADS]

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        captured = step()                     # its outputs live in the graph's memory pool
        graph.capture_end()
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(5)
    for replay in range(3):
        Ed.copy_(torch.randn(Ed.shape, device="cuda", generator=gen).to(Ed.dtype))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in captured]
        eager = step()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(got, eager)):
            assert torch.equal(a, b), (replay, i)
    g.destroy()
