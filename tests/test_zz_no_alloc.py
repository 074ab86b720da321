"""The forward entry point that allocates nothing (bpt_attn_fwd_static) against bpt_attn_fwd, through the C ABI.

Collected last on purpose (the file name sorts after the other tests): a failure here must not hide the others."""
import ctypes

import numpy as np
import pytest
import torch

from paper_1911_04070_amd import binding as bpt
from paper_1911_04070_amd.workloads import Workload, make_inputs

pytestmark = pytest.mark.gpu


def _raw_call(name, g, shp, *ptrs):
    """Calls an entry point of libbpt.so directly: raw pointers, no wrapper logic."""
    fn = getattr(bpt.load_library(), name)
    return fn(g.handle, ctypes.byref(shp), *ptrs)


def _forward_both(g, w, x, lengths=None):
    dev = {k: torch.from_numpy(x[k]).to(torch.bfloat16 if w.dtype == "bf16" else torch.float32).cuda()
           for k in ("Q", "K", "V", "Rel")}
    Q, K, V, R = dev["Q"], dev["K"], dev["V"], dev["Rel"]
    lens_d = torch.tensor(lengths, dtype=torch.int32, device="cuda") if lengths is not None else None
    shp = bpt._shape_of(g, Q, w.scale, lens_d)
    stream = int(torch.cuda.current_stream().cuda_stream)
    # the existing entry point, with a workspace the caller allocates
    need = int(bpt.load_library().bpt_attn_fwd_workspace(g.handle, ctypes.byref(shp)))
    assert need <= bpt.BPT_STATIC_SCRATCH_BYTES
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    out_a, lse_a = torch.empty_like(Q), torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda")
    rc = _raw_call("bpt_attn_fwd", g, shp, Q.data_ptr(), K.data_ptr(), V.data_ptr(), R.data_ptr(), out_a.data_ptr(),
                   lse_a.data_ptr(), ws.data_ptr(), ws.numel(), stream)
    assert rc == bpt.BPT_OK
    # the entry point that allocates nothing: outputs filled with a pattern first, so that rows it did not write show
    out_b = torch.full_like(Q, 7.0)
    lse_b = torch.full(Q.shape[:3], 7.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = _raw_call("bpt_attn_fwd_static", g, shp, Q.data_ptr(), K.data_ptr(), V.data_ptr(), R.data_ptr(),
                   out_b.data_ptr(), lse_b.data_ptr(), stream)
    assert rc == bpt.BPT_OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return (out_a, lse_a), (out_b, lse_b)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_forward_matches_the_forward_with_a_workspace(dtype):
    # two calls in a row on the one static buffer, the second with a smaller input (fewer and shorter partial
    # rows, so most of the buffer still holds the first call's partials), then one with shorter sequences
    print("static scratch", dtype, flush=True)
    cases = [(Workload("static_a", 41, 4096, 3, True, 2, 3, 64, dtype, False), None),
             (Workload("static_b", 42, 1024, 5, False, 1, 2, 64, dtype, False), None),
             (Workload("static_c", 43, 2048, 2, False, 2, 1, 64, dtype, False), [2048, 700])]
    for w, lengths in cases:
        g = bpt.bpt_build_graph(w.n, w.k, w.causal)
        (out_a, lse_a), (out_b, lse_b) = _forward_both(g, w, make_inputs(w, with_dO=False), lengths)
        # the same kernels on the same inputs: the same bits, which is within any tolerance of the parity tests
        assert torch.equal(out_a, out_b), w.name
        assert torch.equal(lse_a, lse_b), w.name
        assert float(lse_b.abs().max()) > 0 and np.isfinite(out_b.float().cpu().numpy()).all()
        g.destroy()


def test_static_scratch_refuses_what_does_not_fit():
    # n = 65536 with 8 heads needs 47 MB of partial rows: more than the static buffer, a clear error and no launch
    g = bpt.bpt_build_graph(65536, 4, True)
    Q = torch.zeros(1, 8, g.num_nodes, 64, dtype=torch.bfloat16, device="cuda")
    R = torch.zeros(g.num_levels, g.rel_width, 64, dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(Q, 7.0)
    lse = torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda")
    shp = bpt._shape_of(g, Q, None)
    assert int(bpt.load_library().bpt_attn_fwd_workspace(g.handle, ctypes.byref(shp))) > bpt.BPT_STATIC_SCRATCH_BYTES
    with pytest.raises(bpt.BptError) as e:
        bpt.bpt_attn_fwd_static(g, Q, Q, Q, R, out, lse)
    assert e.value.status == bpt.BPT_ERR_SCRATCH
    assert "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert float(out.float().min()) == 7.0   # nothing was launched
    g.destroy()
