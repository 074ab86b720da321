"""Host-only checks of the C-ABI boundary: the library loads without a GPU, exports every
symbol include/bpt.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import oracle

from paper_1911_04070_amd import binding as bpt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bpt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bpt_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    names = declared_functions()
    assert "bpt_build_graph" in names and "bpt_attn_fwd" in names and "bpt_attn_bwd" in names
    assert sorted(bpt.EXPORTS) == names


def test_library_exports_every_declared_symbol():
    lib = bpt.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_strerror_is_total():
    seen = set()
    for code in range(0, 7):
        msg = bpt.strerror(code)
        assert msg and msg not in seen
        seen.add(msg)
    assert bpt.strerror(12345) == "unknown status"


@pytest.mark.parametrize("n,k,code", [
    (0, 1, bpt.BPT_ERR_INVALID_ARG), (1, 1, bpt.BPT_ERR_INVALID_ARG), (8, 0, bpt.BPT_ERR_INVALID_ARG),
    (8, -3, bpt.BPT_ERR_INVALID_ARG), (6, 2, bpt.BPT_ERR_UNSUPPORTED), (1000, 2, bpt.BPT_ERR_UNSUPPORTED),
    (1 << 23, 2, bpt.BPT_ERR_UNSUPPORTED), (8, (1 << 20) + 1, bpt.BPT_ERR_UNSUPPORTED),
])
def test_build_graph_rejects_bad_sizes_on_the_host(n, k, code):
    lib = bpt.load_library()
    h = ctypes.c_void_p(123)
    assert lib.bpt_build_graph(n, k, 0, None, ctypes.byref(h)) == code
    assert h.value is None                       # *out is cleared on failure
    assert lib.bpt_build_graph(8, 2, 0, None, None) == bpt.BPT_ERR_INVALID_ARG


def test_build_batch_graph_rejects_bad_arguments_on_the_host():
    lib = bpt.load_library()
    lens = (ctypes.c_int32 * 3)(4, 65, 2)
    for args, code in (((64, 2, 0, lens, 3), bpt.BPT_ERR_INVALID_ARG),          # a length above n
                       ((64, 2, 0, None, 3), bpt.BPT_ERR_INVALID_ARG), ((64, 2, 0, lens, 0), bpt.BPT_ERR_INVALID_ARG),
                       ((48, 2, 0, lens, 1), bpt.BPT_ERR_UNSUPPORTED), ((64, 0, 0, lens, 1), bpt.BPT_ERR_INVALID_ARG),
                       ((64, 2, 0, lens, (1 << 16) + 1), bpt.BPT_ERR_UNSUPPORTED)):
        h = ctypes.c_void_p(123)
        n, k, causal, lengths, batch = args
        assert lib.bpt_build_batch_graph(n, k, causal, lengths, batch, None, ctypes.byref(h)) == code, args
        assert h.value is None
    assert lib.bpt_build_batch_graph(64, 2, 0, lens, 1, None, None) == bpt.BPT_ERR_INVALID_ARG
    h = ctypes.c_void_p(123)
    assert lib.bpt_build_batch_graph_on(None, lens, 1, 0, None, ctypes.byref(h)) == bpt.BPT_ERR_INVALID_ARG and h.value is None
    assert lib.bpt_build_batch_graph_on(None, lens, 1, 0, None, None) == bpt.BPT_ERR_INVALID_ARG


def test_null_graph_is_an_error_everywhere():
    lib = bpt.load_library()
    shp = bpt.BptShape(1, 1, 64, bpt.BPT_F32, 64, 64, 64, 0.0)
    assert lib.bpt_graph_info(None, *([None] * 8)) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_graph_layout(None, None, None, None, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_graph_csr(None, None, None, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_graph_transposed(None, None, None, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_graph_to_host(None, None, None, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_graph_transposed_to_host(None, None, None, None) == bpt.BPT_ERR_INVALID_ARG
    # a refused graph / shape is told apart from "no workspace needed": SIZE_MAX, not 0
    assert lib.bpt_attn_fwd_workspace(None, ctypes.byref(shp)) == 2 ** 64 - 1
    assert lib.bpt_attn_bwd_workspace(None, ctypes.byref(shp)) == 2 ** 64 - 1
    assert lib.bpt_calibrate_gather(None, None, None, 8, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_attn_fwd(None, ctypes.byref(shp), *([None] * 7), 0, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_attn_fwd_static(None, ctypes.byref(shp), *([None] * 7)) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_attn_bwd(None, ctypes.byref(shp), *([None] * 11), 0, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_attn_bwd_query_side(None, ctypes.byref(shp), *([None] * 9), 0, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_attn_bwd_key_side(None, ctypes.byref(shp), *([None] * 9), 0, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_layer_fwd_workspace(None, 1, 1, 64) == 0 and lib.bpt_layer_bwd_workspace(None, 1, 1, 64) == 0
    assert lib.bpt_layer_fwd(None, 1, 1, 0.0, *([None] * 6), 0, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_layer_bwd(None, 1, 1, 0.0, *([None] * 5), 0, *([None] * 5), 0, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_stack_fwd_workspace(None, 1, 1, 64, 2) == 0 and lib.bpt_stack_bwd_workspace(None, 1, 1, 64) == 0
    assert lib.bpt_stack_fwd(None, 1, 1, 2, 0.0, *([None] * 7), 0, None) == bpt.BPT_ERR_INVALID_ARG
    assert lib.bpt_stack_bwd(None, 1, 1, 2, 0.0, *([None] * 4), 0, *([None] * 6), 0, None) == bpt.BPT_ERR_INVALID_ARG
    lib.bpt_graph_destroy(None)                  # a no-op, must not crash


def test_shape_struct_layout_matches_the_header():
    # int32 B,H,D,dtype; int64 stride_b,stride_h,stride_n; float scale (+ padding); pointer seq_len;
    # float dropout_p; uint32 dropout_seed; int32 leave_unkept; int32 grad_dtype
    assert ctypes.sizeof(bpt.BptShape) == 72
    assert bpt.BptShape.dropout_p.offset == 56 and bpt.BptShape.dropout_seed.offset == 60
    assert bpt.BptShape.leave_unkept.offset == 64 and bpt.BptShape.grad_dtype.offset == 68
    assert bpt.BptShape.stride_b.offset == 16 and bpt.BptShape.scale.offset == 40
    assert bpt.BptShape.seq_len.offset == 48


def test_no_cpu_fallback_when_the_library_is_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(bpt, "_lib", None)
    monkeypatch.setattr(bpt, "LIB_PATH", str(tmp_path / "libbpt.so"))
    with pytest.raises(FileNotFoundError):
        bpt.load_library()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1911_04070_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "bpt_oracle" not in text, f


def test_edge_count_of_shorter_sequences_matches_the_oracle():
    # host arithmetic of the library (no device involved) against the oracle's builder
    for n, k, causal in ((2, 1, False), (8, 1, True), (16, 2, False), (32, 3, False), (64, 40, True), (256, 4, False),
                         (512, 4, False), (1024, 7, True)):
        lengths = range(1, n + 1) if n <= 64 else (1, 2, 3, n // 3, n // 2 - 1, n // 2, n // 2 + 1, n - 1, n)
        for length in lengths:
            want = oracle.build_graph_len(n, length, k, causal).num_edges
            assert bpt.bpt_count_edges(n, k, causal, length) == want, (n, k, causal, length)
        assert bpt.bpt_count_edges(n, k, causal, 0) == 0
    with pytest.raises(bpt.BptError):
        bpt.bpt_count_edges(64, 2, False, 65)
    with pytest.raises(bpt.BptError):
        bpt.bpt_count_edges(48, 2, False, 5)
