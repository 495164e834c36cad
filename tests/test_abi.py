"""Host-side checks that need no GPU: the library loads and exports every declared symbol."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "deltacnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dcnn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2203_03996_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    lib = pkg.load_library()
    declared = _declared_symbols()
    assert len(declared) >= 25
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in deltacnn.h but not exported"
    assert sorted(pkg.EXPORTS) == declared


def test_host_side_validation_needs_no_gpu():
    import ctypes as C
    import paper_2203_03996_amd as pkg
    from paper_2203_03996_amd.binding import LayerDesc, LayerSizes
    lib = pkg.load_library()
    assert lib.dcnn_workspace_bytes(1 << 20) > (1 << 20)
    assert lib.dcnn_status_str(0) == b"ok"
    sz = LayerSizes()
    good = pkg.make_desc(pkg.CONV, pkg.F16, 2, 16, 16, 64, k=3, stride=1, pad=1, cout=64, act=pkg.ACT_RELU, eps=0.1)
    assert lib.dcnn_layer_query(C.byref(good), C.byref(sz)) == 0
    assert (sz.on, sz.oh, sz.ow, sz.oc) == (2, 16, 16, 64)
    # x^A, x^T, the delta output, masks, lists and packed weights all live in the state memory
    assert sz.state_bytes > 3 * 2 * 16 * 16 * 64 * 2
    bad = pkg.make_desc(pkg.CONV, pkg.F16, 2, 16, 16, 64, k=3, stride=3, pad=1, cout=64)
    assert lib.dcnn_layer_query(C.byref(bad), C.byref(sz)) == 1          # DCNN_EINVAL
    bad = pkg.make_desc(pkg.ACT, 5, 2, 16, 16, 64, act=pkg.ACT_RELU)
    assert lib.dcnn_layer_query(C.byref(bad), C.byref(sz)) == 3          # DCNN_EDTYPE
    bad = pkg.make_desc(pkg.MAXPOOL, pkg.F32, 1, 2, 2, 4, k=7, stride=2, pad=1)
    assert lib.dcnn_layer_query(C.byref(bad), C.byref(sz)) == 2          # DCNN_ESHAPE
    assert lib.dcnn_ctx_sync(None) == 1 and lib.dcnn_layer_step(None, None, 0) == 1


def test_no_cpu_fallback_without_gpu():
    import torch
    import paper_2203_03996_amd as pkg
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        pkg.Context(1024)
