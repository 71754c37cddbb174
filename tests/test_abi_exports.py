"""The C-ABI library loads on a machine without a GPU and exports every symbol
include/pv.h declares (no compute call is made here)."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    text = (ROOT / "include" / "pv.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pv_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    path = ROOT / "paper_2405_14852_amd" / "libpv.so"
    if not path.exists():
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(str(path))


def test_header_declares_the_four_calls_of_the_path():
    names = declared_functions()
    for f in ("pv_encode_targets", "pv_select_topk_groups", "pv_reencode_groups", "pv_dequantize",
              "pv_create", "pv_destroy", "pv_last_error"):
        assert f in names


def test_every_declared_symbol_is_exported(lib):
    for f in declared_functions():
        assert hasattr(lib, f), f


def test_binding_uses_the_same_names():
    import paper_2405_14852_amd as pkg
    # the context's life cycle is the Python object's; every other call keeps its C name
    for f in set(declared_functions()) - {"pv_create", "pv_destroy", "pv_last_error"}:
        assert hasattr(pkg.PVContext, f), f


def test_null_context_is_rejected_without_a_gpu(lib):
    lib.pv_encode_targets.restype = ctypes.c_int
    assert lib.pv_encode_targets(None, None, None, None, ctypes.c_float(1.0), None) != 0
    lib.pv_last_error.restype = ctypes.c_char_p
    assert b"NULL" in lib.pv_last_error(None)


def test_product_package_does_not_touch_the_oracle():
    for p in (ROOT / "paper_2405_14852_amd").rglob("*"):
        if p.suffix in (".py", ".hip", ".h"):
            text = p.read_text()
            assert "import oracle" not in text and "pvo_" not in text, p


def test_create_without_a_gpu_reports_a_device_error(lib):
    """No GPU in this process: pv_create must fail cleanly (no fallback of any kind)."""
    try:
        import torch
        if torch.cuda.is_available():
            pytest.skip("a GPU is visible")
    except ImportError:
        pass
    lib.pv_create.restype = ctypes.c_int
    h = ctypes.c_void_p()
    st = lib.pv_create(ctypes.byref(h), 0, None)
    assert st != 0 and not h.value


def test_binding_refuses_host_tensors():
    import torch
    from paper_2405_14852_amd import binding
    with pytest.raises(TypeError):
        binding._dev_ptr(torch.zeros(4), torch.float32, "W")
