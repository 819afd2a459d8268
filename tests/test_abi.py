"""The C ABI library loads and exports every symbol include/vattn.h declares (no compute calls)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "vattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vattn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2405_04437_amd as P

    names = _declared()
    assert len(names) >= 15
    lib = ctypes.CDLL(P.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in vattn.h but not exported"
    assert sorted(P.EXPORTED) == names


def test_errors_without_gpu_are_reported_not_fatal():
    import torch
    import paper_2405_04437_amd as P

    if torch.cuda.is_available():
        return
    try:
        P.Vattn(1, 2, 128, 8, 2, 64, 1 << 20)
    except P.VattnError as e:
        assert "hip" in str(e).lower() or "device" in str(e).lower()
    else:
        raise AssertionError("init must fail without a GPU")


def test_null_arguments_are_rejected():
    import paper_2405_04437_amd as P

    assert P.lib.vattn_alloc_reqid(None) == -1 and "null" in P.last_error()
    assert P.lib.vattn_step(None, None, 0) == -1
    assert P.lib.vattn_free_reqid(None, 0) == -1
    assert P.lib.vattn_init(None, None) == -1
