"""The C ABI library loads and exports every symbol include/vattn.h declares (no compute calls)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):     # the method's header and the bench-only one
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(vattn_[a-z_]+)\s*\(", text))
    return sorted(names)


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


def test_scale_must_be_finite_and_positive():
    """Eq. 2 divides by a positive constant: every attention entry point refuses a scale that is zero, negative,
    infinite or NaN before it looks at anything else (so this runs without a GPU or a context)."""
    import paper_2405_04437_amd as P

    L = P.lib
    for bad in (0.0, -0.125, float("inf"), float("-inf"), float("nan")):
        calls = [
            lambda s: L.vattn_attn_decode(None, 0, None, None, None, None, None, 1, s, None, 0),
            lambda s: L.vattn_attn_decode_append(None, 0, None, None, None, None, None, None, None, 1, s, None, 0),
            lambda s: L.vattn_attn_prefill(None, 0, None, None, None, None, None, None, 1, s),
            lambda s: L.vattn_attn_prefill_append(None, 0, None, None, None, None, None, None, None, None, 1, s),
            lambda s: L.vattn_attn_decode_paged(None, None, None, None, None, None, 1, 32, None, 1, None, 1, s, None, 0),
            lambda s: L.vattn_attn_prefill_paged(None, None, None, None, None, None, 1, 64, None, 1, None, None, 1, s),
        ]
        for call in calls:
            assert call(bad) == -1 and "scale must be finite and > 0" in P.last_error(), bad
            assert call(0.125) == -1 and "null" in P.last_error()      # a good scale gets past that check
