"""The C-ABI library loads without a GPU and exports every function include/qoda.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "qoda.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qoda_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_named_entry_points():
    names = _declared()
    for must in ("qoda_quantize", "qoda_dequant_aggregate", "qoda_step", "qoda_fit_levels"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2505_14371_amd import qoda

    if not os.path.exists(qoda.LIB_PATH):
        from paper_2505_14371_amd import build

        build.build()
    lib = ctypes.CDLL(qoda.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert qoda.load() is not None


def test_binding_names_match_the_header():
    from paper_2505_14371_amd import qoda

    for name in _declared():
        short = name[len("qoda_"):]
        if short in ("create", "destroy", "last_error"):
            continue
        assert hasattr(qoda.Context, short) or hasattr(qoda, short), short


def test_null_arguments_are_rejected_without_a_gpu():
    from paper_2505_14371_amd import qoda

    lib = qoda.load()
    assert lib.qoda_create(None, None) == qoda.EINVAL
    out = ctypes.c_void_p()
    assert lib.qoda_create(None, ctypes.byref(out)) == qoda.EINVAL and not out.value
    assert lib.qoda_destroy(None) == qoda.EINVAL
    assert lib.qoda_message_bytes(None) == 0
    assert lib.qoda_last_error(None) == b"null context"
    assert lib.qoda_status(None, None) == qoda.EINVAL


def test_missing_library_is_a_loud_error(monkeypatch, tmp_path):
    from paper_2505_14371_amd import qoda

    monkeypatch.setattr(qoda, "_lib", None)
    monkeypatch.setattr(qoda, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(qoda.QodaError):
        qoda.load()
