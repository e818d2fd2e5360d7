"""The C ABI library loads and exports every symbol include/qrm.h declares (no compute, no GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="qrm.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    return re.findall(r"QRM_API\s+[\w\s\*]+?\b(qrm_\w+)\s*\(", text)


def test_header_declares_the_entry_points():
    names = declared_symbols()
    for must in ("qrm_extract_tiles", "qrm_extractor_forward", "qrm_rs_decode", "qrm_detect",
                 "qrm_create", "qrm_destroy", "qrm_last_error"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2509_02447_amd import binding
    path = binding.lib_path()
    assert os.path.exists(path), "libqrm.so is not built: run __graft_entry__.build()"
    lib = ctypes.CDLL(path)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert set(declared_symbols()) == set(binding.EXPORTS)
    for name in declared_symbols("qrm_diag.h"):
        assert hasattr(lib, name), name
    assert set(declared_symbols("qrm_diag.h")) == set(binding.DIAG_EXPORTS)
    lib.qrm_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.qrm_version()


def test_binding_does_not_touch_the_oracle():
    # the product path must not import the test oracle
    import paper_2509_02447_amd.binding as b
    src = open(b.__file__).read() + open(os.path.join(os.path.dirname(b.__file__), "__init__.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")
    for f in os.listdir(os.path.join(os.path.dirname(b.__file__), "csrc")):
        assert "oracle" not in open(os.path.join(os.path.dirname(b.__file__), "csrc", f)).read()
