"""The C-ABI library loads without a GPU and exports every symbol include/ocn.h declares."""
import ctypes
import os
import re

import paper_1810_08723_amd as ocn
from paper_1810_08723_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ocn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ocn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"ocn_unary", "ocn_binary", "ocn_cast_copy", "ocn_reduce"} <= set(names)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None, n
    assert set(names) == set(B.EXPORTS)


def test_descriptor_layouts_match_the_header():
    # 8 (base) + 8 (offset) + 4 + 4 + 64 + 64 + 4 (+4 pad)
    assert ctypes.sizeof(B.OcnTensor) == 160
    assert B.OcnTensor.size.offset == 24 and B.OcnTensor.stride.offset == 88 and B.OcnTensor.device.offset == 152


def test_dtype_sizes_and_error_strings():
    sizes = dict(bool=1, int8=1, int16=2, int32=4, int64=8, uint8=1, uint16=2, uint32=4, uint64=8,
                 half=2, float=4, double=8, chalf=4, cfloat=8, cdouble=16)
    for k, v in sizes.items():
        assert ocn.dtype_size(k) == v
    assert B.lib().ocn_dtype_size(99) == 0
    seen = set()
    for code in range(0, -13, -1):
        s = B.lib().ocn_error_string(code).decode()
        assert s and s not in seen
        seen.add(s)


def test_no_fallback_when_the_library_is_missing(monkeypatch, tmp_path):
    import importlib
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    try:
        B.lib()
    except ImportError as e:
        assert "no fallback" in str(e)
    else:
        raise AssertionError("a missing library must raise")
    finally:
        monkeypatch.undo()
        importlib.reload(B)
