"""The C-ABI library loads and exports every symbol the header declares; host-only calls work without a GPU."""
import ctypes
import os
import re
import pytest

import paper_2202_04305_amd as sp
from paper_2202_04305_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_in(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(sp_[a-z_]+)\s*\(", text)) - {"sp_alloc_fn", "sp_free_fn"}


def test_header_symbols_are_exported():
    """Both headers: the product interface (spmi.h) and the measurement hooks (spmi_bench.h)."""
    L = sp.load_library()
    product, hooks = declared_in("spmi.h"), declared_in("spmi_bench.h")
    assert hooks == {"sp_profile_read", "sp_stream_copy", "sp_stream_read", "sp_pack_sort_mode"}
    assert not (product & hooks)
    assert "sp_prepare" in product
    assert product | hooks == set(binding.EXPORTS)
    for name in product | hooks:
        assert hasattr(L, name), name


def test_info_struct_matches_the_header():
    """The binding's mirror of sp_info has the header's fields in the header's order."""
    text = open(os.path.join(ROOT, "include", "spmi.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} sp_info;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        for part in decl.split(",") if "[" not in decl else [decl]:
            names.append(re.findall(r"([A-Za-z_]+)\s*(?:\[[A-Z_]+\])?$", part.strip())[0])
    assert names == [f[0] for f in binding.SpInfo._fields_]


def test_a_stale_library_is_rebuilt(monkeypatch):
    """load_library() compiles again when a source is newer than the built library (no silent use of an old build)."""
    from paper_2202_04305_amd import build
    calls = []
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "is_stale", lambda: True)
    monkeypatch.setattr(build, "build", lambda *a, **k: calls.append(1) or build.LIB)
    binding.load_library()
    assert calls == [1]


def test_encode_validation_order():
    def code(*a, **k):
        with pytest.raises(sp.SpError) as e:
            sp.sp_encode(*a, **k)
        return e.value.code
    assert code([0, 1], rank=0) == 2
    assert code([0] * 9) == 2
    assert code([0, 2]) == 3
    assert code([0, 1], [0, 0]) == 4
    assert code([0, 1], [0, 2]) == 4
    assert code([0, 1], None, 12, 32) == 5
    assert code([0, 1], None, 32, 128) == 5
    assert sp.sp_encode([0, 1], None, 8, 16).rank == 2
    assert code([0, 2], [0, 0], 12, 12) == 3     # level type before ordering before width
    assert code([0, 1], [0, 0], 12, 12) == 4
    e = sp.sp_encode([1, 1], [1, 0], 32, 64)
    assert e.rank == 2


def test_status_strings():
    L = sp.load_library()
    assert L.sp_status_str(0) == b"ok"
    assert all(L.sp_status_str(i) for i in range(14))
