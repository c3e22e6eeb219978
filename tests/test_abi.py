"""The C-ABI library loads and exports every symbol the header declares; host-only calls work without a GPU."""
import ctypes
import os
import re
import pytest

import paper_2202_04305_amd as sp
from paper_2202_04305_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    L = sp.load_library()
    text = open(os.path.join(ROOT, "include", "spmi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(sp_[a-z_]+)\s*\(", text)) - {"sp_alloc_fn", "sp_free_fn"}
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


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
