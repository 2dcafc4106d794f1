"""The shared library loads without a GPU and exports every function include/redist.h declares."""
import os
import re

import paper_2112_01075_amd as R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "redist.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(redist_[a-z_]+)\s*\(", text))
    assert {"redist_plan_create", "redist_execute", "redist_plan_destroy", "redist_status_string"} <= names
    L = R.lib()
    for n in sorted(names):
        assert hasattr(L, n), n


def test_status_strings():
    L = R.lib()
    assert L.redist_status_string(0) == b"ok"
    assert all(L.redist_status_string(k) for k in range(0, 12))


def test_box_struct_is_128_bytes():
    import ctypes
    assert ctypes.sizeof(R.Box) == 128
