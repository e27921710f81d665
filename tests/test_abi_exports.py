"""The built library loads and exports every function that include/smartmem.h declares (no compute calls)."""
import ctypes
import os
import re
from paper_2404_13528_amd import binding as sm

HDR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "smartmem.h")


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HDR).read(), flags=re.S)
    names = re.findall(r"\b(sm_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    lib = sm.lib()
    names = declared_functions()
    assert len(names) >= 30 and "sm_layout_plan" in names and "sm_run_chain" in names
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing


def test_version_and_error_string():
    lib = sm.lib()
    assert lib.sm_abi_version() == 1
    rc = lib.sm_map_create(None, None, 0, None)
    assert rc == -1 and b"null" in lib.sm_last_error()
