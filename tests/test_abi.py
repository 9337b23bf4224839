"""The C-ABI library loads and exports every symbol that include/blink.h declares (no GPU needed)."""
import ctypes
import os
import re

import paper_2604_07609_amd as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "blink.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(blink_[a-z_]+)\s*\(", src)))


def test_header_and_binding_agree():
    names = declared_functions()
    assert names and sorted(B.EXPORTS) == names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(B.lib_path())
    for n in declared_functions():
        assert hasattr(lib, n), n


def test_struct_sizes_match_header():
    from paper_2604_07609_amd import binding
    assert ctypes.sizeof(binding.Config) == 104 and ctypes.sizeof(binding.Sampling) == 24 and ctypes.sizeof(binding.Stats) == 88
    assert binding.EVENT_DTYPE.itemsize == 32 and binding.TRACE_DTYPE.itemsize == 80


def test_argument_errors_without_gpu():
    lib = B.load_library()
    assert lib.blink_init(None, None) == B.ERR_INVAL
    assert b"null" in lib.blink_last_error()
    assert lib.blink_run(None, 0) == B.ERR_INVAL and lib.blink_shutdown(None) == B.ERR_INVAL
