"""The C-ABI library loads and exports every symbol include/csv_decode.h declares (no compute without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_21702_amd", "libcsvdecode.so")
HEADER = os.path.join(ROOT, "include", "csv_decode.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(csv_[a-z_0-9]+)\s*\(", src)))


def _lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"csv_build_index", "csv_decode_step", "csv_full_logits"} <= set(names)
    lib = _lib()
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_symbols():
    _lib()
    import paper_2511_21702_amd as csv
    assert sorted(csv.EXPORTS) == _declared()


def test_host_side_argument_checks_need_no_gpu():
    lib = _lib()
    lib.csv_last_error.restype = ctypes.c_char_p
    assert lib.csv_workspace_create(None, 1, 1, None) == -1
    assert lib.csv_decode_step(None, None, None, 1, None, None, None) == -1
    assert b"null" in lib.csv_last_error()
    assert lib.csv_index_dims(None, None, None, None) == -1
