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


def test_kmax_controller_matches_the_oracle_update():
    """Host logic only: the C controller against oracle.kmax_update over a seeded run of fallback counts."""
    import numpy as np
    _lib()
    import paper_2511_21702_amd as csv
    from oracle import csv_oracle as O
    rng = np.random.default_rng(5)
    for literal in (False, True):
        ctl = csv.KmaxController(K0=32064, K_min=1000, K_cap=128256, alpha=0.01, rho_target=0.02, literal=literal)
        K = 32064.0
        for _ in range(500):
            B = int(rng.integers(1, 65))
            nfb = int(rng.binomial(B, 0.1))
            got = ctl.update(nfb, B)
            K = min(max(O.kmax_update(K, nfb / B, 0.01, 0.02, literal=literal), 1000.0), 128256.0)
            assert got == O.kmax_rows(K, 1000, 128256)
            assert abs(ctl.value - K) <= 1e-9 * K
    # range clamps and argument errors
    ctl = csv.KmaxController(K0=1000, K_min=1000, K_cap=1010, alpha=0.5, rho_target=0.02)
    for _ in range(10):
        v = ctl.update(4, 4)
    assert v == 1010
    lib = csv.lib
    assert lib.csv_kmax_update(None, 0, 1) == -1
    import ctypes as C
    c = csv.KmaxCtl()
    assert lib.csv_kmax_init(C.byref(c), 5, 10, 20, 0.01, 0.02, 0) == -1      # K0 below K_min
    assert lib.csv_kmax_init(C.byref(c), 15, 10, 20, 0.01, 0.02, 0) == 0
    assert lib.csv_kmax_update(C.byref(c), 3, 2) == -1                         # more fallbacks than sequences
