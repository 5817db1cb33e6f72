"""Python binding of the CSV-Decode C ABI (include/csv_decode.h) for MI355X.

Argument marshalling only: every step of the path runs in the HIP kernels of libcsvdecode.so.
PyTorch supplies device memory and the stream.  There is no CPU fallback: importing this package
without the built library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcsvdecode.so")

FLAG_TOPK_CERT, FLAG_SOFTMAX_CERT, FLAG_FALLBACK, FLAG_INVALID_INPUT, FLAG_SOFTMAX_RELAXED, FLAG_ABORTED = 1, 2, 4, 8, 16, 32
SCHEDULE_ROUNDS, SCHEDULE_ALG1 = 0, 1
COMBINE_ALL, COMBINE_ANY = 0, 1
MAX_K, MAX_CLUSTERS, MAX_BATCH = 1024, 8192, 256

EXPORTS = [
    "csv_build_index", "csv_index_from_arrays", "csv_index_export", "csv_index_dims", "csv_index_free",
    "csv_workspace_create", "csv_workspace_free", "csv_decode_step", "csv_bounds", "csv_full_logits",
    "csv_profile_begin", "csv_profile_end", "csv_last_error", "csv_kmax_init", "csv_kmax_update",
    "csv_workspace_set_spin_limit", "csv_index_use_bf16_centroids",
    "csv_workspace_set_tail_split", "csv_bounds_static", "csv_index_set_bias_table", "csv_index_get_bias_table",
    "csv_index_set_angular", "csv_index_get_angular",
]
PROFILE_STAGES = ["bounds", "round0", "tail"]


class BuildOpts(C.Structure):
    _fields_ = [("iters", C.c_int), ("h_init_labels", C.c_void_p), ("h_init_rows", C.c_void_p),
                ("radius_slack", C.c_float), ("centroid_bf16", C.c_int), ("spherical", C.c_int), ("bias_table_m", C.c_int)]


class StepParams(C.Structure):
    _fields_ = [("k", C.c_int), ("eps", C.c_float), ("K_max_rows", C.c_int), ("combine", C.c_int),
                ("max_rounds", C.c_int), ("delta_clusters", C.c_int), ("relax", C.c_int), ("top_p", C.c_float),
                ("schedule", C.c_int)]


class KmaxCtl(C.Structure):
    _fields_ = [("K_max", C.c_double), ("alpha", C.c_double), ("rho_target", C.c_double), ("K_min", C.c_int),
                ("K_cap", C.c_int), ("literal", C.c_int)]


class StepOut(C.Structure):
    _fields_ = [("d_ids", C.c_void_p), ("d_logits", C.c_void_p), ("d_lse", C.c_void_p), ("d_flags", C.c_void_p),
                ("d_n_rows", C.c_void_p), ("d_n_clusters", C.c_void_p), ("d_rounds", C.c_void_p),
                ("d_sel_clusters", C.c_void_p), ("d_fallback_count", C.c_void_p),
                ("d_probs", C.c_void_p), ("d_cum", C.c_void_p), ("d_nucleus", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2511_21702_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, ci = C.c_void_p, C.c_int
    lib.csv_last_error.restype = C.c_char_p
    lib.csv_build_index.argtypes = [vp, vp, ci, ci, ci, C.POINTER(BuildOpts), vp, C.POINTER(vp)]
    lib.csv_index_from_arrays.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp, vp, vp, C.POINTER(vp)]
    lib.csv_index_export.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.csv_index_dims.argtypes = [vp, C.POINTER(ci), C.POINTER(ci), C.POINTER(ci)]
    lib.csv_index_free.argtypes = [vp]
    lib.csv_index_free.restype = None
    lib.csv_workspace_create.argtypes = [vp, ci, ci, C.POINTER(vp)]
    lib.csv_workspace_free.argtypes = [vp]
    lib.csv_workspace_free.restype = None
    lib.csv_decode_step.argtypes = [vp, vp, vp, ci, C.POINTER(StepParams), C.POINTER(StepOut), vp]
    lib.csv_bounds.argtypes = [vp, vp, vp, ci, vp, vp, vp]
    lib.csv_full_logits.argtypes = [vp, vp, vp, ci, vp, vp]
    lib.csv_bounds_static.argtypes = [vp, vp, ci, vp, vp, vp]
    lib.csv_index_set_bias_table.argtypes = [vp, ci, vp, vp]
    lib.csv_index_get_bias_table.argtypes = [vp, C.POINTER(ci), vp]
    lib.csv_index_set_angular.argtypes = [vp, vp, vp]
    lib.csv_index_get_angular.argtypes = [vp, C.POINTER(ci), vp]
    lib.csv_profile_begin.argtypes = [vp, ci]
    lib.csv_profile_end.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(ci)]
    lib.csv_kmax_init.argtypes = [C.POINTER(KmaxCtl), ci, ci, ci, C.c_double, C.c_double, ci]
    lib.csv_kmax_update.argtypes = [C.POINTER(KmaxCtl), ci, ci]
    lib.csv_workspace_set_spin_limit.argtypes = [vp, ci]
    lib.csv_index_use_bf16_centroids.argtypes = [vp, vp]
    lib.csv_workspace_set_tail_split.argtypes = [vp, ci]
    return lib


lib = _load()


class CsvError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"csv error {code}: {lib.csv_last_error().decode()}")


def _check(rc: int) -> None:
    if rc != 0:
        raise CsvError(rc)


def _stream(stream=None) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _dev2(t: torch.Tensor, what: str) -> torch.Tensor:
    if not t.is_cuda or t.element_size() != 2 or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous 16-bit (bf16 pattern) CUDA tensor")
    return t


class CsvIndex:
    """Owner of a csv_index handle."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)
        V, d, Cc = C.c_int(), C.c_int(), C.c_int()
        _check(lib.csv_index_dims(self._h, C.byref(V), C.byref(d), C.byref(Cc)))
        self.V, self.d, self.C = V.value, d.value, Cc.value

    def export(self) -> dict:
        import numpy as np
        mu = np.empty((self.C, self.d), np.float32)
        R = np.empty(self.C, np.float32)
        bmax = np.empty(self.C, np.float32)
        n = np.empty(self.C, np.int32)
        perm = np.empty(self.V, np.int32)
        _check(lib.csv_index_export(self._h, mu.ctypes.data, R.ctypes.data, bmax.ctypes.data, n.ctypes.data,
                                    perm.ctypes.data))
        return {"mu": mu, "R": R, "bmax": bmax, "n": n, "perm": perm}

    def set_angular(self, ang, stream=None) -> None:
        """ang: numpy float32 [C, 4] (cos, sin of the angular radius, largest, smallest row norm), or None to remove."""
        import numpy as np
        if ang is None:
            _check(lib.csv_index_set_angular(self._h, None, _stream(stream)))
            return
        t = np.ascontiguousarray(ang, dtype=np.float32)
        assert t.shape == (self.C, 4)
        _check(lib.csv_index_set_angular(self._h, t.ctypes.data, _stream(stream)))

    def angular(self):
        """numpy float32 [C, 4], or None for a Euclidean index."""
        import numpy as np
        present = C.c_int()
        _check(lib.csv_index_get_angular(self._h, C.byref(present), None))
        if not present.value:
            return None
        t = np.empty((self.C, 4), np.float32)
        _check(lib.csv_index_get_angular(self._h, C.byref(present), t.ctypes.data))
        return t

    def set_bias_table(self, table, stream=None) -> None:
        """table: numpy float32 [C, m, 2] of (radius, bias) pairs, or None to remove the table."""
        import numpy as np
        if table is None:
            _check(lib.csv_index_set_bias_table(self._h, 0, None, _stream(stream)))
            return
        t = np.ascontiguousarray(table, dtype=np.float32)
        assert t.ndim == 3 and t.shape[0] == self.C and t.shape[2] == 2
        _check(lib.csv_index_set_bias_table(self._h, t.shape[1], t.ctypes.data, _stream(stream)))

    def bias_table(self):
        """numpy float32 [C, m, 2], or None when the index has no table."""
        import numpy as np
        m = C.c_int()
        _check(lib.csv_index_get_bias_table(self._h, C.byref(m), None))
        if m.value == 0:
            return None
        t = np.empty((self.C, m.value, 2), np.float32)
        _check(lib.csv_index_get_bias_table(self._h, C.byref(m), t.ctypes.data))
        return t

    def free(self) -> None:
        if self._h:
            lib.csv_index_free(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def csv_build_index(W: torch.Tensor, b, C_clusters: int, init_labels=None, init_rows=None, iters: int = 0,
                    radius_slack: float = 2.0 ** -14, stream=None, centroid_bf16: bool = False,
                    bias_table_m: int = 0, spherical: bool = False) -> CsvIndex:
    """W: [V,d] 16-bit CUDA tensor (bf16 patterns, original token order); b: float32 CUDA [V] or None.
    init_labels / init_rows: host int32 numpy arrays (see csv_build_opts)."""
    import numpy as np
    _dev2(W, "W")
    V, d = W.shape
    keep = []
    opts = BuildOpts(iters=iters, h_init_labels=None, h_init_rows=None, radius_slack=radius_slack,
                     centroid_bf16=int(bool(centroid_bf16)), spherical=int(bool(spherical)), bias_table_m=int(bias_table_m))
    if init_labels is not None:
        a = np.ascontiguousarray(init_labels, dtype=np.int32)
        assert a.shape == (V,)
        keep.append(a)
        opts.h_init_labels = a.ctypes.data
    if init_rows is not None:
        a = np.ascontiguousarray(init_rows, dtype=np.int32)
        assert a.shape == (C_clusters,)
        keep.append(a)
        opts.h_init_rows = a.ctypes.data
    out = C.c_void_p()
    bptr = None if b is None else b.data_ptr()
    if b is not None:
        assert b.is_cuda and b.dtype == torch.float32 and b.is_contiguous() and b.numel() == V
    _check(lib.csv_build_index(W.data_ptr(), bptr, V, d, C_clusters, C.byref(opts), _stream(stream), C.byref(out)))
    return CsvIndex(out.value)


def csv_index_from_arrays(W: torch.Tensor, b, mu, R, bmax, n, perm, stream=None, centroid_bf16: bool = False) -> CsvIndex:
    """Import metadata computed elsewhere (host numpy arrays).  centroid_bf16: mu holds bfloat16 values (and the
    radii were measured to them); the index then keeps and reads the centroids as bfloat16."""
    import numpy as np
    _dev2(W, "W")
    V, d = W.shape
    mu = np.ascontiguousarray(mu, dtype=np.float32)
    R = np.ascontiguousarray(R, dtype=np.float32)
    bmax = np.ascontiguousarray(bmax, dtype=np.float32)
    n = np.ascontiguousarray(n, dtype=np.int32)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    Cc = mu.shape[0]
    assert mu.shape == (Cc, d) and R.shape == (Cc,) and bmax.shape == (Cc,) and n.shape == (Cc,) and perm.shape == (V,)
    out = C.c_void_p()
    bptr = None if b is None else b.data_ptr()
    _check(lib.csv_index_from_arrays(W.data_ptr(), bptr, V, d, Cc, mu.ctypes.data, R.ctypes.data, bmax.ctypes.data,
                                     n.ctypes.data, perm.ctypes.data, _stream(stream), C.byref(out)))
    idx = CsvIndex(out.value)
    if centroid_bf16:
        _check(lib.csv_index_use_bf16_centroids(idx._h, _stream(stream)))
    return idx


class CsvWorkspace:
    def __init__(self, index: CsvIndex, B_max: int, K_cap_rows: int):
        out = C.c_void_p()
        _check(lib.csv_workspace_create(index._h, B_max, K_cap_rows, C.byref(out)))
        self._h = out
        self.index = index
        self.B_max, self.K_cap = B_max, K_cap_rows

    def set_tail_split(self, min_batch: int) -> None:
        """Batches of at least min_batch sequences run the tail as one launch per phase (0 = follow recent steps)."""
        _check(lib.csv_workspace_set_tail_split(self._h, min_batch))

    def set_spin_limit(self, polls: int) -> None:
        """Polls a grid barrier of the tail kernel waits before giving the step up (0 = default)."""
        _check(lib.csv_workspace_set_spin_limit(self._h, polls))

    def profile_begin(self, max_steps: int) -> None:
        _check(lib.csv_profile_begin(self._h, max_steps))

    def profile_end(self) -> tuple[dict, int]:
        """(summed milliseconds per stage, recorded steps)."""
        ms = (C.c_float * len(PROFILE_STAGES))()
        n = C.c_int()
        _check(lib.csv_profile_end(self._h, ms, C.byref(n)))
        return dict(zip(PROFILE_STAGES, list(ms))), n.value

    def free(self) -> None:
        if self._h:
            lib.csv_workspace_free(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


@dataclass
class StepBuffers:
    """Device output buffers of csv_decode_step plus the ctypes structs that point at them."""
    ids: torch.Tensor
    logits: torch.Tensor
    lse: torch.Tensor
    flags: torch.Tensor
    n_rows: torch.Tensor
    n_clusters: torch.Tensor
    rounds: torch.Tensor
    sel_clusters: torch.Tensor | None
    fallback_count: torch.Tensor
    params: StepParams
    out: StepOut
    probs: torch.Tensor | None = None
    cum: torch.Tensor | None = None
    nucleus: torch.Tensor | None = None


def make_step_buffers(index: CsvIndex, B: int, k: int, eps: float, K_max_rows: int, combine: int = COMBINE_ALL,
                      want_sel: bool = False, device="cuda", max_rounds: int = 0, delta_clusters: int = 0,
                      relax: bool = False, want_dist: bool = False, top_p: float = 0.0, schedule: int = 0) -> StepBuffers:
    kk = max(k, 1)
    ids = torch.full((B, kk), -2, dtype=torch.int32, device=device)
    logits = torch.zeros((B, kk), dtype=torch.float32, device=device)
    lse = torch.zeros(B, dtype=torch.float32, device=device)
    flags = torch.zeros(B, dtype=torch.int32, device=device)
    n_rows = torch.zeros(B, dtype=torch.int32, device=device)
    n_clusters = torch.zeros(B, dtype=torch.int32, device=device)
    rounds = torch.zeros(B, dtype=torch.int32, device=device)
    sel = torch.full((B, index.C), -1, dtype=torch.int32, device=device) if want_sel else None
    fbc = torch.zeros(1, dtype=torch.int64, device=device)
    probs = torch.full((B, kk), -1.0, dtype=torch.float32, device=device) if want_dist else None
    cum = torch.full((B, kk), -1.0, dtype=torch.float32, device=device) if want_dist else None
    nucleus = torch.full((B,), -1, dtype=torch.int32, device=device) if want_dist else None
    params = StepParams(k=k, eps=eps, K_max_rows=K_max_rows, combine=combine, max_rounds=max_rounds,
                        delta_clusters=delta_clusters, relax=int(bool(relax)), top_p=top_p, schedule=schedule)
    out = StepOut(ids.data_ptr(), logits.data_ptr(), lse.data_ptr(), flags.data_ptr(), n_rows.data_ptr(),
                  n_clusters.data_ptr(), rounds.data_ptr(), sel.data_ptr() if want_sel else None, fbc.data_ptr(),
                  probs.data_ptr() if want_dist else None, cum.data_ptr() if want_dist else None,
                  nucleus.data_ptr() if want_dist else None)
    return StepBuffers(ids, logits, lse, flags, n_rows, n_clusters, rounds, sel, fbc, params, out, probs, cum, nucleus)


def csv_decode_step(ws: CsvWorkspace, index: CsvIndex, h: torch.Tensor, buf: StepBuffers, stream=None) -> StepBuffers:
    """Enqueue one certified decode step for h [B,d] (bf16 patterns).  Results land in `buf` after a stream sync."""
    _dev2(h, "h")
    B = h.shape[0]
    _check(lib.csv_decode_step(ws._h, index._h, h.data_ptr(), B, C.byref(buf.params), C.byref(buf.out), _stream(stream)))
    return buf


def csv_decode_step_raw(ws: CsvWorkspace, index: CsvIndex, h_ptr: int, B: int, buf: StepBuffers, stream_ptr: int) -> None:
    """Same call with a raw device pointer and stream handle (tight loops: no tensor checks)."""
    rc = lib.csv_decode_step(ws._h, index._h, h_ptr, B, C.byref(buf.params), C.byref(buf.out), stream_ptr)
    if rc:
        raise CsvError(rc)


def csv_bounds(ws: CsvWorkspace, index: CsvIndex, h: torch.Tensor, stream=None):
    _dev2(h, "h")
    B = h.shape[0]
    U = torch.empty((B, index.C), dtype=torch.float32, device=h.device)
    hn = torch.empty(B, dtype=torch.float32, device=h.device)
    _check(lib.csv_bounds(ws._h, index._h, h.data_ptr(), B, U.data_ptr(), hn.data_ptr(), _stream(stream)))
    return U, hn


def csv_bounds_static(index: CsvIndex, h: torch.Tensor, U: torch.Tensor, hn: torch.Tensor, stream=None) -> None:
    """csv_bounds without a workspace and without any allocation: the caller passes the output tensors
    U [B,C] float32 and hn [B] float32."""
    _dev2(h, "h")
    B = h.shape[0]
    assert U.is_cuda and U.dtype == torch.float32 and U.is_contiguous() and tuple(U.shape) == (B, index.C)
    assert hn.is_cuda and hn.dtype == torch.float32 and hn.is_contiguous() and hn.numel() == B
    _check(lib.csv_bounds_static(index._h, h.data_ptr(), B, U.data_ptr(), hn.data_ptr(), _stream(stream)))


def csv_full_logits(ws: CsvWorkspace, index: CsvIndex, h: torch.Tensor, out: torch.Tensor | None = None, stream=None):
    _dev2(h, "h")
    B = h.shape[0]
    if out is None:
        out = torch.empty((B, index.V), dtype=torch.float32, device=h.device)
    _check(lib.csv_full_logits(ws._h, index._h, h.data_ptr(), B, out.data_ptr(), _stream(stream)))
    return out


def bits_to_device(bits) -> torch.Tensor:
    """numpy uint16 bf16 patterns -> CUDA int16 tensor with the same bits."""
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


class KmaxController:
    """Host-side adaptive row budget (csv_kmax_init / csv_kmax_update)."""

    def __init__(self, K0: int, K_min: int, K_cap: int, alpha: float = 0.01, rho_target: float = 0.02, literal: bool = False):
        self.ctl = KmaxCtl()
        _check(lib.csv_kmax_init(C.byref(self.ctl), K0, K_min, K_cap, alpha, rho_target, int(literal)))

    def update(self, n_fallback: int, n_sequences: int) -> int:
        rc = lib.csv_kmax_update(C.byref(self.ctl), n_fallback, n_sequences)
        if rc < 0:
            raise CsvError(rc)
        return rc

    @property
    def value(self) -> float:
        return self.ctl.K_max
