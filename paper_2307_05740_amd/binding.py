"""ctypes binding of ``libarrow.so`` (declared in ``include/arrow.h``).

Argument marshalling only: every step of a product runs in the library's HIP
kernels.  The functions carry the C names; :class:`ArrowSpMM` is a small
convenience that owns the torch tensors used as device memory (image and
workspace) for one handle.  There is no CPU fallback: if the shared library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libarrow.so")
_lib = None

ARROW_OK, ARROW_EINVAL, ARROW_ENOMEM, ARROW_ENOTREADY, ARROW_ETOOSMALL, ARROW_EHIP, ARROW_EINTERNAL = \
    0, -1, -2, -3, -4, -5, -6

EXPORTED = [
    "arrow_decompose", "arrow_device_bytes", "arrow_upload", "arrow_workspace_bytes",
    "arrow_set_workspace", "arrow_spmm", "arrow_spmm_static", "arrow_spmm_iter", "arrow_sddmm_device_bytes",
    "arrow_sddmm_upload", "arrow_sddmm", "arrow_export_entry_map", "arrow_gather", "arrow_info",
    "arrow_level_info", "arrow_export_level", "arrow_self_check", "arrow_set_option", "arrow_set_profiling",
    "arrow_get_profile", "arrow_get_level_profile", "arrow_save", "arrow_load", "arrow_last_error",
    "arrow_probe_gather", "arrow_probe_gather_out_bytes",
    "arrow_options_default", "arrow_decompose_with", "arrow_load_with", "arrow_repack",
    "arrow_destroy",
    "csf3_build", "csf3_device_bytes", "csf3_upload", "csf3_workspace_bytes", "csf3_set_workspace",
    "csf3_mttkrp", "csf3_info", "csf3_set_profiling", "csf3_get_profile", "csf3_last_error", "csf3_destroy",
]


class ArrowError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"arrow error {code}: {text}")
        self.code = code


class arrow_info_t(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("nnz", ctypes.c_int64), ("b", ctypes.c_int32),
                ("levels", ctypes.c_int32), ("max_chunks", ctypes.c_int64),
                ("decompose_seconds", ctypes.c_double)]


class arrow_level_info_t(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int64) for name in
                ("n_i", "nnz", "nnz_head_head", "nnz_head_row", "nnz_head_col", "nnz_diag",
                 "short_rows", "chunks", "split_rows", "partials", "nnz_rows", "nnz_chunks",
                 "x_rows_rows", "x_rows_chunks", "window_tiles", "window_rows", "nnz_window",
                 "rows_partials", "chunks_partials", "panel_rows", "panel_bins", "nnz_panel")] + \
               [("blocks", ctypes.c_int32), ("separator_rule", ctypes.c_int32), ("nnz_fused", ctypes.c_int64),
                ("corner", ctypes.c_int64), ("corner_tiles", ctypes.c_int64), ("corner_items", ctypes.c_int64),
                ("nnz_corner", ctypes.c_int64)]


class arrow_options_t(ctypes.Structure):
    _fields_ = [("separators", ctypes.c_int32), ("bfs_tail", ctypes.c_int32), ("head_by_id", ctypes.c_int32),
                ("hubs_first", ctypes.c_int64)] + \
               [(name, ctypes.c_int32) for name in
                ("short_max", "chunk_nnz", "chunk_min", "window_rows", "classes", "class_gran", "class_min",
                 "piece_max", "stage_head", "stage_short", "empty_last", "panel", "panel_min", "window_span",
                 "window_tile_rows")] + \
               [("window_reuse", ctypes.c_double), ("window_level_share", ctypes.c_double)] + \
               [(name, ctypes.c_int32) for name in ("fuse_levels", "corner", "corner_max", "corner_min_tile", "kc")] + \
               [("l2_resident_bytes", ctypes.c_int64)]


class arrow_profile_t(ctypes.Structure):
    _fields_ = [(name, ctypes.c_float) for name in
                ("rows_ms", "chunks_ms", "reduce_ms", "stage_ms", "window_ms", "total_ms")] + \
               [(name, ctypes.c_int32) for name in
                ("rows_launches", "chunks_launches", "reduce_launches", "stage_launches",
                 "window_launches")] + \
               [("panel_ms", ctypes.c_float), ("panel_launches", ctypes.c_int32),
                ("corner_ms", ctypes.c_float), ("corner_launches", ctypes.c_int32)]


class csf3_info_t(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int64) for name in
                ("I", "J", "K", "nnz", "slices", "fibers", "segments", "items", "split_rows", "partials",
                 "distinct_j", "distinct_k")] + [("build_seconds", ctypes.c_double)]


def lib():
    """Load ``libarrow.so``; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           "`python -m paper_2307_05740_amd._build arrow` (no CPU fallback exists)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    L.arrow_decompose.restype = ctypes.c_int
    L.arrow_decompose.argtypes = [i64, vp, vp, vp, i32, ctypes.POINTER(vp)]
    L.arrow_device_bytes.restype = sz
    L.arrow_device_bytes.argtypes = [vp]
    L.arrow_upload.restype = ctypes.c_int
    L.arrow_upload.argtypes = [vp, vp, sz, vp]
    L.arrow_workspace_bytes.restype = sz
    L.arrow_workspace_bytes.argtypes = [vp, i32]
    L.arrow_set_workspace.restype = ctypes.c_int
    L.arrow_set_workspace.argtypes = [vp, vp, sz]
    L.arrow_spmm.restype = ctypes.c_int
    L.arrow_spmm.argtypes = [vp, vp, vp, i32, vp]
    L.arrow_spmm_static.restype = ctypes.c_int
    L.arrow_spmm_static.argtypes = [vp, vp, vp, i32, vp]
    L.arrow_spmm_iter.restype = ctypes.c_int
    L.arrow_spmm_iter.argtypes = [vp, vp, i32, i32, vp]
    L.arrow_sddmm_device_bytes.restype = sz
    L.arrow_sddmm_device_bytes.argtypes = [vp]
    L.arrow_sddmm_upload.restype = ctypes.c_int
    L.arrow_sddmm_upload.argtypes = [vp, vp, sz, vp]
    L.arrow_sddmm.restype = ctypes.c_int
    L.arrow_sddmm.argtypes = [vp, vp, vp, vp, i32, vp]
    L.arrow_export_entry_map.restype = ctypes.c_int
    L.arrow_export_entry_map.argtypes = [vp, vp]
    L.arrow_gather.restype = ctypes.c_int
    L.arrow_gather.argtypes = [vp, i32, vp, vp, i32, vp]
    L.arrow_info.restype = ctypes.c_int
    L.arrow_info.argtypes = [vp, ctypes.POINTER(arrow_info_t)]
    L.arrow_level_info.restype = ctypes.c_int
    L.arrow_level_info.argtypes = [vp, i32, ctypes.POINTER(arrow_level_info_t)]
    L.arrow_export_level.restype = ctypes.c_int
    L.arrow_export_level.argtypes = [vp, i32, vp, vp, vp, vp]
    L.arrow_self_check.restype = ctypes.c_int
    L.arrow_self_check.argtypes = [vp]
    L.arrow_set_option.restype = ctypes.c_int
    L.arrow_set_option.argtypes = [vp, ctypes.c_char_p, i64]
    L.arrow_set_profiling.restype = ctypes.c_int
    L.arrow_set_profiling.argtypes = [vp, i32]
    L.arrow_get_profile.restype = ctypes.c_int
    L.arrow_get_profile.argtypes = [vp, ctypes.POINTER(arrow_profile_t)]
    L.arrow_get_level_profile.restype = ctypes.c_int
    L.arrow_get_level_profile.argtypes = [vp, i32, ctypes.POINTER(arrow_profile_t)]
    L.arrow_save.restype = ctypes.c_int
    L.arrow_save.argtypes = [vp, ctypes.c_char_p]
    L.arrow_load.restype = ctypes.c_int
    L.arrow_load.argtypes = [ctypes.c_char_p, ctypes.POINTER(vp)]
    L.arrow_probe_gather_out_bytes.restype = sz
    L.arrow_probe_gather_out_bytes.argtypes = [i64]
    L.arrow_probe_gather.restype = ctypes.c_int
    L.arrow_probe_gather.argtypes = [vp, i64, i32, i64, i32, i32, i64, vp, sz, vp]
    L.arrow_options_default.restype = None
    L.arrow_options_default.argtypes = [ctypes.POINTER(arrow_options_t)]
    L.arrow_decompose_with.restype = ctypes.c_int
    L.arrow_decompose_with.argtypes = [i64, vp, vp, vp, i32, ctypes.POINTER(arrow_options_t), ctypes.POINTER(vp)]
    L.arrow_load_with.restype = ctypes.c_int
    L.arrow_load_with.argtypes = [ctypes.c_char_p, ctypes.POINTER(arrow_options_t), ctypes.POINTER(vp)]
    L.arrow_repack.restype = ctypes.c_int
    L.arrow_repack.argtypes = [vp, ctypes.POINTER(arrow_options_t)]
    L.arrow_last_error.restype = ctypes.c_char_p
    L.arrow_last_error.argtypes = []
    L.arrow_destroy.restype = None
    L.arrow_destroy.argtypes = [vp]
    L.csf3_build.restype = ctypes.c_int
    L.csf3_build.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, ctypes.POINTER(vp)]
    L.csf3_device_bytes.restype = sz
    L.csf3_device_bytes.argtypes = [vp]
    L.csf3_upload.restype = ctypes.c_int
    L.csf3_upload.argtypes = [vp, vp, sz, vp]
    L.csf3_workspace_bytes.restype = sz
    L.csf3_workspace_bytes.argtypes = [vp, i32]
    L.csf3_set_workspace.restype = ctypes.c_int
    L.csf3_set_workspace.argtypes = [vp, vp, sz]
    L.csf3_mttkrp.restype = ctypes.c_int
    L.csf3_mttkrp.argtypes = [vp, vp, vp, vp, i32, vp]
    L.csf3_info.restype = ctypes.c_int
    L.csf3_info.argtypes = [vp, ctypes.POINTER(csf3_info_t)]
    L.csf3_set_profiling.restype = ctypes.c_int
    L.csf3_set_profiling.argtypes = [vp, i32]
    L.csf3_get_profile.restype = ctypes.c_int
    L.csf3_get_profile.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
    L.csf3_last_error.restype = ctypes.c_char_p
    L.csf3_last_error.argtypes = []
    L.csf3_destroy.restype = None
    L.csf3_destroy.argtypes = [vp]
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != 0:
        raise ArrowError(rc, lib().arrow_last_error().decode())


def arrow_last_error() -> str:
    return lib().arrow_last_error().decode()


def arrow_decompose(rowptr: np.ndarray, colidx: np.ndarray, vals: np.ndarray, b: int,
                    n: int | None = None) -> int:
    """Host CSR (int64 rowptr, int32 colidx, float32 vals) -> opaque handle (an integer address)."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    n = rowptr.shape[0] - 1 if n is None else n
    out = ctypes.c_void_p()
    _check(lib().arrow_decompose(n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, b,
                                 ctypes.byref(out)))
    return out.value


def arrow_options_default(**overrides) -> arrow_options_t:
    """The library's default options (built-in values, then ARROW_* environment overrides), with
    the given fields replaced."""
    opt = arrow_options_t()
    lib().arrow_options_default(ctypes.byref(opt))
    names = {f for f, _ in arrow_options_t._fields_}
    for name, value in overrides.items():
        if name not in names:
            raise KeyError(f"arrow_options_t has no field {name!r}")
        setattr(opt, name, value)
    return opt


def arrow_decompose_with(rowptr: np.ndarray, colidx: np.ndarray, vals: np.ndarray, b: int,
                         opt: arrow_options_t | None, n: int | None = None) -> int:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    n = rowptr.shape[0] - 1 if n is None else n
    out = ctypes.c_void_p()
    _check(lib().arrow_decompose_with(n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, b,
                                      ctypes.byref(opt) if opt is not None else None, ctypes.byref(out)))
    return out.value


def arrow_load_with(path: str, opt: arrow_options_t | None) -> int:
    out = ctypes.c_void_p()
    _check(lib().arrow_load_with(os.fsencode(path), ctypes.byref(opt) if opt is not None else None,
                                 ctypes.byref(out)))
    return out.value


def arrow_repack(h: int, opt: arrow_options_t | None) -> None:
    _check(lib().arrow_repack(h, ctypes.byref(opt) if opt is not None else None))


def arrow_device_bytes(h: int) -> int:
    return int(lib().arrow_device_bytes(h))


def arrow_upload(h: int, dev_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().arrow_upload(h, dev_ptr, nbytes, stream))


def arrow_workspace_bytes(h: int, k: int) -> int:
    return int(lib().arrow_workspace_bytes(h, k))


def arrow_set_workspace(h: int, dev_ptr: int, nbytes: int) -> None:
    _check(lib().arrow_set_workspace(h, dev_ptr, nbytes))


def arrow_spmm(h: int, x_ptr: int, y_ptr: int, k: int, stream: int = 0) -> None:
    _check(lib().arrow_spmm(h, x_ptr, y_ptr, k, stream))


ARROW_STATIC_SCRATCH_BYTES = 64 << 20


def arrow_spmm_static(h: int, x_ptr: int, y_ptr: int, k: int, stream: int = 0) -> None:
    _check(lib().arrow_spmm_static(h, x_ptr, y_ptr, k, stream))


def arrow_spmm_iter(h: int, x_ptr: int, k: int, l: int, stream: int = 0) -> None:
    _check(lib().arrow_spmm_iter(h, x_ptr, k, l, stream))


def arrow_sddmm_device_bytes(h: int) -> int:
    return int(lib().arrow_sddmm_device_bytes(h))


def arrow_sddmm_upload(h: int, dev_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().arrow_sddmm_upload(h, dev_ptr, nbytes, stream))


def arrow_sddmm(h: int, u_ptr: int, v_ptr: int, s_ptr: int, k: int, stream: int = 0) -> None:
    _check(lib().arrow_sddmm(h, u_ptr, v_ptr, s_ptr, k, stream))


def arrow_export_entry_map(h: int) -> np.ndarray:
    """Host copy of the entry map: image order -> index in the caller's CSR arrays."""
    out = np.empty(arrow_info(h)["nnz"], dtype=np.uint32)
    _check(lib().arrow_export_entry_map(h, out.ctypes.data))
    return out


def arrow_gather(h: int, level: int, x_ptr: int, xp_ptr: int, k: int, stream: int = 0) -> None:
    _check(lib().arrow_gather(h, level, x_ptr, xp_ptr, k, stream))


def arrow_info(h: int) -> dict:
    out = arrow_info_t()
    _check(lib().arrow_info(h, ctypes.byref(out)))
    return {f: getattr(out, f) for f, _ in out._fields_}


def arrow_level_info(h: int, level: int) -> dict:
    out = arrow_level_info_t()
    _check(lib().arrow_level_info(h, level, ctypes.byref(out)))
    return {f: getattr(out, f) for f, _ in out._fields_}


def arrow_export_level(h: int, level: int):
    """Host copies ``(perm, rows, cols, vals)`` of level ``level`` in position coordinates."""
    info = arrow_level_info(h, level)
    perm = np.empty(info["n_i"], dtype=np.int32)
    rows = np.empty(info["nnz"], dtype=np.int32)
    cols = np.empty(info["nnz"], dtype=np.int32)
    vals = np.empty(info["nnz"], dtype=np.float32)
    _check(lib().arrow_export_level(h, level, perm.ctypes.data, rows.ctypes.data, cols.ctypes.data,
                                    vals.ctypes.data))
    return perm, rows, cols, vals


def arrow_self_check(h: int) -> None:
    _check(lib().arrow_self_check(h))


def arrow_set_option(h: int, name: str, value: int) -> None:
    _check(lib().arrow_set_option(h, name.encode(), value))


def arrow_set_profiling(h: int, enabled: bool) -> None:
    _check(lib().arrow_set_profiling(h, 1 if enabled else 0))


def arrow_get_profile(h: int) -> dict:
    out = arrow_profile_t()
    _check(lib().arrow_get_profile(h, ctypes.byref(out)))
    return {f: getattr(out, f) for f, _ in out._fields_}


def arrow_get_level_profile(h: int, level: int) -> dict:
    out = arrow_profile_t()
    _check(lib().arrow_get_level_profile(h, level, ctypes.byref(out)))
    return {f: getattr(out, f) for f, _ in out._fields_}


def arrow_save(h: int, path: str) -> None:
    _check(lib().arrow_save(h, os.fsencode(path)))


def arrow_load(path: str) -> int:
    out = ctypes.c_void_p()
    _check(lib().arrow_load(os.fsencode(path), ctypes.byref(out)))
    return out.value


def arrow_probe_gather_out_bytes(gathers: int) -> int:
    return lib().arrow_probe_gather_out_bytes(gathers)


def arrow_probe_gather(x_ptr: int, x_rows: int, k: int, region_rows: int, per_die: bool, from_lds: bool,
                       gathers: int, out_ptr: int, out_bytes: int, stream: int = 0) -> None:
    _check(lib().arrow_probe_gather(x_ptr, x_rows, k, region_rows, int(per_die), int(from_lds), gathers,
                                    out_ptr, out_bytes, stream))


def arrow_destroy(h: int) -> None:
    lib().arrow_destroy(h)


class ArrowSpMM:
    """One decomposed operand bound to torch-owned device memory (plumbing only)."""

    def __init__(self, rowptr=None, colidx=None, vals=None, b: int = 0, device="cuda:0", handle=None,
                 options: arrow_options_t | None = None):
        import torch
        self._torch = torch
        self.device = torch.device(device)
        self.h = handle if handle is not None else arrow_decompose_with(rowptr, colidx, vals, b, options)
        self.info = arrow_info(self.h)
        self.n = self.info["n"]
        self._bind_image()

    def _bind_image(self) -> None:
        torch = self._torch
        nbytes = arrow_device_bytes(self.h)
        with torch.cuda.device(self.device):
            self._image = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
            arrow_upload(self.h, self._image.data_ptr(), self._image.numel(), self._stream())
            torch.cuda.current_stream().synchronize()
        self._ws = None
        self._ws_k = 0
        self._map = None

    def repack(self, options: arrow_options_t | None) -> None:
        """Rebuild the device image with other packing / launch options and bind it again."""
        self._torch.cuda.synchronize(self.device)
        arrow_repack(self.h, options)
        self._bind_image()

    def _stream(self) -> int:
        return self._torch.cuda.current_stream(self.device).cuda_stream

    def _ensure_workspace(self, k: int) -> None:
        if self._ws is not None and self._ws_k >= k:
            return
        torch = self._torch
        torch.cuda.current_stream(self.device).synchronize()
        nbytes = arrow_workspace_bytes(self.h, k)
        self._ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        self._ws_k = k
        arrow_set_workspace(self.h, self._ws.data_ptr(), self._ws.numel())

    def levels(self):
        return [arrow_level_info(self.h, i) for i in range(self.info["levels"])]

    def spmm(self, X, Y=None):
        torch = self._torch
        assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 2 and X.is_contiguous()
        assert X.shape[0] == self.n
        k = X.shape[1]
        if Y is None:
            Y = torch.empty_like(X)
        assert Y.shape == X.shape and Y.dtype == torch.float32 and Y.is_contiguous()
        self._ensure_workspace(k)
        arrow_spmm(self.h, X.data_ptr(), Y.data_ptr(), k, self._stream())
        return Y

    def spmm_iter(self, X, l: int):
        torch = self._torch
        assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 2 and X.is_contiguous()
        assert X.shape[0] == self.n
        self._ensure_workspace(X.shape[1])
        arrow_spmm_iter(self.h, X.data_ptr(), X.shape[1], l, self._stream())
        return X

    def sddmm(self, U, V, S=None):
        """``S[p] = a_p <U[i], V[j]>`` for the nonzeros p = (i, j), in the caller's CSR order."""
        torch = self._torch
        for M in (U, V):
            assert M.is_cuda and M.dtype == torch.float32 and M.dim() == 2 and M.is_contiguous()
            assert M.shape[0] == self.n
        assert U.shape == V.shape
        k = U.shape[1]
        if self._map is None:
            nbytes = arrow_sddmm_device_bytes(self.h)
            self._map = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
            arrow_sddmm_upload(self.h, self._map.data_ptr(), self._map.numel(), self._stream())
            torch.cuda.current_stream(self.device).synchronize()
        if S is None:
            S = torch.empty(self.info["nnz"], dtype=torch.float32, device=self.device)
        assert S.dtype == torch.float32 and S.is_contiguous() and S.numel() == self.info["nnz"]
        self._ensure_workspace(k)
        arrow_sddmm(self.h, U.data_ptr(), V.data_ptr(), S.data_ptr(), k, self._stream())
        return S

    def gather(self, level: int, X):
        torch = self._torch
        n_i = arrow_level_info(self.h, level)["n_i"]
        Xp = torch.empty((n_i, X.shape[1]), dtype=torch.float32, device=self.device)
        arrow_gather(self.h, level, X.data_ptr(), Xp.data_ptr(), X.shape[1], self._stream())
        return Xp

    def close(self) -> None:
        if self.h:
            self._torch.cuda.synchronize(self.device)
            arrow_destroy(self.h)
            self.h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---------------------------------------------------------------------------------------------
# order-3 MTTKRP (include/csf3.h)
# ---------------------------------------------------------------------------------------------
def _check3(rc: int) -> None:
    if rc != 0:
        raise ArrowError(rc, lib().csf3_last_error().decode())


def csf3_last_error() -> str:
    return lib().csf3_last_error().decode()


def csf3_build(dims, ti: np.ndarray, tj: np.ndarray, tk: np.ndarray, tv: np.ndarray) -> int:
    """Host coordinate list (int32 i, j, k; float32 values) -> opaque handle (an integer address)."""
    ti = np.ascontiguousarray(ti, dtype=np.int32)
    tj = np.ascontiguousarray(tj, dtype=np.int32)
    tk = np.ascontiguousarray(tk, dtype=np.int32)
    tv = np.ascontiguousarray(tv, dtype=np.float32)
    assert ti.shape == tj.shape == tk.shape == tv.shape and ti.ndim == 1
    out = ctypes.c_void_p()
    _check3(lib().csf3_build(int(dims[0]), int(dims[1]), int(dims[2]), ti.shape[0], ti.ctypes.data,
                             tj.ctypes.data, tk.ctypes.data, tv.ctypes.data, ctypes.byref(out)))
    return out.value


def csf3_device_bytes(h: int) -> int:
    return int(lib().csf3_device_bytes(h))


def csf3_upload(h: int, dev_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check3(lib().csf3_upload(h, dev_ptr, nbytes, stream))


def csf3_workspace_bytes(h: int, R: int) -> int:
    return int(lib().csf3_workspace_bytes(h, R))


def csf3_set_workspace(h: int, dev_ptr: int, nbytes: int) -> None:
    _check3(lib().csf3_set_workspace(h, dev_ptr, nbytes))


def csf3_mttkrp(h: int, b_ptr: int, c_ptr: int, a_ptr: int, R: int, stream: int = 0) -> None:
    _check3(lib().csf3_mttkrp(h, b_ptr, c_ptr, a_ptr, R, stream))


def csf3_info(h: int) -> dict:
    out = csf3_info_t()
    _check3(lib().csf3_info(h, ctypes.byref(out)))
    return {f: getattr(out, f) for f, _ in out._fields_}


def csf3_set_profiling(h: int, enabled: bool) -> None:
    _check3(lib().csf3_set_profiling(h, 1 if enabled else 0))


def csf3_get_profile(h: int) -> dict:
    a, b = ctypes.c_float(), ctypes.c_float()
    _check3(lib().csf3_get_profile(h, ctypes.byref(a), ctypes.byref(b)))
    return {"kernel_ms": a.value, "reduce_ms": b.value}


def csf3_destroy(h: int) -> None:
    lib().csf3_destroy(h)


class Csf3Mttkrp:
    """One order-3 tensor bound to torch-owned device memory (plumbing only)."""

    def __init__(self, dims, ti, tj, tk, tv, device="cuda:0"):
        import torch
        self._torch = torch
        self.device = torch.device(device)
        self.h = csf3_build(dims, ti, tj, tk, tv)
        self.info = csf3_info(self.h)
        nbytes = csf3_device_bytes(self.h)
        with torch.cuda.device(self.device):
            self._image = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
            csf3_upload(self.h, self._image.data_ptr(), self._image.numel(), self._stream())
            torch.cuda.current_stream().synchronize()
        self._ws = None
        self._ws_R = 0

    def _stream(self) -> int:
        return self._torch.cuda.current_stream(self.device).cuda_stream

    def mttkrp(self, B, C, A=None):
        torch = self._torch
        for M, rows in ((B, self.info["J"]), (C, self.info["K"])):
            assert M.is_cuda and M.dtype == torch.float32 and M.dim() == 2 and M.is_contiguous()
            assert M.shape[0] == rows
        assert B.shape[1] == C.shape[1]
        R = B.shape[1]
        if A is None:
            A = torch.empty((self.info["I"], R), dtype=torch.float32, device=self.device)
        assert A.shape == (self.info["I"], R) and A.dtype == torch.float32 and A.is_contiguous()
        if self._ws is None or self._ws_R < R:
            torch.cuda.current_stream(self.device).synchronize()
            self._ws = torch.empty(csf3_workspace_bytes(self.h, R), dtype=torch.uint8, device=self.device)
            self._ws_R = R
            csf3_set_workspace(self.h, self._ws.data_ptr(), self._ws.numel())
        csf3_mttkrp(self.h, B.data_ptr(), C.data_ptr(), A.data_ptr(), R, self._stream())
        return A

    def close(self) -> None:
        if self.h:
            self._torch.cuda.synchronize(self.device)
            csf3_destroy(self.h)
            self.h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
