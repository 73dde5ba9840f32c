"""ctypes binding of libmaxk.so (see include/maxk.h for the contract of each call)."""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional

import torch

_HERE = Path(__file__).resolve().parent
_LIB: Optional[ctypes.CDLL] = None

BWD_AUTO, BWD_PULL_CSC, BWD_PUSH_CSR, BWD_EXPAND_REDUCE, BWD_SLAB_PULL, BWD_TILED = 0, 1, 2, 3, 4, 5
VALUE_F32, VALUE_BF16, VALUE_F16 = 0, 1, 2

EXPORTS = (
    "maxk_graph_create", "maxk_graph_destroy", "maxk_graph_reserve", "maxk_graph_reserve_narrow",
    "maxk_graph_set_bwd_mode", "maxk_graph_bwd_choice",
    "maxk_graph_info",
    "maxk_topk_cbsr", "maxk_spgemm_fwd", "maxk_spgemm_fwd_noalloc", "maxk_topk_cbsr_narrow", "maxk_spgemm_fwd_narrow", "maxk_sspmm_bwd",
    "maxk_sspmm_bwd_narrow", "maxk_cbsr_scatter", "spmm_baseline", "maxk_status_string",
    "maxk_last_hip_error", "maxk_version", "maxk_fwd_private_copies", "maxk_graph_cached_tables",
)


class MaxKError(RuntimeError):
    pass


def lib_path() -> Path:
    return _HERE / "libmaxk.so"


def load_library() -> ctypes.CDLL:
    """Loads the in-tree libmaxk.so; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    p = lib_path()
    if not p.exists():
        raise MaxKError(f"{p} not found: build it first (python -m paper_2312_08656_amd.build); there is no fallback path")
    lib = ctypes.CDLL(str(p))
    i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    lib.maxk_graph_create.argtypes = [ctypes.POINTER(vp), i64, i64, vp, vp, vp, vp]
    lib.maxk_graph_destroy.argtypes = [vp]
    lib.maxk_graph_reserve.argtypes = [vp, i32, i32]
    lib.maxk_graph_reserve_narrow.argtypes = [vp, i32, i32, i32]
    lib.maxk_graph_set_bwd_mode.argtypes = [vp, i32]
    lib.maxk_graph_bwd_choice.argtypes = [vp, i32, i32]
    lib.maxk_graph_bwd_choice.restype = i32
    lib.maxk_graph_info.argtypes = [vp] + [ctypes.POINTER(i64)] * 6
    lib.maxk_topk_cbsr.argtypes = [vp, i64, i32, i32, vp, vp, i32, vp]
    lib.maxk_spgemm_fwd.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    lib.maxk_spgemm_fwd_noalloc.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    lib.maxk_topk_cbsr_narrow.argtypes = [vp, i64, i32, i32, vp, i32, vp, i32, vp]
    lib.maxk_spgemm_fwd_narrow.argtypes = [vp, vp, i32, vp, i32, i32, i32, vp, vp]
    lib.maxk_sspmm_bwd.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    lib.maxk_sspmm_bwd_narrow.argtypes = [vp, vp, i32, vp, i32, i32, i32, vp, vp]
    lib.maxk_cbsr_scatter.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp]
    lib.spmm_baseline.argtypes = [vp, vp, i32, vp, vp]
    for name in ("maxk_graph_create", "maxk_graph_destroy", "maxk_graph_reserve", "maxk_graph_reserve_narrow",
                 "maxk_graph_set_bwd_mode",
                 "maxk_graph_info", "maxk_topk_cbsr", "maxk_spgemm_fwd", "maxk_spgemm_fwd_noalloc", "maxk_topk_cbsr_narrow",
                 "maxk_spgemm_fwd_narrow", "maxk_sspmm_bwd", "maxk_sspmm_bwd_narrow", "maxk_cbsr_scatter",
                 "spmm_baseline",
                 "maxk_last_hip_error", "maxk_version"):
        getattr(lib, name).restype = i32
    lib.maxk_status_string.argtypes = [i32]
    lib.maxk_status_string.restype = ctypes.c_char_p
    lib.maxk_fwd_private_copies.argtypes = [i32]
    lib.maxk_graph_cached_tables.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.maxk_graph_cached_tables.restype = i32
    lib.maxk_fwd_private_copies.restype = i32
    lib.maxk_last_hip_error.argtypes = []
    lib.maxk_version.argtypes = []
    _LIB = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != 0:
        lib = load_library()
        msg = lib.maxk_status_string(status).decode()
        raise MaxKError(f"{what}: {msg} (status {status}, hipError {lib.maxk_last_hip_error()})")


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, what: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise MaxKError(f"{what}: expected a contiguous device tensor of {dtype}")
    return t.data_ptr()


def index_dtype(index_bytes: int):
    return {1: torch.uint8, 2: torch.uint16, 4: torch.int32}[index_bytes]


_INDEX_BYTES = {torch.uint8: 1, torch.uint16: 2, torch.int16: 2, torch.int32: 4}
_VALUE_TYPE = {torch.float32: VALUE_F32, torch.bfloat16: VALUE_BF16, torch.float16: VALUE_F16}


class MaxKGraph:
    """Owns a maxk_graph handle and keeps the CSR tensors it aliases alive."""

    def __init__(self, rowptr: torch.Tensor, colidx: torch.Tensor, val: torch.Tensor):
        lib = load_library()
        self.N = int(rowptr.shape[0]) - 1
        self.nnz = int(colidx.shape[0])
        self._keep = (rowptr, colidx, val)
        self._h = ctypes.c_void_p()
        _check(lib.maxk_graph_create(ctypes.byref(self._h), self.N, self.nnz, _dev(rowptr, torch.int32, "rowptr"),
                                     _dev(colidx, torch.int32, "colidx") if self.nnz else None,
                                     _dev(val, torch.float32, "val") if self.nnz else None, _stream()),
               "maxk_graph_create")

    @property
    def handle(self):
        if not self._h:
            raise MaxKError("graph handle already destroyed")
        return self._h

    def reserve(self, dim: int, k: int, dy_dtype=torch.float32) -> None:
        """Builds every workspace and table that compute calls with (dim' <= dim, k' <= k; backward: this dim, k and
        dY dtype) need, so that they allocate nothing."""
        _check(load_library().maxk_graph_reserve_narrow(self.handle, dim, k, _VALUE_TYPE[dy_dtype]),
               "maxk_graph_reserve_narrow")

    def set_bwd_mode(self, mode: int) -> None:
        _check(load_library().maxk_graph_set_bwd_mode(self.handle, mode), "maxk_graph_set_bwd_mode")

    def bwd_choice(self, dim: int, k: int) -> str:
        """Name of the backward kernel maxk_sspmm_bwd would run for (dim, k)."""
        c = load_library().maxk_graph_bwd_choice(self.handle, dim, k)
        if c < 0:
            _check(c, "maxk_graph_bwd_choice")
        return {BWD_PULL_CSC: "pull", BWD_PUSH_CSR: "push", BWD_EXPAND_REDUCE: "expand_reduce",
                BWD_SLAB_PULL: "slab_pull", BWD_TILED: "tiled"}[c]

    def info(self) -> dict:
        vals = [ctypes.c_int64() for _ in range(6)]
        _check(load_library().maxk_graph_info(self.handle, *[ctypes.byref(v) for v in vals]), "maxk_graph_info")
        names = ("N", "nnz", "n_fwd_items", "n_split_rows", "max_degree", "workspace_bytes")
        return {n: int(v.value) for n, v in zip(names, vals)}

    def cached_tables(self) -> tuple:
        """(slab tables, tiled visit lists) the handle holds -- a test hook."""
        a, b = ctypes.c_int32(), ctypes.c_int32()
        _check(load_library().maxk_graph_cached_tables(self.handle, ctypes.byref(a), ctypes.byref(b)),
               "maxk_graph_cached_tables")
        return int(a.value), int(b.value)

    def destroy(self) -> None:
        if self._h:
            load_library().maxk_graph_destroy(self._h)
            self._h = ctypes.c_void_p()
            self._keep = ()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def maxk_graph_create(rowptr: torch.Tensor, colidx: torch.Tensor, val: torch.Tensor) -> MaxKGraph:
    return MaxKGraph(rowptr, colidx, val)


def maxk_graph_destroy(g: MaxKGraph) -> None:
    g.destroy()


def maxk_topk_cbsr(H: torch.Tensor, k: int, sp_data: torch.Tensor, sp_index: torch.Tensor) -> None:
    """sp_data [N,k] fp32 and sp_index [N,k] (uint8 / uint16 / int32) are overwritten."""
    N, dim = H.shape
    ib = _INDEX_BYTES[sp_index.dtype]
    if tuple(sp_data.shape) != (N, k) or tuple(sp_index.shape) != (N, k):
        raise MaxKError("maxk_topk_cbsr: sp_data / sp_index must be [N, k]")
    _check(load_library().maxk_topk_cbsr(_dev(H, torch.float32, "H"), N, dim, k, _dev(sp_data, torch.float32, "sp_data"),
                                         _dev(sp_index, sp_index.dtype, "sp_index"), ib, _stream()), "maxk_topk_cbsr")


def maxk_spgemm_fwd(g: MaxKGraph, sp_data: torch.Tensor, sp_index: torch.Tensor, dim: int, Y: torch.Tensor) -> None:
    """Y [N,dim] fp32 is overwritten with A * X, X given as CBSR."""
    N, k = sp_data.shape
    if N != g.N or tuple(sp_index.shape) != (N, k) or tuple(Y.shape) != (N, dim):
        raise MaxKError("maxk_spgemm_fwd: shape mismatch")
    ib = _INDEX_BYTES[sp_index.dtype]
    _check(load_library().maxk_spgemm_fwd(g.handle, _dev(sp_data, torch.float32, "sp_data"),
                                          _dev(sp_index, sp_index.dtype, "sp_index"), ib, dim, k,
                                          _dev(Y, torch.float32, "Y"), _stream()), "maxk_spgemm_fwd")


def maxk_spgemm_fwd_noalloc(g: MaxKGraph, sp_data: torch.Tensor, sp_index: torch.Tensor, dim: int,
                            Y: torch.Tensor) -> None:
    """maxk_spgemm_fwd with its scratch memory in the library's fixed device array: allocates nothing."""
    N, k = sp_data.shape
    if N != g.N or tuple(sp_index.shape) != (N, k) or tuple(Y.shape) != (N, dim):
        raise MaxKError("maxk_spgemm_fwd_noalloc: shape mismatch")
    ib = _INDEX_BYTES[sp_index.dtype]
    _check(load_library().maxk_spgemm_fwd_noalloc(g.handle, _dev(sp_data, torch.float32, "sp_data"),
                                                  _dev(sp_index, sp_index.dtype, "sp_index"), ib, dim, k,
                                                  _dev(Y, torch.float32, "Y"), _stream()), "maxk_spgemm_fwd_noalloc")


def maxk_topk_cbsr_narrow(H: torch.Tensor, k: int, sp_data: torch.Tensor, sp_index: torch.Tensor) -> None:
    """As maxk_topk_cbsr, the values stored in sp_data's own dtype (bfloat16, float16 or float32)."""
    N, dim = H.shape
    ib = _INDEX_BYTES[sp_index.dtype]
    if sp_data.dtype not in _VALUE_TYPE:
        raise MaxKError("maxk_topk_cbsr_narrow: sp_data must be float32, bfloat16 or float16")
    if tuple(sp_data.shape) != (N, k) or tuple(sp_index.shape) != (N, k):
        raise MaxKError("maxk_topk_cbsr_narrow: sp_data / sp_index must be [N, k]")
    _check(load_library().maxk_topk_cbsr_narrow(_dev(H, torch.float32, "H"), N, dim, k,
                                                _dev(sp_data, sp_data.dtype, "sp_data"), _VALUE_TYPE[sp_data.dtype],
                                                _dev(sp_index, sp_index.dtype, "sp_index"), ib, _stream()),
           "maxk_topk_cbsr_narrow")


def maxk_spgemm_fwd_narrow(g: MaxKGraph, sp_data: torch.Tensor, sp_index: torch.Tensor, dim: int,
                           Y: torch.Tensor) -> None:
    """As maxk_spgemm_fwd with the CBSR values in sp_data's own dtype (bfloat16, float16 or float32)."""
    N, k = sp_data.shape
    if sp_data.dtype not in _VALUE_TYPE:
        raise MaxKError("maxk_spgemm_fwd_narrow: sp_data must be float32, bfloat16 or float16")
    if N != g.N or tuple(sp_index.shape) != (N, k) or tuple(Y.shape) != (N, dim):
        raise MaxKError("maxk_spgemm_fwd_narrow: shape mismatch")
    ib = _INDEX_BYTES[sp_index.dtype]
    _check(load_library().maxk_spgemm_fwd_narrow(g.handle, _dev(sp_data, sp_data.dtype, "sp_data"),
                                                 _VALUE_TYPE[sp_data.dtype], _dev(sp_index, sp_index.dtype, "sp_index"),
                                                 ib, dim, k, _dev(Y, torch.float32, "Y"), _stream()),
           "maxk_spgemm_fwd_narrow")


def maxk_sspmm_bwd(g: MaxKGraph, dY: torch.Tensor, sp_index: torch.Tensor, dXs: torch.Tensor) -> None:
    """dXs [N,k] fp32 is overwritten with (A^T dY) sampled at sp_index."""
    N, dim = dY.shape
    k = sp_index.shape[1]
    if N != g.N or tuple(sp_index.shape) != (N, k) or tuple(dXs.shape) != (N, k):
        raise MaxKError("maxk_sspmm_bwd: shape mismatch")
    ib = _INDEX_BYTES[sp_index.dtype]
    _check(load_library().maxk_sspmm_bwd(g.handle, _dev(dY, torch.float32, "dY"),
                                         _dev(sp_index, sp_index.dtype, "sp_index"), ib, dim, k,
                                         _dev(dXs, torch.float32, "dXs"), _stream()), "maxk_sspmm_bwd")


def maxk_sspmm_bwd_narrow(g: MaxKGraph, dY: torch.Tensor, sp_index: torch.Tensor, dXs: torch.Tensor) -> None:
    """As maxk_sspmm_bwd with dY in its own dtype (bfloat16, float16 or float32); dXs stays fp32."""
    N, dim = dY.shape
    k = sp_index.shape[1]
    if dY.dtype not in _VALUE_TYPE:
        raise MaxKError("maxk_sspmm_bwd_narrow: dY must be float32, bfloat16 or float16")
    if N != g.N or tuple(sp_index.shape) != (N, k) or tuple(dXs.shape) != (N, k):
        raise MaxKError("maxk_sspmm_bwd_narrow: shape mismatch")
    ib = _INDEX_BYTES[sp_index.dtype]
    _check(load_library().maxk_sspmm_bwd_narrow(g.handle, _dev(dY, dY.dtype, "dY"), _VALUE_TYPE[dY.dtype],
                                                _dev(sp_index, sp_index.dtype, "sp_index"), ib, dim, k,
                                                _dev(dXs, torch.float32, "dXs"), _stream()), "maxk_sspmm_bwd_narrow")


def maxk_cbsr_scatter(values: torch.Tensor, sp_index: torch.Tensor, dense: torch.Tensor) -> None:
    """dense [N,dim] fp32 is overwritten: values [N,k] placed at the CBSR columns, zeros elsewhere."""
    N, k = values.shape
    dim = dense.shape[1]
    if tuple(sp_index.shape) != (N, k) or dense.shape[0] != N:
        raise MaxKError("maxk_cbsr_scatter: shape mismatch")
    ib = _INDEX_BYTES[sp_index.dtype]
    _check(load_library().maxk_cbsr_scatter(_dev(values, torch.float32, "values"),
                                            _dev(sp_index, sp_index.dtype, "sp_index"), ib, N, dim, k,
                                            _dev(dense, torch.float32, "dense"), _stream()), "maxk_cbsr_scatter")


def spmm_baseline(g: MaxKGraph, H: torch.Tensor, Y: torch.Tensor) -> None:
    """Y [N,dim] fp32 is overwritten with A * H (dense features)."""
    N, dim = H.shape
    if N != g.N or tuple(Y.shape) != (N, dim):
        raise MaxKError("spmm_baseline: shape mismatch")
    _check(load_library().spmm_baseline(g.handle, _dev(H, torch.float32, "H"), dim, _dev(Y, torch.float32, "Y"),
                                        _stream()), "spmm_baseline")
