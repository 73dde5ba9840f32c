"""CPU oracle for the MaxK-GNN aggregation path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``maxk_oracle.c`` (plain C, fp64 accumulation, the
definitions of Sec. 3.1-3.2 / Eq. 1-3 of the paper written out).  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import this package;
the HIP library and its Python binding never do, and this package imports
nothing from them.

Functions take and return NumPy arrays:

    topk_cbsr(H, k)                          -> sp_data f32 [N,k], sp_index i32 [N,k]
    spgemm_fwd(rowptr, col, val, sp_data, sp_index, dim, rows=None) -> Y f64, Yabs f64
    sspmm_bwd(rowptr, col, val, dY, sp_index, nodes=None)           -> D f64, Dabs f64
    spmm(rowptr, col, val, H, rows=None)                            -> Y f64, Yabs f64
    cbsr_scatter(dXs, sp_index, dim)                                -> dH f32 [N,dim]
    narrow(x, value_type)  fp32 -> uint16 patterns ("bf16" or "f16", round to nearest even)
    widen(h, value_type)   uint16 patterns -> the fp32 values they stand for

``rows`` / ``nodes`` restrict the outputs to a sample (full-size parity checks
compute sampled outputs one by one).  The ``*abs`` arrays hold, per output
element, the sum of |terms|, which the parity bound is stated in.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_LIB_PATH = _HERE / "liboracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile maxk_oracle.c into liboracle.so (gcc, OpenMP)."""
    src = _HERE / "maxk_oracle.c"
    if force or not _LIB_PATH.exists() or _LIB_PATH.stat().st_mtime < src.stat().st_mtime:
        tmp = _LIB_PATH.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", str(src), "-o", str(tmp), "-lm"]
        )
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(str(_LIB_PATH))
    i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
    lib.oracle_topk_cbsr.argtypes = [vp, i64, i32, i32, vp, vp]
    lib.oracle_topk_cbsr.restype = ctypes.c_int
    lib.oracle_spgemm_fwd.argtypes = [i64, vp, vp, vp, vp, vp, i32, i32, vp, i64, vp, vp]
    lib.oracle_spgemm_fwd.restype = ctypes.c_int
    lib.oracle_spmm.argtypes = [i64, vp, vp, vp, vp, i32, vp, i64, vp, vp]
    lib.oracle_spmm.restype = ctypes.c_int
    lib.oracle_sspmm_bwd.argtypes = [i64, vp, vp, vp, vp, vp, i32, i32, vp, i64, i64, i64, vp, vp]
    lib.oracle_sspmm_bwd.restype = ctypes.c_int
    lib.oracle_cbsr_scatter.argtypes = [vp, vp, i64, i32, i32, vp]
    lib.oracle_cbsr_scatter.restype = ctypes.c_int
    lib.oracle_narrow.argtypes = [vp, i64, i32, vp]
    lib.oracle_narrow.restype = ctypes.c_int
    lib.oracle_widen.argtypes = [vp, i64, i32, vp]
    lib.oracle_widen.restype = ctypes.c_int
    lib.oracle_num_threads.argtypes = []
    lib.oracle_num_threads.restype = i32
    _lib = lib
    return lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def topk_cbsr(H: np.ndarray, k: int):
    """MaxK + CBSR packing (Sec. 3.1 definition; Sec. 3.2): see oracle_topk_cbsr."""
    H = _c(H, np.float32)
    N, dim = H.shape
    sp_data = np.empty((N, k), dtype=np.float32)
    sp_index = np.empty((N, k), dtype=np.int32)
    rc = _load().oracle_topk_cbsr(_p(H), N, dim, k, _p(sp_data), _p(sp_index))
    if rc != 0:
        raise ValueError("oracle_topk_cbsr: bad arguments or NaN in H")
    return sp_data, sp_index


def spgemm_fwd(rowptr, col, val, sp_data, sp_index, dim: int, rows=None):
    """Forward aggregation Y = A * MaxK(H) from the CBSR (Eq. 2 left)."""
    rowptr, col, val = _c(rowptr, np.int32), _c(col, np.int32), _c(val, np.float32)
    sp_data, sp_index = _c(sp_data, np.float32), _c(sp_index, np.int32)
    N = rowptr.shape[0] - 1
    k = sp_data.shape[1]
    assert sp_data.shape == (N, k) and sp_index.shape == (N, k)
    if rows is not None:
        rows = _c(rows, np.int64)
        n_out = rows.shape[0]
    else:
        n_out = N
    Y = np.empty((n_out, dim), dtype=np.float64)
    Yabs = np.empty((n_out, dim), dtype=np.float64)
    rc = _load().oracle_spgemm_fwd(N, _p(rowptr), _p(col), _p(val), _p(sp_data), _p(sp_index), dim, k, _p(rows),
                                   n_out, _p(Y), _p(Yabs))
    if rc != 0:
        raise ValueError("oracle_spgemm_fwd: bad arguments")
    return Y, Yabs


def spmm(rowptr, col, val, H, rows=None):
    """Dense-feature SpMM Y = A * H (the comparison operator of Sec. 5.2)."""
    rowptr, col, val = _c(rowptr, np.int32), _c(col, np.int32), _c(val, np.float32)
    H = _c(H, np.float32)
    N = rowptr.shape[0] - 1
    dim = H.shape[1]
    if rows is not None:
        rows = _c(rows, np.int64)
        n_out = rows.shape[0]
    else:
        n_out = N
    Y = np.empty((n_out, dim), dtype=np.float64)
    Yabs = np.empty((n_out, dim), dtype=np.float64)
    rc = _load().oracle_spmm(N, _p(rowptr), _p(col), _p(val), _p(H), dim, _p(rows), n_out, _p(Y), _p(Yabs))
    if rc != 0:
        raise ValueError("oracle_spmm: bad arguments")
    return Y, Yabs


def cbsr_scatter(dXs, sp_index, dim: int):
    """MaxK backward: dense dH with dXs placed at the CBSR columns, zeros elsewhere (Sec. 3.1 definition (ii))."""
    dXs, sp_index = _c(dXs, np.float32), _c(sp_index, np.int32)
    N, k = dXs.shape
    assert sp_index.shape == (N, k)
    dH = np.empty((N, dim), dtype=np.float32)
    rc = _load().oracle_cbsr_scatter(_p(dXs), _p(sp_index), N, dim, k, _p(dH))
    if rc != 0:
        raise ValueError("oracle_cbsr_scatter: bad arguments")
    return dH


def sspmm_bwd(rowptr, col, val, dY, sp_index, nodes=None, src_range=None):
    """Backward aggregation dXs = (A^T dY) sampled at sp_index (Eq. 2 right, Eq. 3, Alg. 2).

    ``nodes``: output only these destination nodes (rows of the result follow
    the order given).  ``src_range``: (begin, end) restriction of the source
    rows, used only to bound a timed sample.
    """
    rowptr, col, val = _c(rowptr, np.int32), _c(col, np.int32), _c(val, np.float32)
    dY, sp_index = _c(dY, np.float32), _c(sp_index, np.int32)
    N = rowptr.shape[0] - 1
    dim = dY.shape[1]
    k = sp_index.shape[1]
    assert dY.shape[0] == N and sp_index.shape[0] == N
    slot = None
    n_out = N
    if nodes is not None:
        nodes = _c(nodes, np.int64)
        assert np.unique(nodes).shape[0] == nodes.shape[0], "sampled nodes must be distinct"
        slot = np.full(N, -1, dtype=np.int64)
        slot[nodes] = np.arange(nodes.shape[0], dtype=np.int64)
        n_out = nodes.shape[0]
    b, e = (0, N) if src_range is None else src_range
    D = np.empty((n_out, k), dtype=np.float64)
    Dabs = np.empty((n_out, k), dtype=np.float64)
    rc = _load().oracle_sspmm_bwd(N, _p(rowptr), _p(col), _p(val), _p(dY), _p(sp_index), dim, k, _p(slot), n_out,
                                  b, e, _p(D), _p(Dabs))
    if rc != 0:
        raise ValueError("oracle_sspmm_bwd: bad arguments")
    return D, Dabs


_VALUE_TYPES = {"bf16": 1, "f16": 2}


def narrow(x, value_type: str) -> np.ndarray:
    """CBSR values in 2 bytes: the uint16 bit patterns of x rounded to nearest even ("bf16" or "f16")."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    if _load().oracle_narrow(_p(x), x.size, _VALUE_TYPES[value_type], _p(out)) != 0:
        raise ValueError("oracle_narrow: NaN in the input or bad type")
    return out


def widen(h, value_type: str) -> np.ndarray:
    """The fp32 values that uint16 patterns of the given 16-bit format stand for (exact)."""
    h = _c(h, np.uint16)
    out = np.empty(h.shape, np.float32)
    if _load().oracle_widen(_p(h), h.size, _VALUE_TYPES[value_type], _p(out)) != 0:
        raise ValueError("oracle_widen: bad type")
    return out
