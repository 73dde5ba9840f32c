"""Seeded synthetic inputs shaped like the paper's workloads (Table 1 graph sizes,
hidden width 256/384 of Table 4, the k sweep of Section 5.1).

Input manufacture only: no top-k, no aggregation arithmetic lives here.  The
same NumPy arrays are handed to the CPU oracle and (after a copy to HBM) to the
HIP library, so neither side ever sees values produced by the other.

The heavy lifting (R-MAT descent, dedup, CSR build, Box-Muller) is plain C with
OpenMP in ``synth.c``; this module compiles it on first use with gcc, loads it
with ctypes and names the benchmark configurations.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from pathlib import Path
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libsynth.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile synth.c into libsynth.so (gcc, OpenMP)."""
    src = _HERE / "synth.c"
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
    u64, i64, i32, dbl, vp = ctypes.c_uint64, ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
    lib.synth_normal_f32.argtypes = [u64, i64, vp]
    lib.synth_normal_f32.restype = None
    lib.synth_tie_rows.argtypes = [u64, i64, i32, i32, i32, i32, vp]
    lib.synth_tie_rows.restype = i64
    lib.synth_unique_edges.argtypes = [u64, i32, i64, dbl, dbl, dbl, i64, i32, vp]
    lib.synth_unique_edges.restype = i64
    lib.synth_build_csr.argtypes = [vp, i64, i64, i32, i32, vp, vp]
    lib.synth_build_csr.restype = i64
    lib.synth_gcn_weights.argtypes = [i64, vp, vp, vp]
    lib.synth_gcn_weights.restype = None
    lib.synth_mean_weights.argtypes = [i64, vp, vp]
    lib.synth_mean_weights.restype = None
    lib.synth_num_threads.argtypes = []
    lib.synth_num_threads.restype = i32
    _lib = lib
    return lib


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


# --------------------------------------------------------------------------- configs


@dataclass(frozen=True)
class Config:
    """One benchmark workload: graph recipe + feature shape + the k values it is run at."""

    name: str
    N: int
    M: int  # unique non-loop edges drawn (unordered pairs unless directed)
    scale: int  # R-MAT levels; 0 = uniform pairs
    abc: Tuple[float, float, float] = (0.25, 0.25, 0.25)
    directed: bool = False  # True: ordered pairs, not symmetrised (A^T != A)
    dim: int = 256
    ks: Tuple[int, ...] = (32,)
    index_bytes: int = 1
    tie_percent: int = 0  # share of feature rows rewritten as exact-tie rows
    graph_seed: int = 0
    h_seed: int = 1
    dy_seed: int = 2
    stands_for: str = ""

    @property
    def nnz(self) -> int:
        return self.M * (1 if self.directed else 2) + self.N


CONFIGS: Dict[str, Config] = {
    c.name: c
    for c in [
        Config("tiny", 1024, 8192, 0, dim=64, ks=(8,), stands_for="unit-test size"),
        Config("tiny_directed", 1024, 16384, 0, directed=True, dim=64, ks=(8,), stands_for="unit-test size, A^T != A"),
        Config("sparse_mid", 169_343, 1_166_243, 18, (0.57, 0.19, 0.19), dim=256, ks=(16, 32, 64),
               stands_for="ogbn-arxiv row of Table 1"),
        Config("dense", 232_965, 57_307_945, 18, (0.40, 0.22, 0.22), dim=256, ks=(8, 16, 32, 64, 96, 128),
               stands_for="Reddit row of Table 1"),
        Config("large_sparse", 2_449_029, 61_859_140, 22, (0.57, 0.19, 0.19), dim=256, ks=(64,),
               stands_for="ogbn-products row of Table 1"),
        Config("wide_hidden", 716_847, 13_954_819, 20, (0.65, 0.15, 0.15), directed=True, dim=384,
               ks=(32, 96, 192), index_bytes=2, tie_percent=5, stands_for="Yelp row of Table 1, hidden 384"),
        # three more degree profiles from the average-degree > 50 group of the kernel evaluation (Sec. 5.2):
        # a tiny, very dense graph; one denser than the headline; a large one of moderate degree
        Config("ddi_like", 4_267, 1_067_911, 13, (0.30, 0.25, 0.25), dim=256, ks=(8, 16, 32, 64),
               stands_for="ddi row of Table 1"),
        Config("proteins_like", 132_534, 39_561_252, 18, (0.40, 0.22, 0.22), dim=256, ks=(8, 16, 32, 64),
               stands_for="ogbn-proteins row of Table 1"),
        Config("ppa_like", 576_289, 21_231_931, 20, (0.45, 0.22, 0.22), dim=256, ks=(8, 16, 32, 64),
               stands_for="ppa row of Table 1"),
    ]
}


@dataclass
class Graph:
    N: int
    rowptr: np.ndarray  # int32 [N+1]
    col: np.ndarray  # int32 [nnz], sorted & unique per row
    val: np.ndarray  # float32 [nnz]
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.col.shape[0])


# --------------------------------------------------------------------------- graphs


def _cache_dir() -> Optional[Path]:
    d = os.environ.get("MAXK_SYNTH_CACHE", "/tmp/maxk_synth_cache")
    if d in ("", "0", "off"):
        return None
    p = Path(d)
    try:
        p.mkdir(parents=True, exist_ok=True)
    except OSError:
        return None
    return p


def make_graph(N: int, M: int, scale: int, abc=(0.25, 0.25, 0.25), directed: bool = False, self_loops: bool = True,
               seed: int = 0, weights: str = "gcn") -> Graph:
    """First M unique non-loop edges of a seeded candidate stream -> CSR (+ weights).

    Undirected graphs are symmetrised (both directions stored).  ``weights``:
    "gcn" -> 1/sqrt(d_i d_j) with d = stored entries per row, "mean" -> 1/d_i,
    "normal" -> signed N(0,1) values (a general sparse matrix for unit tests).
    """
    lib = _load()
    keys = np.empty(max(M, 1), dtype=np.uint64)
    used = lib.synth_unique_edges(seed, scale, N, float(abc[0]), float(abc[1]), float(abc[2]), M, int(directed),
                                  _ptr(keys))
    if used < 0:
        raise RuntimeError("edge generation failed (too few unique edges available?)")
    nnz = M * (1 if directed else 2) + (N if self_loops else 0)
    rowptr = np.empty(N + 1, dtype=np.int32)
    col = np.empty(max(nnz, 1), dtype=np.int32)
    got = lib.synth_build_csr(_ptr(keys), M, N, int(not directed), int(self_loops), _ptr(rowptr), _ptr(col))
    if got != nnz:
        raise RuntimeError("CSR build failed")
    col = col[:nnz]
    del keys
    g = Graph(N, rowptr, col, np.empty(0, np.float32), {"candidates_used": int(used)})
    g.val = make_weights(g, weights, seed)
    deg = np.diff(rowptr)
    g.meta.update(nnz=int(nnz), max_degree=int(deg.max()) if N else 0, avg_degree=float(nnz) / max(N, 1))
    return g


def make_weights(g: Graph, kind: str = "gcn", seed: int = 0) -> np.ndarray:
    lib = _load()
    val = np.empty(g.col.shape[0], dtype=np.float32)
    if kind == "gcn":
        lib.synth_gcn_weights(g.N, _ptr(g.rowptr), _ptr(g.col), _ptr(val))
    elif kind == "mean":
        lib.synth_mean_weights(g.N, _ptr(g.rowptr), _ptr(val))
    elif kind == "normal":
        lib.synth_normal_f32(seed + 977, val.shape[0], _ptr(val))
    else:
        raise ValueError(kind)
    return val


def graph(name: str) -> Graph:
    """The graph of a named configuration (cached on disk under MAXK_SYNTH_CACHE)."""
    cfg = CONFIGS[name]
    cdir = _cache_dir()
    tag = f"{cfg.name}_N{cfg.N}_M{cfg.M}_s{cfg.scale}_{cfg.abc[0]}_{cfg.abc[1]}_{cfg.abc[2]}_d{int(cfg.directed)}_g{cfg.graph_seed}"
    if cdir is not None and cfg.nnz > 1_000_000:
        fr, fc = cdir / (tag + ".rowptr.npy"), cdir / (tag + ".col.npy")
        if fr.exists() and fc.exists():
            try:
                rowptr, col = np.load(fr), np.load(fc)
                if rowptr.shape[0] == cfg.N + 1 and col.shape[0] == cfg.nnz:
                    g = Graph(cfg.N, rowptr, col, np.empty(0, np.float32), {"cached": True})
                    g.val = make_weights(g, "gcn")
                    deg = np.diff(rowptr)
                    g.meta.update(nnz=int(cfg.nnz), max_degree=int(deg.max()), avg_degree=cfg.nnz / cfg.N)
                    return g
            except Exception:
                pass
    g = make_graph(cfg.N, cfg.M, cfg.scale, cfg.abc, cfg.directed, True, cfg.graph_seed, "gcn")
    if cdir is not None and cfg.nnz > 1_000_000:
        try:
            for arr, suffix in ((g.rowptr, ".rowptr.npy"), (g.col, ".col.npy")):
                tmp = cdir / (tag + suffix + ".tmp%d.npy" % os.getpid())
                np.save(tmp, arr)
                os.replace(tmp, cdir / (tag + suffix))
        except OSError:
            pass
    return g


# --------------------------------------------------------------------------- features


def normal_matrix(N: int, dim: int, seed: int) -> np.ndarray:
    """N x dim fp32 ~ N(0,1), a pure function of (seed, flat index)."""
    lib = _load()
    out = np.empty((N, dim), dtype=np.float32)
    lib.synth_normal_f32(seed, N * dim, _ptr(out))
    return out


def add_tie_rows(H: np.ndarray, seed: int, percent: int = 5, pool: int = 64, const_every: int = 16) -> int:
    """Rewrite `percent`% of rows (hash of row id) so duplicated values straddle every rank."""
    lib = _load()
    N, dim = H.shape
    return int(lib.synth_tie_rows(seed, N, dim, percent, pool, const_every, _ptr(H)))


def features(name: str, which: str = "H") -> np.ndarray:
    """H (seed h_seed) or dY (seed dy_seed) of a named configuration."""
    cfg = CONFIGS[name]
    seed = cfg.h_seed if which == "H" else cfg.dy_seed
    X = normal_matrix(cfg.N, cfg.dim, seed)
    if cfg.tie_percent:
        add_tie_rows(X, seed, cfg.tie_percent)
    return X


def num_threads() -> int:
    return int(_load().synth_num_threads())
