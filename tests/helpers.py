"""Shared test helpers: golden-file parser and NumPy brute-force definitions.

The brute-force routines here are written independently of ``oracle/`` (dense
matrices, library matmul) and are what the oracle is pinned against on tiny
inputs.  They are test code, not part of the oracle or of the product.
"""
from pathlib import Path

import numpy as np

GOLDEN = Path(__file__).resolve().parent / "golden"

# parity bound fixed by the benchmark spec: |err| <= 1e-5 * sum|terms| + 1e-6
REL_TERMS = 1e-5
ABS_FLOOR = 1e-6


def read_golden(name):
    """Parse a [section]-structured text fixture into {section: list of rows of floats}."""
    out, cur = {}, None
    for line in (GOLDEN / name).read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            out[cur] = []
            continue
        out[cur].append(line.split())
    return out


def dense_from_csr(rowptr, col, val, N):
    A = np.zeros((N, N), dtype=np.float64)
    for i in range(N):
        for p in range(rowptr[i], rowptr[i + 1]):
            A[i, col[p]] += float(val[p])  # duplicates add (CSR semantics)
    return A


def csr_from_coo(N, triples):
    triples = sorted(triples, key=lambda t: (t[0], t[1]))
    rowptr = np.zeros(N + 1, dtype=np.int32)
    for i, _, _ in triples:
        rowptr[i + 1] += 1
    rowptr = np.cumsum(rowptr).astype(np.int32)
    col = np.array([t[1] for t in triples], dtype=np.int32)
    val = np.array([t[2] for t in triples], dtype=np.float32)
    return rowptr, col, val


def scatter_cbsr(sp_data, sp_index, dim):
    """Dense N x dim matrix holding the CBSR entries, zeros elsewhere (fp64)."""
    N, k = sp_data.shape
    X = np.zeros((N, dim), dtype=np.float64)
    for i in range(N):
        for t in range(k):
            X[i, sp_index[i, t]] += float(sp_data[i, t])
    return X


def check_topk_properties(H, k, sp_data, sp_index):
    """Oracle-free characterisation of the MaxK/CBSR result (unique answer):
    (1) indices strictly ascending in [0, dim); (2) data bit-equals H there;
    (3) min kept >= max dropped; (4) any dropped column whose value equals the
    smallest kept value lies to the right of every kept column with that value."""
    H = np.asarray(H, dtype=np.float32)
    N, dim = H.shape
    idx = np.asarray(sp_index).astype(np.int64)
    assert idx.shape == (N, k) and sp_data.shape == (N, k)
    assert (idx >= 0).all() and (idx < dim).all()
    if k > 1:
        assert (np.diff(idx, axis=1) > 0).all(), "indices not strictly ascending"
    picked = np.take_along_axis(H, idx, axis=1)
    assert np.array_equal(picked.view(np.uint32), np.asarray(sp_data, dtype=np.float32).view(np.uint32)), \
        "sp_data bits differ from H at sp_index"
    if k == dim:
        return
    kept = np.zeros((N, dim), dtype=bool)
    np.put_along_axis(kept, idx, True, axis=1)
    min_kept = np.where(kept, H, np.inf).min(axis=1)
    max_drop = np.where(~kept, H, -np.inf).max(axis=1)
    assert (min_kept >= max_drop).all(), "a dropped value exceeds a kept one"
    cols = np.arange(dim)[None, :]
    kept_tie = kept & (H == min_kept[:, None])
    drop_tie = (~kept) & (H == min_kept[:, None])
    last_kept_tie = np.where(kept_tie, cols, -1).max(axis=1)
    first_drop_tie = np.where(drop_tie, cols, dim).min(axis=1)
    assert (first_drop_tie > last_kept_tie).all(), "tie at the k-th value not broken toward the lower column"


def within_bound(got, ref, refabs):
    """|got - ref| <= 1e-5 * sum|terms| + 1e-6, elementwise; returns (ok, worst ratio)."""
    err = np.abs(np.asarray(got, dtype=np.float64) - ref)
    bound = REL_TERMS * refabs + ABS_FLOOR
    ratio = float((err / bound).max()) if err.size else 0.0
    return bool((err <= bound).all()), ratio
