"""The seeded input generators: structure of the graphs and features they emit."""
import numpy as np
import scipy.sparse as sp

import synth


def _check_csr(g):
    assert g.rowptr.dtype == np.int32 and g.col.dtype == np.int32 and g.val.dtype == np.float32
    assert g.rowptr[0] == 0 and g.rowptr[-1] == g.nnz
    for i in range(0, g.N, max(1, g.N // 200)):
        c = g.col[g.rowptr[i]:g.rowptr[i + 1]]
        assert (np.diff(c) > 0).all()  # sorted, unique
        assert i in c  # self-loop


def test_tiny_undirected_is_symmetric_with_self_loops():
    g = synth.graph("tiny")
    assert g.nnz == 17_408 == synth.CONFIGS["tiny"].nnz
    _check_csr(g)
    A = sp.csr_matrix((g.val, g.col, g.rowptr), shape=(g.N, g.N))
    assert abs(A - A.T).max() == 0
    deg = np.diff(g.rowptr).astype(np.float64)
    i = np.repeat(np.arange(g.N), np.diff(g.rowptr))
    np.testing.assert_array_equal(g.val, (1.0 / np.sqrt(deg[i] * deg[g.col])).astype(np.float32))


def test_tiny_directed_is_not_symmetric():
    g = synth.graph("tiny_directed")
    assert g.nnz == 16_384 + 1024
    _check_csr(g)
    A = sp.csr_matrix((np.ones_like(g.val), g.col, g.rowptr), shape=(g.N, g.N))
    assert abs(A - A.T).sum() > 1000


def test_rmat_mid_size_is_deterministic_and_skewed():
    cfg = synth.CONFIGS["sparse_mid"]
    g1 = synth.make_graph(cfg.N, cfg.M, cfg.scale, cfg.abc, seed=0)
    g2 = synth.make_graph(cfg.N, cfg.M, cfg.scale, cfg.abc, seed=0)
    assert g1.nnz == cfg.nnz == 2_501_829
    assert np.array_equal(g1.col, g2.col) and np.array_equal(g1.rowptr, g2.rowptr)
    _check_csr(g1)
    assert g1.meta["max_degree"] > 50 * g1.meta["avg_degree"]  # power-law tail
    g3 = synth.make_graph(cfg.N, cfg.M, cfg.scale, cfg.abc, seed=1)
    assert not np.array_equal(g1.col, g3.col)


def test_features_are_standard_normal_and_seeded():
    X = synth.normal_matrix(4000, 256, seed=1)
    assert X.dtype == np.float32
    assert abs(float(X.mean())) < 5e-3 and abs(float(X.std()) - 1.0) < 5e-3
    assert np.array_equal(X, synth.normal_matrix(4000, 256, seed=1))
    assert not np.array_equal(X, synth.normal_matrix(4000, 256, seed=2))
    assert np.isfinite(X).all()


def test_tie_rows_have_duplicates_straddling_ranks():
    X = synth.normal_matrix(4000, 384, seed=3)
    n = synth.add_tie_rows(X, seed=3, percent=5)
    assert 120 < n < 280
    distinct = np.array([np.unique(r).shape[0] for r in X])
    tie = distinct <= 64
    assert tie.sum() == n
    assert (distinct[tie] == 1).sum() >= 1  # some constant rows
    assert (distinct[~tie] > 380).all()
