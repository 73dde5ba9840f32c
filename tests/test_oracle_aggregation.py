"""Pins for the oracle's forward SpGEMM, backward SSpMM and dense SpMM
(Sec. 3.2, Eq. 2-3, Alg. 1-2): dense brute force, library SpMM, closed forms,
the adjoint identity on non-symmetric matrices, and a hand-worked golden."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import synth
from helpers import csr_from_coo, dense_from_csr, read_golden, scatter_cbsr


def _small_graph(N, M, directed, seed, weights):
    return synth.make_graph(N, M, 0, directed=directed, self_loops=(seed % 2 == 0), seed=seed, weights=weights)


def _brute_forward(g, sp_data, sp_index, dim):
    A = dense_from_csr(g.rowptr, g.col, g.val, g.N)
    X = scatter_cbsr(sp_data, sp_index, dim)
    return A @ X, np.abs(A) @ np.abs(X)


def _brute_backward(g, dY, sp_index):
    A = dense_from_csr(g.rowptr, g.col, g.val, g.N)
    G = A.T @ dY.astype(np.float64)
    Gabs = np.abs(A).T @ np.abs(dY.astype(np.float64))
    ix = sp_index.astype(np.int64)
    return np.take_along_axis(G, ix, axis=1), np.take_along_axis(Gabs, ix, axis=1)


def test_golden_hand_worked_example():
    g = read_golden("fig5_fig6_shape_example.txt")
    N, dim, k = (int(r[1]) for r in g["dims"])
    rowptr, col, val = csr_from_coo(N, [(int(a), int(b), float(c)) for a, b, c in g["A_coo"]])
    sp_index = np.array(g["sp_index"], dtype=np.int32)
    sp_data = np.array(g["sp_data"], dtype=np.float32)
    Y, _ = oracle.spgemm_fwd(rowptr, col, val, sp_data, sp_index, dim)
    assert np.array_equal(Y, np.array(g["Y"], dtype=np.float64))
    dY = np.array(g["dY"], dtype=np.float32)
    D, _ = oracle.sspmm_bwd(rowptr, col, val, dY, sp_index)
    assert np.array_equal(D, np.array(g["dXs"], dtype=np.float64))


@pytest.mark.parametrize("N,M,directed,dim,k,seed", [
    (8, 10, True, 6, 3, 1), (33, 150, True, 16, 5, 2), (64, 400, False, 64, 8, 3), (50, 300, True, 24, 24, 4),
    (40, 200, True, 20, 1, 5),
])
def test_forward_and_backward_match_dense_brute_force(N, M, directed, dim, k, seed):
    g = _small_graph(N, M, directed, seed, "normal")  # signed weights, A^T != A when directed
    H = synth.normal_matrix(N, dim, seed + 100)
    dY = synth.normal_matrix(N, dim, seed + 200)
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    Y, Yabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, sp_data, sp_index, dim)
    Yb, Yabsb = _brute_forward(g, sp_data, sp_index, dim)
    np.testing.assert_allclose(Y, Yb, rtol=0, atol=1e-12)
    np.testing.assert_allclose(Yabs, Yabsb, rtol=0, atol=1e-12)
    D, Dabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, sp_index)
    Db, Dabsb = _brute_backward(g, dY, sp_index)
    np.testing.assert_allclose(D, Db, rtol=0, atol=1e-12)
    np.testing.assert_allclose(Dabs, Dabsb, rtol=0, atol=1e-12)
    if directed:
        # the transpose matters on this input: using A instead of A^T would be caught
        A = dense_from_csr(g.rowptr, g.col, g.val, N)
        wrong = np.take_along_axis(A @ dY.astype(np.float64), sp_index.astype(np.int64), axis=1)
        assert np.abs(wrong - D).max() > 1e-3


def test_k_equals_dim_reduces_to_library_spmm():
    g = synth.make_graph(500, 4000, 9, (0.5, 0.2, 0.2), directed=True, seed=7, weights="normal")
    dim = 48
    H = synth.normal_matrix(g.N, dim, 1)
    dY = synth.normal_matrix(g.N, dim, 2)
    A = sp.csr_matrix((g.val.astype(np.float64), g.col, g.rowptr), shape=(g.N, g.N))
    sp_data, sp_index = oracle.topk_cbsr(H, dim)
    Y, _ = oracle.spgemm_fwd(g.rowptr, g.col, g.val, sp_data, sp_index, dim)
    np.testing.assert_allclose(Y, A @ H.astype(np.float64), rtol=0, atol=1e-11)
    Yd, Ydabs = oracle.spmm(g.rowptr, g.col, g.val, H)
    np.testing.assert_allclose(Yd, A @ H.astype(np.float64), rtol=0, atol=1e-11)
    np.testing.assert_allclose(Ydabs, abs(A) @ np.abs(H.astype(np.float64)), rtol=0, atol=1e-11)
    D, _ = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, sp_index)
    np.testing.assert_allclose(D, A.T @ dY.astype(np.float64), rtol=0, atol=1e-11)


def test_identity_adjacency():
    N, dim, k = 30, 32, 7
    rowptr = np.arange(N + 1, dtype=np.int32)
    col = np.arange(N, dtype=np.int32)
    val = np.ones(N, dtype=np.float32)
    H = synth.normal_matrix(N, dim, 3)
    dY = synth.normal_matrix(N, dim, 4)
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    Y, _ = oracle.spgemm_fwd(rowptr, col, val, sp_data, sp_index, dim)
    assert np.array_equal(Y, scatter_cbsr(sp_data, sp_index, dim))
    assert ((Y != 0).sum(axis=1) == k).all()  # exactly k survivors per row
    D, _ = oracle.sspmm_bwd(rowptr, col, val, dY, sp_index)
    assert np.array_equal(D, np.take_along_axis(dY.astype(np.float64), sp_index.astype(np.int64), axis=1))


def test_adjoint_identity_on_nonsymmetric_matrix():
    # <A X, dY> = <X, A^T dY> with X supported on the CBSR pattern
    g = synth.make_graph(2000, 30000, 11, (0.55, 0.2, 0.15), directed=True, seed=9, weights="normal")
    dim, k = 64, 12
    H = synth.normal_matrix(g.N, dim, 5)
    dY = synth.normal_matrix(g.N, dim, 6)
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    Y, _ = oracle.spgemm_fwd(g.rowptr, g.col, g.val, sp_data, sp_index, dim)
    D, _ = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, sp_index)
    lhs = float((Y * dY.astype(np.float64)).sum())
    rhs = float((sp_data.astype(np.float64) * D).sum())
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))
    # and the same identity fails if the matrix is not transposed
    A = sp.csr_matrix((g.val.astype(np.float64), g.col, g.rowptr), shape=(g.N, g.N))
    wrongD = np.take_along_axis(np.asarray(A @ dY.astype(np.float64)), sp_index.astype(np.int64), axis=1)
    assert abs(lhs - float((sp_data.astype(np.float64) * wrongD).sum())) > 1e-3 * abs(lhs)


def test_linearity_and_row_permutation_invariance():
    g = synth.make_graph(300, 2500, 0, directed=True, seed=13, weights="normal")
    dim, k = 32, 6
    H = synth.normal_matrix(g.N, dim, 7)
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    Y1, _ = oracle.spgemm_fwd(g.rowptr, g.col, g.val, sp_data, sp_index, dim)
    Y2, _ = oracle.spgemm_fwd(g.rowptr, g.col, (2 * g.val).astype(np.float32), sp_data, sp_index, dim)
    assert np.array_equal(Y2, 2 * Y1)  # scaling by 2 is exact
    Y3, _ = oracle.spgemm_fwd(g.rowptr, g.col, g.val, (4 * sp_data).astype(np.float32), sp_index, dim)
    assert np.array_equal(Y3, 4 * Y1)
    perm = np.random.default_rng(1).permutation(k)
    Y4, _ = oracle.spgemm_fwd(g.rowptr, g.col, g.val, sp_data[:, perm].copy(), sp_index[:, perm].copy(), dim)
    np.testing.assert_allclose(Y4, Y1, rtol=0, atol=1e-13)


def test_empty_rows_columns_and_duplicates():
    # node 1 has no out-entries, node 3 has no in-entries, entry (0,2) is stored twice
    N, dim, k = 4, 5, 2
    rowptr, col, val = csr_from_coo(N, [(0, 2, 1.5), (0, 2, 0.5), (0, 0, 1.0), (2, 1, -2.0), (3, 0, 4.0)])
    H = np.array([[1, 2, 3, 4, 5], [5, 4, 3, 2, 1], [0, 9, 0, 8, 0], [1, 1, 1, 1, 1]], dtype=np.float32)
    dY = np.arange(20, dtype=np.float32).reshape(4, 5)
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    Y, Yabs = oracle.spgemm_fwd(rowptr, col, val, sp_data, sp_index, dim)
    assert np.array_equal(Y[1], np.zeros(dim))
    # row 0 = 1.0*X0 + (1.5+0.5)*X2 ; X0 = [0,0,0,4,5], X2 = [0,9,0,8,0]
    assert np.array_equal(Y[0], np.array([0, 18, 0, 20, 5], dtype=np.float64))
    D, _ = oracle.sspmm_bwd(rowptr, col, val, dY, sp_index)
    assert np.array_equal(D[3], np.zeros(k))
    # node 2 (idx [1,3]) receives (1.5+0.5) * dY[0,[1,3]] = 2*[1,3]
    assert np.array_equal(D[2], np.array([2.0, 6.0]))


def test_row_and_node_sampling_agree_with_full_result():
    g = synth.graph("tiny_directed")
    cfg = synth.CONFIGS["tiny_directed"]
    H, dY = synth.features("tiny_directed", "H"), synth.features("tiny_directed", "dY")
    sp_data, sp_index = oracle.topk_cbsr(H, 8)
    Y, Yabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, sp_data, sp_index, cfg.dim)
    rows = np.array([5, 0, 1023, 77], dtype=np.int64)
    Ys, Yabss = oracle.spgemm_fwd(g.rowptr, g.col, g.val, sp_data, sp_index, cfg.dim, rows=rows)
    assert np.array_equal(Ys, Y[rows]) and np.array_equal(Yabss, Yabs[rows])
    D, Dabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, sp_index)
    Ds, Dabss = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, sp_index, nodes=rows)
    np.testing.assert_allclose(Ds, D[rows], rtol=0, atol=1e-13)
    np.testing.assert_allclose(Dabss, Dabs[rows], rtol=0, atol=1e-13)
    Hs, _ = oracle.spmm(g.rowptr, g.col, g.val, H, rows=rows)
    Hf, _ = oracle.spmm(g.rowptr, g.col, g.val, H)
    assert np.array_equal(Hs, Hf[rows])


def test_cbsr_scatter_and_the_whole_backward_chain_against_torch_autograd():
    # MaxK's backward keeps the forward pattern (Sec. 3.1 definition (ii)): with X = H * mask,
    # Y = A X and L = <Y, dY>, plain PyTorch autograd on dense CPU tensors gives dL/dH = (A^T dY) * mask.
    import torch
    g = synth.make_graph(60, 500, 0, directed=True, seed=21, weights="normal")
    dim, k = 24, 7
    H = synth.normal_matrix(g.N, dim, 8)
    dY = synth.normal_matrix(g.N, dim, 9)
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    D, _ = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, sp_index)
    dH = oracle.cbsr_scatter(D.astype(np.float32), sp_index, dim)
    # placement alone, against NumPy
    want = np.zeros((g.N, dim), dtype=np.float32)
    np.put_along_axis(want, sp_index.astype(np.int64), D.astype(np.float32), axis=1)
    assert np.array_equal(dH, want)
    assert ((dH != 0).sum(axis=1) <= k).all()
    # the chain, against autograd
    order = np.argsort(-H, axis=1, kind="stable")[:, :k]
    mask = np.zeros((g.N, dim), dtype=np.float64)
    np.put_along_axis(mask, order, 1.0, axis=1)
    A = torch.from_numpy(dense_from_csr(g.rowptr, g.col, g.val, g.N))
    Ht = torch.from_numpy(H.astype(np.float64)).requires_grad_(True)
    Y = A @ (Ht * torch.from_numpy(mask))
    (Y * torch.from_numpy(dY.astype(np.float64))).sum().backward()
    np.testing.assert_allclose(dH, Ht.grad.numpy(), rtol=0, atol=2e-6)
