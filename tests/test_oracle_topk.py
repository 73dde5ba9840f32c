"""Pins for the oracle's MaxK / CBSR step (Sec. 3.1 definition, Eq. 1; Sec. 3.2 CBSR)."""
import numpy as np
import pytest

import oracle
import synth
from helpers import check_topk_properties, read_golden


def _argsort_reference(H, k):
    # library routine with exactly the tie rule: stable sort of -H = value desc, column asc
    order = np.argsort(-H, axis=1, kind="stable")[:, :k]
    idx = np.sort(order, axis=1)
    return np.take_along_axis(H, idx, axis=1), idx.astype(np.int32)


def test_golden_hand_worked_example():
    g = read_golden("fig5_fig6_shape_example.txt")
    H = np.array(g["H"], dtype=np.float32)
    k = int(g["dims"][2][1])
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    assert np.array_equal(sp_index, np.array(g["sp_index"], dtype=np.int32))
    want = np.array(g["sp_data"], dtype=np.float32)
    assert np.array_equal(sp_data.view(np.uint32), want.view(np.uint32))  # includes the sign of -0.0
    assert np.signbit(sp_data[4, 0]) and not np.signbit(sp_data[4, 1])


@pytest.mark.parametrize("dim,k", [(6, 3), (64, 8), (64, 1), (64, 64), (256, 32), (256, 200), (384, 96), (37, 5)])
def test_matches_stable_argsort_and_properties(dim, k):
    H = synth.normal_matrix(300, dim, seed=11 + dim + k)
    sp_data, sp_index = oracle.topk_cbsr(H, k)
    check_topk_properties(H, k, sp_data, sp_index)
    d2, i2 = _argsort_reference(H, k)
    assert np.array_equal(sp_index, i2)
    assert np.array_equal(sp_data.view(np.uint32), d2.view(np.uint32))


def test_tie_rows_lower_column_wins():
    H = synth.normal_matrix(2000, 384, seed=5)
    n = synth.add_tie_rows(H, seed=5, percent=50, pool=16, const_every=8)
    assert n > 500
    for k in (1, 32, 96, 192, 383):
        sp_data, sp_index = oracle.topk_cbsr(H, k)
        check_topk_properties(H, k, sp_data, sp_index)
        d2, i2 = _argsort_reference(H, k)
        assert np.array_equal(sp_index, i2)


def test_special_cases():
    rng = np.random.default_rng(0)
    H = rng.standard_normal((50, 40)).astype(np.float32)
    # k = 1 is the first-occurrence argmax
    d, i = oracle.topk_cbsr(H, 1)
    assert np.array_equal(i[:, 0], np.argmax(H, axis=1))
    # k = dim is the identity
    d, i = oracle.topk_cbsr(H, 40)
    assert np.array_equal(i, np.tile(np.arange(40, dtype=np.int32), (50, 1)))
    assert np.array_equal(d.view(np.uint32), H.view(np.uint32))
    # constant rows keep columns 0..k-1
    C = np.full((7, 40), 3.25, dtype=np.float32)
    d, i = oracle.topk_cbsr(C, 9)
    assert np.array_equal(i, np.tile(np.arange(9, dtype=np.int32), (7, 1)))
    # selection is by signed value, not magnitude: large negatives lose
    S = np.array([[-100.0, 1.0, -50.0, 2.0, 0.5, -0.25]], dtype=np.float32)
    d, i = oracle.topk_cbsr(S, 3)
    assert i.tolist() == [[1, 3, 4]]
    # ... and negatives survive when they rank in the top k
    d, i = oracle.topk_cbsr(S, 5)
    assert i.tolist() == [[1, 2, 3, 4, 5]]


def test_signed_zero_and_infinities():
    H = np.array([[-0.0, 0.0, -0.0, 0.0, -1.0, 1.0],
                  [np.inf, -np.inf, 0.0, np.inf, 5.0, -0.0]], dtype=np.float32)
    d, i = oracle.topk_cbsr(H, 3)
    # row 0: 1.0 first, then zeros tie regardless of sign -> lowest columns 0, 1
    assert i[0].tolist() == [0, 1, 5]
    assert np.signbit(d[0, 0]) and not np.signbit(d[0, 1])
    # row 1: both +inf, then 5.0
    assert i[1].tolist() == [0, 3, 4]
    check_topk_properties(H, 3, d, i)


def test_nan_is_rejected():
    H = np.zeros((2, 8), dtype=np.float32)
    H[1, 3] = np.nan
    with pytest.raises(ValueError):
        oracle.topk_cbsr(H, 2)


def test_property_checker_catches_planted_mistakes():
    # the checker itself must reject wrong answers (mistakes planted on the CPU side)
    H = np.array([[1.0, 3.0, 3.0, 2.0, 3.0, 0.0]], dtype=np.float32)
    good_d, good_i = oracle.topk_cbsr(H, 2)
    assert good_i.tolist() == [[1, 2]]
    check_topk_properties(H, 2, good_d, good_i)
    for bad in ([[1, 4]], [[2, 4]], [[2, 1]], [[0, 1]]):
        bi = np.array(bad, dtype=np.int32)
        bd = np.take_along_axis(H, bi.astype(np.int64), axis=1)
        with pytest.raises(AssertionError):
            check_topk_properties(H, 2, bd, bi)
