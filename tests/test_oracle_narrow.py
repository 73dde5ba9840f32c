"""Pins for the oracle's 16-bit CBSR value formats (bf16 / fp16, round to nearest even).

The conversions are pinned to things other than themselves: NumPy's float16 cast and PyTorch's
bfloat16 cast (independent library routines with the same rounding rule), hand-worked halfway
cases, the round trip over every bit pattern, and the error bound of each format.
"""
import numpy as np
import pytest
import torch

import oracle


def _special_values():
    v = [0.0, -0.0, 1.0, -1.0, 0.1, 3.14159274, 65504.0, 65519.996, 65520.0, 70000.0, -70000.0, 2.0 ** -14,
         2.0 ** -14 * (1 - 2.0 ** -11), 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -26, 1e-30, -1e-30,
         3.0e38, -3.0e38, 3.4028235e38, np.inf, -np.inf, 2.0 ** -126, 2.0 ** -140]
    return np.array(v, dtype=np.float32)


def _random_values(seed, n):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n).astype(np.float32)
    b = (rng.standard_normal(n) * np.exp2(rng.integers(-30, 18, n))).astype(np.float32)
    # all fp32 patterns of a few exponents around the fp16 subnormal boundary and the halfway points
    c = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32).view(np.float32)
    c = c[np.isfinite(c)]
    return np.concatenate([a, b, c])


def test_f16_matches_numpy_cast():
    x = np.concatenate([_special_values(), _random_values(1, 200_000)])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = oracle.narrow(x, "f16")
    np.testing.assert_array_equal(got, want)


def test_bf16_matches_torch_cast():
    x = np.concatenate([_special_values(), _random_values(2, 200_000)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.narrow(x, "bf16")
    np.testing.assert_array_equal(got, want)


def test_hand_worked_halfway_cases():
    # bf16 keeps 8 significant bits: the neighbours of 1 are 1 and 1 + 2^-7
    x = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, 1 + 2.0 ** -8 - 2.0 ** -20,
                  -(1 + 2.0 ** -8), 255.5 * 2.0 ** -7 * 2], np.float32)
    got = oracle.widen(oracle.narrow(x, "bf16"), "bf16")
    #   halfway -> even (1.0) | halfway -> even (1 + 2^-6) | just above -> up | just below -> down | sign symmetric
    want = np.array([1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7, 1.0, -1.0, 4.0], np.float32)
    np.testing.assert_array_equal(got, want)
    # fp16 keeps 11 significant bits: neighbours of 1 are 1 and 1 + 2^-10; 2049 and 2051 are halfway at spacing 2
    x = np.array([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 2049.0, 2051.0, 65520.0, 65519.0, 2.0 ** -25, 3 * 2.0 ** -25],
                 np.float32)
    got = oracle.widen(oracle.narrow(x, "f16"), "f16")
    want = np.array([1.0, 1 + 2.0 ** -9, 2048.0, 2052.0, np.inf, 65504.0, 0.0, 2.0 ** -23], np.float32)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("vt", ["bf16", "f16"])
def test_round_trip_over_every_pattern(vt):
    h = np.arange(65536, dtype=np.uint16)
    x = oracle.widen(h, vt)
    keep = ~np.isnan(x)
    assert keep.sum() == 65536 - (2 * 127 if vt == "bf16" else 2 * 1023)  # NaN patterns of the format
    np.testing.assert_array_equal(oracle.narrow(x[keep], vt), h[keep])
    # widening agrees with the libraries' reading of the patterns
    if vt == "f16":
        lib = h.view(np.float16).astype(np.float32)
    else:
        lib = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(x[keep], lib[keep])


@pytest.mark.parametrize("vt,rel,tiny", [("bf16", 2.0 ** -8, 0.0), ("f16", 2.0 ** -11, 2.0 ** -25)])
def test_error_bound_and_monotone(vt, rel, tiny):
    rng = np.random.default_rng(3)
    x = np.sort((rng.standard_normal(100_000) * 8).astype(np.float32))
    y = oracle.widen(oracle.narrow(x, vt), vt)
    err = np.abs(y.astype(np.float64) - x.astype(np.float64))
    assert np.all(err <= rel * np.abs(x.astype(np.float64)) + tiny)  # half a unit in the last kept place
    assert np.all(np.diff(y) >= 0)                                   # rounding preserves order
    assert np.array_equal(np.signbit(y), np.signbit(x))


def test_nan_is_rejected():
    with pytest.raises(ValueError):
        oracle.narrow(np.array([1.0, np.nan], np.float32), "bf16")
    with pytest.raises(ValueError):
        oracle.narrow(np.array([np.nan], np.float32), "f16")
