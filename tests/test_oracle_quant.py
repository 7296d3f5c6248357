"""Pins for the oracle's quantiser (Eq. 6) and fp16 conversion: invariants,
closed forms and library cross-checks.  CPU only."""
import numpy as np
import pytest


def test_half_to_float_matches_numpy_for_every_half(oracle):
    h = np.arange(65536, dtype=np.uint16)
    ref = h.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in h], np.float32)
    both_nan = np.isnan(ref) & np.isnan(got)
    assert np.array_equal(ref.view(np.uint32)[~both_nan], got.view(np.uint32)[~both_nan])


def test_float_to_half_matches_numpy(oracle):
    rng = np.random.default_rng(7)
    xs = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 6, 20000).astype(np.float32),
        np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 70000.0, -65520.0, 5.9604645e-8, 2.9802322e-8,
                  2.98023224e-8 * 1.0000001, 6.097555e-5, 6.1035156e-5, 1.0009765625, 1.00048828125,
                  1.00146484375, 2047.5, 2048.5, 1e-10, -1e-10], np.float32)])
    # every exact midpoint between neighbouring halves in a few binades (ties must go to even)
    for e in (-14, -3, 0, 7, 15):
        m = np.arange(1024, 2048, dtype=np.float64)
        xs = np.concatenate([xs, ((m + 0.5) * 2.0 ** (e - 10)).astype(np.float32)])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(v) for v in xs], np.uint16)
    assert np.array_equal(ref, got)


@pytest.mark.parametrize("q", [1, 2, 3, 4, 6, 8])
def test_min_maps_to_zero_max_to_top_for_relu_data(oracle, q):
    rng = np.random.default_rng(q)
    x = np.maximum(rng.standard_normal(5000), 0).astype(np.float32)
    sym, qi = oracle.quantize(x, q)
    assert qi.x_min == 0.0 and qi.zero_point == 0.0
    assert sym[np.argmin(x)] == 0
    assert sym[np.argmax(x)] == (1 << q) - 1
    assert sym.max() == (1 << q) - 1 and sym.min() == 0


@pytest.mark.parametrize("q", [2, 4, 8])
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_range_monotone_and_min_to_zero_general(oracle, q, dtype):
    rng = np.random.default_rng(100 + q)
    x = (rng.standard_normal(8000) * 3 + 0.7).astype(dtype)
    sym, qi = oracle.quantize(x, q)
    top = (1 << q) - 1
    assert sym.min() >= 0 and sym.max() <= top
    assert sym[np.argmin(x)] == 0                       # x_min always lands on 0
    assert sym[np.argmax(x)] in (top - 1, top)          # the rounded zero point may shift the grid by half a step
    order = np.argsort(x.astype(np.float64), kind="stable")
    assert np.all(np.diff(sym[order].astype(np.int32)) >= 0)   # monotone
    # against the real-valued definition: |xhat - (x - x_min)/s| <= 1/2 (rounding) + 1/2 (rounded z)
    xd = x.astype(np.float64)
    s = (xd.max() - xd.min()) / top
    ideal = (xd - xd.min()) / s
    assert np.max(np.abs(sym - ideal)) <= 1.0 + 1e-3


def test_closed_forms_exact_arithmetic(oracle):
    # integers 0..255 at Q=8: s = 1, z = 0, xhat = x
    x = np.arange(256, dtype=np.float32)
    sym, qi = oracle.quantize(x, 8)
    assert qi.scale == 1.0 and qi.zero_point == 0.0
    assert np.array_equal(sym, np.arange(256))
    # shifted: -128..127 -> z = 128
    sym, qi = oracle.quantize(x - 128, 8)
    assert qi.scale == 1.0 and qi.zero_point == 128.0
    assert np.array_equal(sym, np.arange(256))
    # scaled by a power of two: s = 0.25
    sym, qi = oracle.quantize((x - 128) * 0.25, 8)
    assert qi.scale == 0.25 and qi.zero_point == 128.0
    assert np.array_equal(sym, np.arange(256))
    # a spot value: X spans [0, 2.55], Q = 8 -> s ~ 0.01, 1.0 -> 100
    xs = np.array([0.0, 1.0, 2.55], np.float32)
    sym, qi = oracle.quantize(xs, 8)
    assert abs(qi.scale - 0.01) < 1e-6 and list(sym) == [0, 100, 255]


def test_rounding_is_nearest_ties_to_even(oracle):
    x = np.array([0.0, 0.5, 1.5, 2.5, 3.5, 0.49999997, 0.50000006, 255.0], np.float32)
    sym, qi = oracle.quantize(x, 8)
    assert qi.scale == 1.0
    assert list(sym) == [0, 0, 2, 2, 4, 0, 1, 255]


def test_one_bit_splits_at_midpoint(oracle):
    x = np.array([2.0, 2.9, 2.999, 3.001, 3.5, 4.0], np.float32)   # midpoint 3.0
    sym, qi = oracle.quantize(x, 1)
    assert qi.scale == 2.0 and qi.zero_point == -1.0
    assert list(sym) == [0, 0, 0, 1, 1, 1]


def test_constant_tensor_and_empty(oracle):
    x = np.full(100, 3.25, np.float32)
    sym, qi = oracle.quantize(x, 8)
    assert qi.scale == 0.0 and np.all(sym == 0)
    assert np.all(oracle.dequantize(sym, qi) == np.float32(3.25))
    sym, qi = oracle.quantize(np.zeros(0, np.float32), 8)
    assert sym.size == 0 and qi.x_min == 0 and qi.x_max == 0


def test_negative_zero_is_canonicalised(oracle):
    x = np.array([-0.0, 1.0], np.float32)
    mn, mx = oracle.minmax(x)
    assert np.float32(mn).view(np.uint32) == 0
    qi = oracle.qinfo_from_minmax(mn, mx, 8)
    assert np.float32(qi.zero_point).view(np.uint32) == 0      # +0.0, not -0.0


@pytest.mark.parametrize("bad", [np.nan, np.inf, -np.inf])
def test_nonfinite_is_rejected(oracle, bad):
    x = np.ones(10, np.float32)
    x[3] = bad
    with pytest.raises(oracle.OracleError) as e:
        oracle.quantize(x, 8)
    assert e.value.code == oracle.ERR_NONFINITE
    xh = np.ones(10, np.float16)
    xh[9] = bad
    with pytest.raises(oracle.OracleError):
        oracle.quantize(xh, 8)


def test_range_overflow_is_rejected(oracle):
    x = np.array([-3e38, 3e38], np.float32)
    with pytest.raises(oracle.OracleError) as e:
        oracle.quantize(x, 8)
    assert e.value.code == oracle.ERR_NONFINITE


@pytest.mark.parametrize("q", [2, 4, 8])
def test_dequantize_error_bound(oracle, q):
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(4000) * 2 - 1).astype(np.float32)
    sym, qi = oracle.quantize(x, q)
    y = oracle.dequantize(sym, qi)
    # |x - s*(xhat - z)| <= s/2 (rounding of xhat) + s/2 (rounding of z), plus float error
    assert np.max(np.abs(y.astype(np.float64) - x)) <= qi.scale * (1.0 + 1e-3)
    yh = oracle.dequantize(sym, qi, oracle.F16)
    assert np.array_equal(yh.view(np.uint16), y.astype(np.float16).view(np.uint16))


def test_dequantize_closed_form(oracle):
    qi = oracle.qinfo_from_minmax(-32.0, 31.75, 8)      # s = 0.25, z = 128
    assert qi.scale == 0.25 and qi.zero_point == 128.0
    y = oracle.dequantize(np.arange(256, dtype=np.uint8), qi)
    assert np.array_equal(y, (np.arange(256) - 128) * np.float32(0.25))
