"""Pins for the oracle's transport codec (Section 7.5: affine min-max quantisation of the states that travel).
Runs without a GPU."""
import numpy as np
import pytest


def rows(seed, n, d, spread=1.0):
    r = np.random.default_rng(seed)
    return (r.standard_normal((n, d)) * spread * np.exp(r.uniform(-3, 3, size=(n, 1)))).astype(np.float32)


@pytest.mark.parametrize("bits", [8, 4])
def test_hand_example(oracle, bits):
    levels = 2 ** bits - 1
    x = np.array([[0.0, 1.0, 2.0, 3.0]], np.float32) * np.float32(levels) / np.float32(3.0)   # 0, L/3, 2L/3, L
    codes, params = oracle.quantize_rows(x, bits)
    assert params[0, 0] == np.float32(1.0) and params[0, 1] == 0.0          # scale = L / L, lo = 0
    want = [0, levels // 3, 2 * levels // 3, levels]
    got = list(codes[0]) if bits == 8 else [codes[0, 0] & 15, codes[0, 0] >> 4, codes[0, 1] & 15, codes[0, 1] >> 4]
    assert got == want
    np.testing.assert_array_equal(oracle.dequantize_rows(codes, params, bits)[0], np.array(want, np.float32))


def test_four_bit_packing_order(oracle):
    x = np.arange(16, dtype=np.float32)[None]                  # levels 15, scale 1: code = channel index
    codes, _ = oracle.quantize_rows(x, 4)
    assert list(codes[0]) == [(2 * k) | ((2 * k + 1) << 4) for k in range(8)]


def test_rounding_is_half_up_on_the_grid(oracle):
    # lo = 0, hi = 255 -> scale 1; 0.5 rounds up to 1, 1.4999 down to 1, 254.5 up to 255
    x = np.zeros((1, 8), np.float32)
    x[0, :5] = [0.0, 0.5, 1.4999, 254.5, 255.0]
    codes, params = oracle.quantize_rows(x, 8)
    assert params[0, 0] == 1.0 and list(codes[0, :5]) == [0, 1, 1, 255, 255]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("d", [64, 128])
def test_round_trip_within_half_a_step(oracle, bits, d):
    X = rows(bits + d, 300, d)
    codes, params = oracle.quantize_rows(X, bits)
    Xh = oracle.dequantize_rows(codes, params, bits)
    scale, lo = params[:, :1].astype(np.float64), params[:, 1:].astype(np.float64)
    hi = X.max(axis=1, keepdims=True).astype(np.float64)
    err = np.abs(Xh.astype(np.float64) - X)
    # half a step, plus the single-precision rounding of the quotient, the sum and the reconstruction
    bound = 0.5 * scale + 4 * np.finfo(np.float32).eps * np.maximum(np.abs(lo), np.abs(hi))
    assert (err <= bound).all()
    levels = 2 ** bits - 1
    q = codes.astype(int) if bits == 8 else np.stack([codes & 15, codes >> 4], -1).reshape(len(X), d).astype(int)
    assert q.min() >= 0 and q.max() <= levels
    assert (q[np.arange(len(X)), X.argmin(1)] == 0).all() and (q[np.arange(len(X)), X.argmax(1)] == levels).all()
    np.testing.assert_array_equal(params[:, 1], X.min(1))                     # lo is the exact minimum
    np.testing.assert_array_equal(Xh[np.arange(len(X)), X.argmin(1)], X.min(1))
    # codes never decrease when the value increases
    order = np.argsort(X, axis=1, kind="stable")
    assert (np.diff(np.take_along_axis(q, order, 1), axis=1) >= 0).all()


def test_constant_row_and_affine_equivariance(oracle):
    x = np.full((2, 64), 3.25, np.float32)
    codes, params = oracle.quantize_rows(x, 8)
    assert not codes.any() and (params[:, 0] == 0).all() and (params[:, 1] == 3.25).all()
    np.testing.assert_array_equal(oracle.dequantize_rows(codes, params, 8), x)
    # exact powers of two and exact shifts commute with the codec: the codes do not change
    X = np.round(rows(3, 50, 64) * 64) / 64
    c0, p0 = oracle.quantize_rows(X.astype(np.float32), 8)
    c1, p1 = oracle.quantize_rows((X * 4).astype(np.float32), 8)
    np.testing.assert_array_equal(c0, c1)
    np.testing.assert_array_equal(p1, p0 * 4)


def test_planted_mistakes_are_caught(oracle):
    """Truncation instead of rounding, or levels = 2^bits, would break the hand examples above; here: a symmetric
    (zero-centred) range instead of min-max would not map the minimum to code 0."""
    X = rows(9, 20, 64) + 5.0
    codes, params = oracle.quantize_rows(X, 8)
    assert (codes.min(axis=1) == 0).all() and (codes.max(axis=1) == 255).all()
    assert (params[:, 1] > 0).any()
