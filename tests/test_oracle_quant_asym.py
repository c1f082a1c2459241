"""Pins of the oracle's asymmetric min-max quantizer and of the zero-point algebra of the layer.

What fixes the expected values here is the Background section of the paper (Eq. 1, its
de-quantization function, the range-based scale that prevents clipping, and the range bound
Eq. "range_ubound"), integer special cases whose codes can be written down by hand, and an
independent floating-point route through the layer (de-quantized activations times de-quantized
weights), not the oracle's own formulas.
"""
import numpy as np
import pytest

from oracle import stamp_oracle as so


def _rows(seed, s=24, d=96, dtype=np.float32):
    rng = np.random.default_rng(seed)
    T = rng.standard_normal((s, d)).astype(dtype)
    T[1] += 3.0          # one-sided positive row
    T[2] -= 5.0          # one-sided negative row
    T[3] *= 1e-3
    T[4] = 0.0           # zero row
    T[5, :] = 2.5        # constant row
    T[6, 7] = 40.0       # outlier
    return T


@pytest.mark.parametrize("bits", [4, 8])
def test_integer_rows_are_reproduced_exactly(bits):
    # a row that holds every integer of [-a, qmax - a] has range qmax, scale 1, offset a, codes x + a
    qm = (1 << bits) - 1
    for a in (0, 3, qm // 2, qm):
        x = np.arange(-a, qm - a + 1, dtype=np.float32)[None, :]
        codes, scale, z = so.quantize_tokens_asym(x, np.array([bits]))
        assert scale[0] == 1.0 and z[0] == a
        assert np.array_equal(codes[0].astype(np.int64), (x[0] + a).astype(np.int64))
        assert np.array_equal(so.dequantize_tokens_asym(codes, scale, z), x)


def test_hand_worked_row():
    # 4 bits, values 0.0 .. 3.0: range 3, scale 0.2, offset 0; 1.1 / 0.2 = 5.5 -> 6 (ties to even do not
    # apply: 5.5 is not representable exactly, fl(1.1 * 5) = 5.5 exactly in fp32 -> rne gives 6)
    x = np.array([[0.0, 3.0, 1.1, 0.29, 0.31, 2.9]], dtype=np.float32)
    codes, scale, z = so.quantize_tokens_asym(x, np.array([4]))
    assert z[0] == 0 and abs(float(scale[0]) - 0.2) < 1e-7
    assert codes[0].tolist() == [0, 15, 6, 1, 2, 14]
    # shifted so that the minimum is negative: offset moves, codes of the same grid points follow
    x2 = np.array([[-1.0, 2.0, 0.0]], dtype=np.float32)
    codes2, scale2, z2 = so.quantize_tokens_asym(x2, np.array([4]))
    assert z2[0] == 5 and codes2[0].tolist() == [0, 15, 5]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_codes_range_offsets_and_zero(bits, dtype):
    T = _rows(1, dtype=dtype)
    b = np.full(T.shape[0], bits)
    codes, scale, z = so.quantize_tokens_asym(T, b, dtype)
    qm = (1 << bits) - 1
    assert codes.dtype == np.uint8 and codes.max() <= qm
    assert np.array_equal(z, np.rint(z))
    # a token whose range straddles 0 has its offset inside the code range; a one-sided token keeps its own
    # range max - min, so its offset leaves the code range: below 0 when all entries are positive, above
    # 2^b - 1 when all are negative
    for i in (0, 3, 6):
        assert T[i].min() < 0 < T[i].max() and 0 <= z[i] <= qm
    assert T[1].min() > 0 and z[1] < 0
    assert T[2].max() < 0 and z[2] > qm
    # zero row: everything zero
    assert scale[4] == 0 and z[4] == 0 and not codes[4].any()
    # the minimum of every row takes code 0, the maximum takes 2^b - 1 (to within the one code that the two
    # separately rounded products can differ by)
    for i in (0, 1, 2, 3, 6):
        assert codes[i][np.argmin(T[i])] == 0
        assert codes[i][np.argmax(T[i])] >= qm - 1
    # every grid point is a multiple of the scale: code z de-quantizes to exactly 0
    D = so.dequantize_tokens_asym(np.zeros((T.shape[0], 1), dtype=np.uint8), scale, np.zeros_like(z), dtype)
    assert not D.any()


@pytest.mark.parametrize("bits", [4, 8])
def test_strictly_positive_row_takes_the_printed_range(bits):
    """Background, range-setting sentence: range = max - min and the offset comes from the minimum, also for
    a token that does not contain 0.  (A range widened to contain 0 would give scale = max / (2^b - 1) and
    code(min) > 0 here.)"""
    qm = (1 << bits) - 1
    rng = np.random.default_rng(11)
    x = (10.0 + rng.random((3, 200))).astype(np.float64)      # values in [10, 11)
    x[1] = -x[1]                                               # strictly negative row
    x[2] = 7.0 + np.arange(200) / 199.0 * 3.0                  # 7 .. 10, ends attained
    codes, scale, z = so.quantize_tokens_asym(x, np.full(3, bits), np.float64)
    span = x.max(axis=1) - x.min(axis=1)
    assert np.allclose(scale, span / qm, rtol=1e-13)
    assert np.all(scale < np.abs(x).max(axis=1) / qm / 3)      # far below what a range containing 0 gives
    for i in range(3):
        assert codes[i][np.argmin(x[i])] == 0
        assert codes[i][np.argmax(x[i])] >= qm - 1
    err = so.dequantize_tokens_asym(codes, scale, z, np.float64) - x
    assert np.all(np.abs(err) <= scale[:, None] * (0.5 + 1e-9))
    # per-token error bound of Eq. "range_ubound" with the token's own range
    assert np.all((err ** 2).sum(axis=1) <= x.shape[1] / 4.0 * span ** 2 / qm ** 2 * (1 + 1e-9))
    # hand-worked: 4 bits, values 3 .. 6 in steps of 0.2: range 3, scale 0.2, x / scale = 15 .. 30, offset -15
    xs = (3.0 + 0.2 * np.arange(16))[None, :]
    c, s_, z_ = so.quantize_tokens_asym(xs, np.array([4]), np.float64)
    assert abs(s_[0] - 0.2) < 1e-15 and z_[0] == -15 and c[0].tolist() == list(range(16))


@pytest.mark.parametrize("bits", [4, 8])
def test_constant_rows(bits):
    """max = min: the printed scale would divide by zero; the reading taken is range = |value|, which still
    reproduces the token to within rounding; a zero token gets scale 0."""
    qm = (1 << bits) - 1
    x = np.stack([np.full(32, 2.5), np.full(32, -0.75), np.zeros(32)]).astype(np.float32)
    codes, scale, z = so.quantize_tokens_asym(x, np.full(3, bits))
    assert np.allclose(scale[:2], np.array([2.5, 0.75]) / qm, rtol=1e-6) and scale[2] == 0
    assert z.tolist() == [-qm, qm, 0] and not codes.any()
    d = so.dequantize_tokens_asym(codes, scale, z)
    assert np.allclose(d, x, rtol=1e-6, atol=0)


@pytest.mark.parametrize("bits", [4, 8])
def test_error_at_most_half_a_step_and_range_bound(bits):
    # no clipping (range-based scale) -> rounding error only: |x_hat - x| <= scale / 2, hence the paper's
    # bound ||x_hat - x||^2 <= d / 4 * range^2 / (2^b - 1)^2 with range = max - min
    T = _rows(2, s=64, d=256, dtype=np.float64)
    b = np.full(T.shape[0], bits)
    codes, scale, z = so.quantize_tokens_asym(T, b, np.float64)
    err = so.dequantize_tokens_asym(codes, scale, z, np.float64) - T
    assert np.all(np.abs(err) <= scale[:, None] * (0.5 + 1e-9))
    qm = (1 << bits) - 1
    rng = T.max(axis=1) - T.min(axis=1)
    flat = rng == 0
    rng[flat] = np.abs(T.max(axis=1))[flat]
    assert np.allclose(scale, rng / qm, rtol=1e-12)
    assert np.all((err ** 2).sum(axis=1) <= T.shape[1] / 4.0 * (rng / qm) ** 2 * (1 + 1e-9))


def test_fp32_and_fp64_agree_except_at_rounding_boundaries():
    T = _rows(3, s=32, d=512)
    b = np.where(np.arange(32) < 4, 8, 4)
    c32, s32, z32 = so.quantize_tokens_asym(T, b, np.float32)
    c64, s64, z64 = so.quantize_tokens_asym(T.astype(np.float64), b, np.float64)
    assert np.allclose(s32, s64, rtol=1e-6)
    assert np.array_equal(z32, z64)
    diff = c32.astype(np.int32) - c64.astype(np.int32)
    assert np.max(np.abs(diff)) <= 1 and np.count_nonzero(diff) < 0.002 * diff.size


def test_asymmetric_beats_symmetric_on_skewed_tokens():
    # one-sided data wastes half of a symmetric grid; the min-max grid does not
    rng = np.random.default_rng(4)
    T = np.abs(rng.standard_normal((16, 512))).astype(np.float32) + 0.5
    b = np.full(16, 4)
    ca, sa, za = so.quantize_tokens_asym(T, b)
    cs, ss = so.quantize_tokens(T, b)
    ea = so.sqnr_db(T, so.dequantize_tokens_asym(ca, sa, za))
    es = so.sqnr_db(T, so.dequantize_tokens(cs, ss))
    assert ea > es + 5.0     # about 6 dB: one extra bit


@pytest.mark.parametrize("xform,levels,gh,gw,s", [("haar1d", 6, 0, 0, 64), ("haar2d", 3, 8, 8, 64)])
def test_layer_with_offsets_equals_dense_dequantized_route(xform, levels, gh, gw, s):
    # independent route: de-quantize activations and weights to floating point, multiply, inverse-transform
    rng = np.random.default_rng(5)
    d, N, k = 48, 40, 4
    X = (rng.standard_normal((2, s, d)) + 0.7).astype(np.float32)
    W = (rng.standard_normal((d, N)) * 0.05).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    out = so.stamp_linear_forward(X, W, xform, levels, k, grid_h=gh, grid_w=gw, bias=bias, act_quant="asym")
    assert out["codes"].dtype == np.uint8 and "zeros" in out
    Wq = out["qw"].astype(np.float64) * out["sw"].astype(np.float64)[None, :]
    for b in range(2):
        Tq = so.dequantize_tokens_asym(out["codes"][b], out["scales"][b], out["zeros"][b], np.float64)
        Y = so.sequence_inverse(Tq @ Wq, xform, levels, gh, gw, np.float64) + bias[None, :]
        assert np.max(np.abs(out["Y"][b] - Y)) <= 2e-5 * np.max(np.abs(Y))
    # and the 8-bit tokens use the 8-bit grid
    assert out["codes"][:, :k].max() > 15 and out["codes"][:, k:].max() <= 15


def test_k_equals_s_limit_is_eight_bit_everywhere():
    rng = np.random.default_rng(6)
    X = rng.standard_normal((1, 32, 64)).astype(np.float32)
    W = (rng.standard_normal((64, 24)) * 0.05).astype(np.float32)
    o8 = so.stamp_linear_forward(X, W, "haar1d", 5, 32, act_quant="asym")
    o4 = so.stamp_linear_forward(X, W, "haar1d", 5, 0, act_quant="asym")
    ref = X[0].astype(np.float64) @ (o8["qw"].astype(np.float64) * o8["sw"].astype(np.float64)[None, :])
    assert so.sqnr_db(ref, o8["Y"][0]) > so.sqnr_db(ref, o4["Y"][0]) + 20.0   # 4 more bits ~ 24 dB
