"""Pins for the oracle's quantizer, integer GEMM and the whole STaMP linear layer."""
import os

import numpy as np
import pytest

from gen import get_workload, make_inputs
from oracle import stamp_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_effective_bits_match_the_paper():
    for line in open(os.path.join(GOLDEN, "effective_bits.txt")):
        if line.startswith("#") or not line.strip():
            continue
        s, k, bh, bl, eff = line.split()
        assert so.effective_bits(int(s), int(k), int(bh), int(bl)) == float(eff)
        b = so.token_bits(int(s), int(k), int(bh), int(bl))
        assert b.mean() == float(eff) and (b[:int(k)] == int(bh)).all() and (b[int(k):] == int(bl)).all()


def test_qmax():
    assert so.qmax_of(8) == 127 and so.qmax_of(4) == 7


def _rne_scalar(v):
    """round half to even on a python float, independent of numpy."""
    f = np.floor(v)
    r = v - f
    if r > 0.5:
        return f + 1
    if r < 0.5:
        return f
    return f if (int(f) % 2 == 0) else f + 1


def test_quantizer_against_scalar_loops():
    """Brute force on a small input, written as python loops from Eq. 1 (symmetric form)."""
    rng = np.random.default_rng(0)
    T = rng.standard_normal((6, 11)).astype(np.float32) * np.float32(3.0)
    T[2] = 0.0                                      # a zero row
    T[3, 4] = 0.5 * np.max(np.abs(T[3]))            # something exactly representable
    bits = np.array([8, 8, 4, 4, 4, 8])
    codes, scale = so.quantize_tokens(T, bits, np.float32)
    assert codes.dtype == np.int8 and scale.dtype == np.float32
    for i in range(6):
        qm = 2 ** (int(bits[i]) - 1) - 1
        a = np.float32(max(abs(float(v)) for v in T[i]))
        if a == 0:
            assert scale[i] == 0 and not codes[i].any()
            continue
        assert scale[i] == np.float32(a / np.float32(qm))
        inv = np.float32(np.float32(qm) / a)
        for j in range(11):
            prod = np.float32(T[i, j] * inv)                 # one fp32 multiply
            q = _rne_scalar(float(prod))
            q = max(-qm, min(qm, q))
            assert codes[i, j] == q, (i, j)
        assert np.max(np.abs(codes[i])) == qm                 # the absmax element attains qmax


def test_round_half_to_even_is_used():
    # a row whose absmax is exactly qmax => inv = 1 and codes = rne(values)
    T = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]], dtype=np.float32)
    codes, scale = so.quantize_tokens(T, np.array([4]), np.float32)
    assert scale[0] == 1.0
    assert codes[0].tolist() == [7, 0, 2, 2, 0, -2, -2, 4]


def test_no_clipping_error_bound_and_range():
    """Range-based scale => no clipping, each element errs by at most scale/2 (the step used in the
    proof of Eq. range_ubound); hence per token ||x - Q(x)||^2 <= d/4 scale^2."""
    rng = np.random.default_rng(1)
    T = (rng.standard_normal((64, 257)) * rng.uniform(0.01, 100, size=(64, 1))).astype(np.float32)
    bits = so.token_bits(64, 8)
    codes, scale = so.quantize_tokens(T, bits, np.float32)
    deq = so.dequantize_tokens(codes, scale, np.float64)
    err = np.abs(T.astype(np.float64) - deq)
    assert (err <= 0.5 * scale[:, None].astype(np.float64) * (1 + 2.0 ** -20)).all()
    qm = np.where(bits == 8, 127, 7)[:, None]
    assert (np.abs(codes) <= qm).all() and (np.abs(codes).max(axis=1) == qm[:, 0]).all()
    assert (np.sum(err ** 2, axis=1) <= 257 / 4 * scale.astype(np.float64) ** 2 * (1 + 1e-6)).all()
    # symmetric analogue of Theorem 1 (absmax <= norm): total error <= d/4 sum_i ||T_i||^2 / qmax_i^2
    bound = 257 / 4 * np.sum(np.sum(T.astype(np.float64) ** 2, axis=1) / qm[:, 0] ** 2)
    assert np.sum(err ** 2) <= bound


def test_identity_transform_k0_is_textbook_per_token_rtn():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((1, 16, 40)).astype(np.float32)
    out = so.quantize_activation(X, "identity", 0, k_hi=0)
    a = np.abs(X[0]).max(axis=1, keepdims=True)
    ref = np.clip(np.rint(X[0] * (np.float32(7) / a)), -7, 7).astype(np.int8)
    assert np.array_equal(out["codes"][0], ref)
    assert np.array_equal(out["scales"][0], (a / np.float32(7))[:, 0])


def test_all_high_limit():
    # k = s: every token at 8 bits, i.e. plain per-token int8 quantization of L X
    rng = np.random.default_rng(3)
    X = rng.standard_normal((2, 32, 24)).astype(np.float32)
    out = so.quantize_activation(X, "haar1d", 5, k_hi=32)
    assert (out["bits"] == 8).all()
    for b in range(2):
        T = so.haar1d_forward(X[b], 5, np.float32)
        c, s = so.quantize_tokens(T, np.full(32, 8), np.float32)
        assert np.array_equal(out["codes"][b], c) and np.array_equal(out["scales"][b], s)
        assert np.abs(out["codes"][b]).max() == 127


def test_weight_quantization_is_per_output_channel():
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((48, 10)) * 0.02).astype(np.float32)
    W[:, 3] = 0
    qw, sw = so.quantize_weight(W, 4, np.float32)
    assert qw.shape == (48, 10) and sw.shape == (10,)
    for n in range(10):
        a = np.float32(np.abs(W[:, n]).max())
        if a == 0:
            assert sw[n] == 0 and not qw[:, n].any()
            continue
        assert sw[n] == np.float32(a / np.float32(7))
        ref = np.clip(np.rint(W[:, n] * np.float32(np.float32(7) / a)), -7, 7)
        assert np.array_equal(qw[:, n], ref.astype(np.int8))
        assert np.abs(qw[:, n]).max() == 7


def test_int_gemm_against_triple_loop():
    rng = np.random.default_rng(5)
    q = rng.integers(-127, 128, size=(7, 13)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(13, 5)).astype(np.int8)
    acc = so.int_gemm(q, qw)
    assert acc.dtype == np.int32
    for m in range(7):
        for n in range(5):
            tot = 0
            for k in range(13):
                tot += int(q[m, k]) * int(qw[k, n])
            assert acc[m, n] == tot
    # extreme magnitudes at the largest benchmark depth stay exact and inside 24 bits
    q = np.full((2, 8192), 127, dtype=np.int8); q[1] = -127
    qw = np.full((8192, 3), 7, dtype=np.int8); qw[:, 1] = -7
    acc = so.int_gemm(q, qw)
    assert acc[0, 0] == 8192 * 127 * 7 and acc[1, 0] == -8192 * 127 * 7 and acc[0, 1] == -8192 * 127 * 7
    assert abs(int(acc[0, 0])) < 2 ** 24


def test_eight_bit_rows_fp32_conversion_bound():
    """The de-quantization converts the integer sum to fp32: exact below 2^24.  With 8-bit codes of magnitude up to
    128 (the stored form of the asymmetric code 0) against weight codes of magnitude 7 the worst case reaches
    128 * 7 * d_in, so the conversion is exact for every input up to d_in = 18720 (the bound include/stamp.h states);
    the oracle refuses a sum beyond it instead of rounding silently."""
    d_ok = 18720
    q = np.full((1, d_ok), -128, dtype=np.int16)
    qw = np.full((d_ok, 2), 7, dtype=np.int8); qw[:, 1] = -7
    acc = so.int_gemm(q, qw)
    assert acc[0, 0] == -128 * 7 * d_ok and acc[0, 1] == 128 * 7 * d_ok
    assert abs(int(acc[0, 0])) < 2 ** 24 and float(np.float32(acc[0, 0])) == float(acc[0, 0])
    d_bad = 18752   # the next multiple of 32 whose worst case passes 2^24
    assert 128 * 7 * d_bad > 2 ** 24
    with pytest.raises(AssertionError, match="exact fp32 integer range"):
        so.int_gemm(np.full((1, d_bad), -128, dtype=np.int16), np.full((d_bad, 1), 7, dtype=np.int8))
    # symmetric codes stop at 127: exact up to d_in = 18848
    assert 127 * 7 * 18848 < 2 ** 24 < 127 * 7 * 18880
    # an odd sum just above 2^24 is what the conversion would round
    assert float(np.float32(2 ** 24 + 1)) != float(2 ** 24 + 1)


def test_round_to_bf16():
    y = np.array([1.0, 1.00390625, 1.01171875, -3.140625, 1.0 + 2.0 ** -9, 0.0], dtype=np.float32)
    r = so.round_to_bf16(y)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties -> 1 + 2^-6 (even)
    assert r.tolist() == [1.0, 1.0, 1.015625, -3.140625, 1.0, 0.0]
    import torch
    z = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    assert np.array_equal(so.round_to_bf16(z), torch.from_numpy(z).to(torch.bfloat16).float().numpy())


@pytest.mark.parametrize("xform,kw", [("haar1d", dict(levels=6)), ("haar2d", dict(levels=3, grid_h=8, grid_w=8)),
                                      ("identity", dict(levels=0))])
def test_commutation_identity_without_quantization(xform, kw):
    """L^-1((L X) W) = X W (section "Method", the identity that lets the inverse follow the GEMM)."""
    rng = np.random.default_rng(6)
    X = rng.standard_normal((64, 20))
    W = rng.standard_normal((20, 9))
    T = so.sequence_forward(X, xform, dtype=np.float64, **kw)
    Y = so.sequence_inverse(T @ W, xform, dtype=np.float64, **kw)
    assert np.allclose(Y, X @ W, atol=1e-12)
    # option (ii): transformed bias l = L 1 added before the inverse gives the same result
    beta = rng.standard_normal(9)
    ell = so.sequence_forward(np.ones((64, 1)), xform, dtype=np.float64, **kw)[:, 0]
    Y2 = so.sequence_inverse(T @ W + np.outer(ell, beta), xform, dtype=np.float64, **kw)
    assert np.allclose(Y2, X @ W + beta, atol=1e-12)


def test_linear_forward_step_by_step_small():
    """The whole layer on a tiny case against a direct evaluation with dense L (fp64 definition):
    Y = L^T (diag(scale) * (codes @ qw) * diag(sw)) + bias, with codes from the fp32 path."""
    rng = np.random.default_rng(8)
    s, d, N, k = 16, 12, 7, 2
    X = rng.standard_normal((1, s, d)).astype(np.float32)
    W = (rng.standard_normal((d, N)) * 0.02).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    out = so.stamp_linear_forward(X, W, "haar1d", 4, k, bias=bias)
    L = so.haar1d_matrix(s, 4)
    T = L @ X[0].astype(np.float64)
    assert np.max(np.abs(out["T"][0] - T)) < 1e-5
    # codes can differ from the fp64-derived ones only on near-ties; here demand <= 1 code step
    for i in range(s):
        qm = 127 if i < k else 7
        a = np.abs(T[i]).max()
        ref = np.clip(np.rint(T[i] * (qm / a)), -qm, qm)
        assert np.max(np.abs(out["codes"][0, i] - ref)) <= 1
        assert np.isclose(out["scales"][0, i], a / qm, rtol=1e-6)
    acc = out["codes"][0].astype(np.int64) @ out["qw"].astype(np.int64)
    assert np.array_equal(out["acc"][0], acc)
    Yt = acc * out["scales"][0].astype(np.float64)[:, None] * out["sw"].astype(np.float64)[None, :]
    Y = L.T @ Yt + bias
    assert np.max(np.abs(out["Y"][0] - Y)) <= 1e-5 * np.max(np.abs(Y))
    assert np.max(np.abs(out["Yt"][0] - Yt)) <= 1e-6 * np.max(np.abs(Yt))


def test_linear_forward_fp32_vs_fp64_mode_cfg1():
    """fp32 bit-reference mode against the fp64 definition on the small benchmark configuration:
    same scales to fp32 rounding, codes equal except near rounding boundaries, outputs close."""
    w = get_workload("cfg1")
    inp = make_inputs(w)
    o32 = so.stamp_linear_forward(inp["X_f32"], inp["W"], w.xform, w.levels, w.k_hi, dtype=np.float32)
    o64 = so.stamp_linear_forward(inp["X_f32"], inp["W"], w.xform, w.levels, w.k_hi, dtype=np.float64)
    assert np.allclose(o32["scales"], o64["scales"], rtol=1e-5)
    diff = o32["codes"].astype(np.int32) - o64["codes"].astype(np.int32)
    assert np.abs(diff).max() <= 1 and np.count_nonzero(diff) < 1e-3 * diff.size
    assert np.array_equal(o32["qw"], o64["qw"])
    ref = inp["X_f32"][0].astype(np.float64) @ inp["W"].astype(np.float64)
    assert so.sqnr_db(o64["Y"][0], o32["Y"][0]) > 35.0
    # the paper's qualitative claim: the sequence transform raises SQNR over the same mixed
    # precision without it (sanity on AR(1) input; no threshold from the paper)
    oid = so.stamp_linear_forward(inp["X_f32"], inp["W"], "identity", 0, w.k_hi, dtype=np.float32)
    assert so.sqnr_db(ref, o32["Y"][0]) > so.sqnr_db(ref, oid["Y"][0]) + 1.0


def test_sqnr():
    a = np.array([3.0, 4.0])
    assert np.isclose(so.sqnr_db(a, a * 0.9), 20.0)
    assert so.sqnr_db(a, a) == float("inf")
