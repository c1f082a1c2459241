"""Pins for the oracle's sequence transforms: nothing here compares the oracle with itself only.

Each test checks the butterfly implementations against something the paper or the mathematics
fixes: hand-written small matrices (tests/golden/haar_small.txt), the dense matrix built from the
Haar basis functions, orthogonality (Theorem 1 requires an orthogonal L), energy preservation
(the note after Theorem 1), closed forms, and the structure the GPU design relies on.
"""
import os

import numpy as np
import pytest

from oracle import stamp_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_small_matrices():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "haar_small.txt")) if l.strip() and not l.startswith("#")]
    mats, i = {}, 0
    while i < len(rows):
        s = int(rows[i][0])
        mats[s] = np.array([[float(v) for v in r] for r in rows[i + 1:i + 1 + s]])
        i += 1 + s
    return mats


def _apply_rowwise(fn, s, **kw):
    """Matrix of a linear map on R^s obtained by pushing the identity through fn."""
    return fn(np.eye(s), **kw)


@pytest.mark.parametrize("s", [2, 4])
def test_small_matrices_match_textbook(s):
    L_ref = _read_small_matrices()[s]
    J = int(np.log2(s))
    # forward(I) has column j = L e_j, i.e. it is L itself
    L_bfly = so.haar1d_forward(np.eye(s), J, np.float64)
    assert np.allclose(L_bfly, L_ref, atol=1e-15)
    assert np.allclose(so.haar1d_matrix(s, J), L_ref, atol=1e-15)


@pytest.mark.parametrize("s,J", [(8, 3), (16, 4), (16, 2), (64, 6), (256, 8), (256, 3), (32, 0)])
def test_haar1d_butterflies_equal_dense_definition(s, J):
    L = so.haar1d_matrix(s, J)
    assert np.allclose(L @ L.T, np.eye(s), atol=1e-14)            # orthogonal
    rng = np.random.default_rng(s + J)
    x = rng.standard_normal((s, 5))
    t64 = so.haar1d_forward(x, J, np.float64)
    assert np.allclose(t64, L @ x, atol=1e-13)
    assert np.allclose(so.haar1d_inverse(t64, J, np.float64), x, atol=1e-13)
    assert np.allclose(so.haar1d_inverse(L @ x, J, np.float64), L.T @ (L @ x), atol=1e-13)
    # fp32 bit-reference mode stays within fp32 rounding of the definition
    t32 = so.haar1d_forward(x.astype(np.float32), J, np.float32)
    assert t32.dtype == np.float32
    ref = L @ x.astype(np.float32).astype(np.float64)
    assert np.max(np.abs(t32 - ref)) <= 1e-5 * np.max(np.abs(ref))


@pytest.mark.parametrize("s", [8, 64, 1024])
def test_haar1d_closed_forms(s):
    J = int(np.log2(s))
    # constant c -> slot 0 = c sqrt(s), the rest 0
    t = so.haar1d_forward(np.full((s, 1), 3.0), J, np.float64)[:, 0]
    assert np.isclose(t[0], 3.0 * np.sqrt(s)) and np.allclose(t[1:], 0.0)
    # unit impulse at token 0 -> slot 0 = 1/sqrt(s), slot s/2^l = 2^(-l/2), rest 0
    e0 = np.zeros((s, 1)); e0[0] = 1.0
    t = so.haar1d_forward(e0, J, np.float64)[:, 0]
    expect = np.zeros(s); expect[0] = 1 / np.sqrt(s)
    for l in range(1, J + 1):
        expect[s >> l] = 2.0 ** (-l / 2.0)
    assert np.allclose(t, expect, atol=1e-15)
    # impulse at the LAST token: the wavelets are (+ first half, - second half) => negative details
    el = np.zeros((s, 1)); el[-1] = 1.0
    t = so.haar1d_forward(el, J, np.float64)[:, 0]
    expect = np.zeros(s); expect[0] = 1 / np.sqrt(s)
    for l in range(1, J + 1):
        expect[(s >> l) + (s >> l) - 1] = -(2.0 ** (-l / 2.0))
    assert np.allclose(t, expect, atol=1e-15)
    # alternating +1/-1 -> every level-1 detail = sqrt 2, everything else 0
    alt = np.where(np.arange(s) % 2 == 0, 1.0, -1.0)[:, None]
    t = so.haar1d_forward(alt, J, np.float64)[:, 0]
    assert np.allclose(t[:s // 2], 0.0) and np.allclose(t[s // 2:], np.sqrt(2.0))
    # L 1 = sqrt(s) e_0: the transformed bias direction of the commutation identity
    one = so.haar1d_forward(np.ones((s, 1)), J, np.float64)[:, 0]
    assert np.isclose(one[0], np.sqrt(s)) and np.allclose(one[1:], 0)


def test_haar1d_energy_preserved_and_roundtrip_fp32():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((512, 33)).astype(np.float32)
    t = so.haar1d_forward(x, 9, np.float32)
    e_in = np.sum(x.astype(np.float64) ** 2)
    e_out = np.sum(t.astype(np.float64) ** 2)
    assert abs(e_in - e_out) <= 1e-5 * e_in
    back = so.haar1d_inverse(t, 9, np.float32)
    assert np.max(np.abs(back - x)) <= 2e-6 * np.max(np.abs(x))


def test_haar1d_partial_levels_leave_coarse_approximations():
    # J levels on s tokens: the first s/2^J slots are block sums / 2^(J/2)
    s, J = 64, 3
    rng = np.random.default_rng(3)
    x = rng.standard_normal((s, 2))
    t = so.haar1d_forward(x, J, np.float64)
    blocks = x.reshape(s >> J, 1 << J, 2).sum(axis=1) / np.sqrt(1 << J)
    assert np.allclose(t[:s >> J], blocks)


def test_stamp_order_slot_meaning_1d():
    # slot p >= 1 with m = floor(log2 p): the wavelet of level J-m at position p-2^m
    s, J = 32, 5
    L = so.haar1d_matrix(s, J)
    for p in range(1, s):
        m = int(np.floor(np.log2(p)))
        l, i = J - m, p - (1 << m)
        support = np.nonzero(L[p])[0]
        assert support.min() == i << l and support.max() == ((i + 1) << l) - 1
        assert L[p, i << l] > 0 > L[p, ((i + 1) << l) - 1]


@pytest.mark.parametrize("H,W,J", [(2, 2, 1), (4, 4, 2), (8, 8, 3), (8, 8, 1), (16, 8, 2), (4, 16, 2), (64, 64, 6)])
def test_haar2d_butterflies_equal_dense_definition(H, W, J):
    s = H * W
    rng = np.random.default_rng(H * 100 + W + J)
    x = rng.standard_normal((s, 3))
    t = so.haar2d_forward(x, H, W, J, np.float64)
    if s <= 256:
        L = so.haar2d_matrix(H, W, J)
        assert np.allclose(L @ L.T, np.eye(s), atol=1e-14)
        assert np.allclose(t, L @ x, atol=1e-13)
    assert np.allclose(so.haar2d_inverse(t, H, W, J, np.float64), x, atol=1e-12)
    assert np.isclose(np.sum(t * t), np.sum(x * x), rtol=1e-12)
    t32 = so.haar2d_forward(x.astype(np.float32), H, W, J, np.float32)
    assert t32.dtype == np.float32
    assert np.max(np.abs(t32 - so.haar2d_forward(x.astype(np.float32).astype(np.float64), H, W, J, np.float64))) \
        <= 1e-5 * np.max(np.abs(t))
    back32 = so.haar2d_inverse(t32, H, W, J, np.float32)
    assert np.max(np.abs(back32 - x)) <= 4e-6 * np.max(np.abs(x))


def test_haar2d_one_level_of_outer_product_is_outer_product_of_1d():
    # separability: a 2-D level applied to u v^T gives (one 1-D level of u)(one 1-D level of v)^T
    rng = np.random.default_rng(11)
    H, W = 8, 16
    u, v = rng.standard_normal(H), rng.standard_normal(W)
    g = so.haar2d_forward_grid(np.outer(u, v).reshape(H * W, 1), H, W, 1, np.float64)[:, :, 0]
    u1 = so.haar1d_forward(u[:, None], 1, np.float64)[:, 0]
    v1 = so.haar1d_forward(v[:, None], 1, np.float64)[:, 0]
    assert np.allclose(g, np.outer(u1, v1), atol=1e-14)


def test_haar2d_band_orientation_and_order():
    H = W = 4
    # a field that varies only along the width (columns): only LL and the W band respond
    x = np.tile(np.array([1.0, -1.0, 1.0, -1.0]), (H, 1)).reshape(H * W, 1)
    g = so.haar2d_forward_grid(x, H, W, 1, np.float64)[:, :, 0]
    assert np.allclose(g[:2, :2], 0) and np.allclose(g[:2, 2:], 2.0)      # top-right = width difference
    assert np.allclose(g[2:, :], 0)
    # varies only along the height: bottom-left band
    x = np.tile(np.array([1.0, -1.0, 1.0, -1.0])[:, None], (1, W)).reshape(H * W, 1)
    g = so.haar2d_forward_grid(x, H, W, 1, np.float64)[:, :, 0]
    assert np.allclose(g[2:, :2], 2.0) and np.allclose(g[:2, :], 0) and np.allclose(g[2:, 2:], 0)
    # constant c -> LL of the full pyramid = c sqrt(HW)
    t = so.haar2d_forward(np.full((H * W, 1), 2.0), H, W, 2, np.float64)[:, 0]
    assert np.isclose(t[0], 2.0 * 4.0) and np.allclose(t[1:], 0)
    # STaMP order: for every m the first (H/2^m)(W/2^m) slots are the top-left block
    H = W = 16
    perm = so.stamp_order_2d(H, W, 4)
    assert sorted(perm.tolist()) == list(range(H * W))
    for m in range(0, 5):
        h, w = H >> m, W >> m
        r, c = np.divmod(perm[:h * w], W)
        assert r.max() == h - 1 and c.max() == w - 1
    # within a level the band order is top-right, bottom-left, bottom-right
    perm = so.stamp_order_2d(4, 4, 1)
    assert perm[4:8].tolist() == [2, 3, 6, 7] and perm[8:12].tolist() == [8, 9, 12, 13]
    assert perm[12:16].tolist() == [10, 11, 14, 15]


def test_three_level_2d_on_64x64_leaves_64_low_tokens():
    # the paper's setting: three 2-D levels on 4096 image tokens leave 4096/4^3 = 64 LL tokens,
    # the number of 8-bit tokens (section "Overhead Estimates")
    perm = so.stamp_order_2d(64, 64, 3)
    r, c = np.divmod(perm[:64], 64)
    assert r.max() == 7 and c.max() == 7
    # and the full 6-level pyramid's first 64 slots span exactly that same 8x8 block
    perm6 = so.stamp_order_2d(64, 64, 6)
    assert sorted(perm6[:64].tolist()) == sorted(perm[:64].tolist())


@pytest.mark.parametrize("s,k", [(256, 8), (2048, 64), (64, 64), (64, 1)])
def test_block_locality_1d(s, k):
    """Structure the GPU kernels rely on: with k a power of two, every slot p >= k has its support
    inside one aligned block of s/k tokens, and the first k slots are the full transform of the
    per-block approximations (block sums / sqrt(s/k))."""
    J = int(np.log2(s))
    R = s // k
    L = so.haar1d_matrix(s, J) if s <= 256 else None
    if L is not None:
        for p in range(k, s):
            sup = np.nonzero(L[p])[0]
            assert sup.min() // R == sup.max() // R
    rng = np.random.default_rng(s + k)
    x = rng.standard_normal((s, 2))
    t = so.haar1d_forward(x, J, np.float64)
    approx = x.reshape(k, R, 2).sum(axis=1) / np.sqrt(R)
    assert np.allclose(t[:k], so.haar1d_forward(approx, int(np.log2(k)), np.float64), atol=1e-12)


def test_block_locality_2d():
    H = W = 16
    k = 16  # 4x4 coarse grid, blocks of 4x4 tokens
    L = so.haar2d_matrix(H, W, 4)
    for p in range(k, H * W):
        r, c = np.divmod(np.nonzero(L[p])[0], W)
        assert r.min() // 4 == r.max() // 4 and c.min() // 4 == c.max() // 4
    rng = np.random.default_rng(5)
    x = rng.standard_normal((H * W, 2))
    t = so.haar2d_forward(x, H, W, 4, np.float64)
    approx = x.reshape(4, 4, 4, 4, 2).sum(axis=(1, 3)) / 4.0      # block sums / sqrt(16)
    assert np.allclose(t[:k], so.haar2d_forward(approx.reshape(16, 2), 4, 4, 2, np.float64), atol=1e-12)


def test_energy_concentration_on_correlated_input():
    # every DWT step moves energy into the leading half of the slots (section "Efficient Energy Concentration"): on an AR(1) stream the first k slots
    # hold far more than k/s of the energy (sanity, no threshold from the paper)
    from gen import get_workload, make_inputs
    w = get_workload("cfg1", n_outlier_channels=0)
    x = make_inputs(w, need_weight=False)["X_f32"][0]
    t = so.haar1d_forward(x, w.levels, np.float64)
    frac = np.sum(t[:w.k_hi] ** 2) / np.sum(t ** 2)
    assert frac > 10 * w.k_hi / w.seq_len
    one_level = so.haar1d_forward(x, 1, np.float64)
    assert np.sum(one_level[:128] ** 2) > 0.9 * np.sum(one_level ** 2)


def test_sink_token_leaks_into_slots_powers_of_two():
    # a massive first token reaches slots 0, 1, 2, 4, ..., s/2 of the full-depth transform
    s = 2048
    x = np.zeros((s, 1)); x[0] = 100.0
    t = so.haar1d_forward(x, 11, np.float64)[:, 0]
    assert sorted(np.nonzero(t)[0].tolist()) == [0] + [1 << m for m in range(11)]
