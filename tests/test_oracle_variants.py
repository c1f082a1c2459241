"""Pins of the oracle's other sequence transforms (Haar on any length and with the first token left out, WHT, DCT),
of the transformed-bias form of the layer, and of the per-block (group) quantizer.

Expected values come from hand-worked matrices (tests/golden/haar_ragged_small.txt), orthogonality (Theorem 1 needs
an orthogonal L), library routines (scipy's Hadamard matrix and orthonormal DCT-II), closed forms, the commutation
identity of section "Method", and scalar-loop brute force."""
import os

import numpy as np
import pytest
from scipy.fft import dct as scipy_dct
from scipy.linalg import hadamard

from oracle import stamp_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _ragged_cases():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "haar_ragged_small.txt")) if l.strip() and not l.startswith("#")]
    out, i = [], 0
    while i < len(rows):
        s, J, skip = int(rows[i][0]), int(rows[i][1]), int(rows[i][2])
        out.append((s, J, bool(skip), np.array([[float(v) for v in r] for r in rows[i + 1:i + 1 + s]])))
        i += 1 + s
    return out


@pytest.mark.parametrize("s,J,skip,L_ref", _ragged_cases(), ids=lambda v: str(v) if not isinstance(v, np.ndarray) else "L")
def test_ragged_haar_hand_worked(s, J, skip, L_ref):
    assert np.allclose(L_ref @ L_ref.T, np.eye(s), atol=1e-15)      # the hand-worked matrices are orthogonal
    assert np.allclose(so.haar1d_ragged_forward(np.eye(s), J, np.float64, skip), L_ref, atol=1e-15)
    assert np.allclose(so.haar1d_ragged_matrix(s, J, skip), L_ref, atol=1e-15)


@pytest.mark.parametrize("s,J,skip", [(7, 3, False), (12, 4, False), (12, 2, False), (2049, 3, False), (2049, 12, False),
                                      (2048, 3, True), (65, 6, True), (9, 0, False)])
def test_ragged_haar_is_orthogonal_and_matches_dense(s, J, skip):
    L = so.haar1d_ragged_matrix(s, J, skip)
    assert np.allclose(L @ L.T, np.eye(s), atol=1e-13)
    rng = np.random.default_rng(s + J)
    x = rng.standard_normal((s, 3))
    t = so.haar1d_ragged_forward(x, J, np.float64, skip)
    assert np.allclose(t, L @ x, atol=1e-12)
    assert np.allclose(so.haar1d_ragged_inverse(t, J, np.float64, skip), x, atol=1e-12)
    assert np.isclose(np.sum(t * t), np.sum(x * x))                  # energy preserved
    if skip:
        assert np.array_equal(t[0], x[0])                            # the first token is not touched
    t32 = so.haar1d_ragged_forward(x.astype(np.float32), J, np.float32, skip)
    ref = L @ x.astype(np.float32).astype(np.float64)
    assert t32.dtype == np.float32 and np.max(np.abs(t32 - ref)) <= 2e-6 * np.max(np.abs(ref)) * max(J, 1)


@pytest.mark.parametrize("s,J", [(8, 3), (64, 4), (256, 8)])
def test_ragged_haar_on_a_power_of_two_is_the_haar_transform(s, J):
    assert np.allclose(so.haar1d_ragged_matrix(s, J), so.haar1d_matrix(s, J), atol=1e-14)


def test_ragged_sizes_and_full_depth():
    assert so.ragged_level_sizes(2047, 3) == [2047, 1024, 512, 256]
    assert so.max_ragged_levels(2047) == 11 and so.max_ragged_levels(2049) == 12 and so.max_ragged_levels(1) == 0
    # full depth on a constant: the single approximation holds all the energy, c sqrt(s)
    for s in (7, 12, 100):
        t = so.haar1d_ragged_forward(np.full((s, 1), 2.0), so.max_ragged_levels(s), np.float64)[:, 0]
        # not every token has the same weight in the approximation, so details need not vanish; energy does add up
        assert np.isclose(np.sum(t * t), 4.0 * s)
    with pytest.raises(ValueError):
        so.haar1d_ragged_forward(np.zeros((7, 1)), 4)


def test_sink_token_stays_in_slot_0_when_left_out():
    """The massive first token of a language model leaks into the power-of-two slots under the plain transform
    (pinned elsewhere); left out of L it stays where it is (appendix "Experimental details", LLMs)."""
    s = 2048
    x = np.zeros((s, 1)); x[0] = 100.0
    t = so.sequence_forward(x, "haar1d", 3, dtype=np.float64, skip_first=True)[:, 0]
    assert t[0] == 100.0 and not t[1:].any()
    # the three-level transform of the other 2047 tokens leaves 256 approximations: with the first token, 257 coarse slots
    assert so.ragged_level_sizes(s - 1, 3)[-1] == 256


def _sequency_hadamard(s):
    H = hadamard(s).astype(np.float64)
    changes = (np.diff(H, axis=1) != 0).sum(axis=1)
    assert sorted(changes.tolist()) == list(range(s))
    return H[np.argsort(changes)] / np.sqrt(s)


@pytest.mark.parametrize("s", [2, 8, 64, 512])
def test_wht_is_the_sequency_ordered_hadamard_matrix(s):
    Hs = _sequency_hadamard(s)
    assert np.allclose(Hs @ Hs.T, np.eye(s), atol=1e-13) and np.allclose(Hs, Hs.T)
    rng = np.random.default_rng(s)
    x = rng.standard_normal((s, 4))
    t = so.wht_forward(x, np.float64)
    assert np.allclose(t, Hs @ x, atol=1e-12)
    assert np.allclose(so.wht_inverse(t, np.float64), x, atol=1e-12)
    t32 = so.wht_forward(x.astype(np.float32), np.float32)
    assert t32.dtype == np.float32 and np.max(np.abs(t32 - Hs @ x.astype(np.float32))) <= 1e-5 * np.max(np.abs(t))
    # row q of the matrix changes sign q times; a constant lands in slot 0
    c = so.wht_forward(np.full((s, 1), 1.5), np.float64)[:, 0]
    assert np.isclose(c[0], 1.5 * np.sqrt(s)) and np.allclose(c[1:], 0)


@pytest.mark.parametrize("s", [4, 12, 64, 300])
def test_dct_is_the_orthonormal_dct2(s):
    C = so.dct_matrix(s)
    assert np.allclose(C @ C.T, np.eye(s), atol=1e-12)
    rng = np.random.default_rng(s)
    x = rng.standard_normal((s, 4))
    t = so.dct_forward(x, np.float64)
    assert np.allclose(t, scipy_dct(x, type=2, norm="ortho", axis=0), atol=1e-12)
    assert np.allclose(so.dct_inverse(t, np.float64), x, atol=1e-12)
    t32 = so.dct_forward(x.astype(np.float32), np.float32)
    assert t32.dtype == np.float32 and np.max(np.abs(t32 - t)) <= 1e-6 * np.max(np.abs(t))


def test_fourier_type_transforms_concentrate_energy_of_correlated_tokens():
    rng = np.random.default_rng(0)
    s, d, rho = 512, 64, 0.95
    e = rng.standard_normal((s, d))
    x = np.empty_like(e); x[0] = e[0] / np.sqrt(1 - rho ** 2)
    for t in range(1, s):
        x[t] = rho * x[t - 1] + e[t]
    total = np.sum(x * x)
    for name in ("wht", "dct"):
        T = so.sequence_forward(x, name, 0, dtype=np.float64)
        assert np.isclose(np.sum(T * T), total)
        assert np.sum(T[:32] ** 2) > 0.6 * total     # 1/16 of the slots hold most of the energy


@pytest.mark.parametrize("xform,levels,kw,s", [("haar1d", 5, {}, 32), ("haar1d", 3, {}, 64), ("haar1d", 4, {"skip_first": True}, 33),
                                                ("haar1d", 3, {}, 21), ("haar2d", 2, {"grid_h": 8, "grid_w": 8}, 64),
                                                ("wht", 0, {}, 32), ("dct", 0, {}, 24)])
def test_transformed_bias_equals_bias_after_inverse(xform, levels, kw, s):
    """Third form of the commutation identity: L^-1 (Q(LX) W + (L 1) b^T) = L^-1 (Q(LX) W) + 1 b^T."""
    rng = np.random.default_rng(7)
    d, N, k = 32, 20, 4
    X = rng.standard_normal((2, s, d)).astype(np.float32)
    W = (rng.standard_normal((d, N)) * 0.1).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    skip = kw.pop("skip_first", False)
    a = so.stamp_linear_forward(X, W, xform, levels, k, bias=bias, dtype=np.float64, skip_first=skip, **kw)
    b = so.stamp_linear_forward(X, W, xform, levels, k, bias=bias, dtype=np.float64, skip_first=skip, bias_mode="transformed", **kw)
    assert np.array_equal(a["codes"], b["codes"])
    assert np.allclose(a["Y"], b["Y"], atol=1e-11)
    # l = L 1 itself: for the full-depth power-of-two Haar transform it is sqrt(s) e_0
    if xform == "haar1d" and not skip and s == 32:
        ell = so.sequence_forward(np.ones((s, 1)), xform, levels, dtype=np.float64)[:, 0]
        assert np.isclose(ell[0], np.sqrt(s)) and np.allclose(ell[1:], 0)


def test_grouped_quantizer_against_scalar_loops():
    rng = np.random.default_rng(3)
    s, d, group = 6, 150, 64       # last group has 22 channels
    T = rng.standard_normal((s, d)).astype(np.float32)
    T[2, 70:128] = 0.0             # one group of one token all zero
    bits = np.array([8, 8, 4, 4, 4, 4])
    codes, scales = so.quantize_tokens_grouped(T, bits, group)
    assert scales.shape == (s, 3)
    for i in range(s):
        qm = 127 if bits[i] == 8 else 7
        for g in range(3):
            seg = T[i, g * group:(g + 1) * group]
            a = np.float32(np.max(np.abs(seg)))
            if a == 0:
                assert scales[i, g] == 0 and not codes[i, g * group:(g + 1) * group].any()
                continue
            assert scales[i, g] == np.float32(a / np.float32(qm))
            inv = np.float32(np.float32(qm) / a)
            for j, v in enumerate(seg):
                assert codes[i, g * group + j] == int(np.clip(np.rint(np.float32(v * inv)), -qm, qm))
            assert np.max(np.abs(codes[i, g * group:(g + 1) * group])) == qm
    # error at most half a step of the group's own scale: finer than one scale per token
    deq = np.repeat(scales, group, axis=1)[:, :d] * codes
    assert np.all(np.abs(deq - T) <= np.repeat(scales, group, axis=1)[:, :d] * 0.5000001)
    c1, s1 = so.quantize_tokens(T, bits)
    assert np.sum((deq - T) ** 2) < np.sum((c1 * s1[:, None] - T) ** 2)


def test_grouped_layer_equals_dense_dequantized_route():
    rng = np.random.default_rng(4)
    B, s, d, N, k = 2, 64, 160, 24, 4
    X = rng.standard_normal((B, s, d)).astype(np.float32)
    X[:, :, 5] *= 30.0
    W = (rng.standard_normal((d, N)) * 0.05).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    out = so.stamp_linear_forward_grouped(X, W, "haar2d", 3, k, 64, grid_h=8, grid_w=8, bias=bias)
    Wd = out["qw"].astype(np.float64) * np.repeat(out["swg"].astype(np.float64), 64, axis=0)[:d]
    for b in range(B):
        Td = out["codes"][b].astype(np.float64) * np.repeat(out["scales"][b].astype(np.float64), 64, axis=1)[:, :d]
        Y = so.sequence_inverse(Td @ Wd, "haar2d", 3, 8, 8, np.float64) + bias[None, :]
        assert np.max(np.abs(out["Y"][b] - Y)) <= 2e-5 * np.max(np.abs(Y))
    # weights: one scale per (group, output channel)
    assert out["swg"].shape == (3, N) and np.all(np.max(np.abs(out["qw"][:64]), axis=0) == 7)
    # group scales absorb the outlier channel: better than per-token scales on the same input
    ref = X.astype(np.float64) @ W.astype(np.float64) + bias
    per_token = so.stamp_linear_forward(X, W, "haar2d", 3, k, grid_h=8, grid_w=8, bias=bias)
    assert so.sqnr_db(ref, out["Y"]) > so.sqnr_db(ref, per_token["Y"]) + 3.0
