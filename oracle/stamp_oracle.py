"""CPU oracle for the STaMP quantized linear layer (arXiv 2510.26771).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP library is checked
against.  Only tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product path never does, and it shares no code with the HIP sources.

What it computes is the paper's Algorithm "STaMP Linear" (section "Sequence Transform and Mixed
Precision"), taken step by step:

    X <- L X            sequence transform along the tokens (Haar DWT, section "Efficient
                        Energy Concentration")
    x_i <- Q(x_i; b_i)  per-token quantization (Background, Eq. 1), b_i = 8 for the first k
                        transformed tokens and 4 for the rest (section "Optimal bit allocation")
    Y <- X W            integer matrix product against per-output-channel quantized weights
    Y <- L^-1 Y         inverse sequence transform (valid by the commutation identity of
                        section "Method")
    Y <- Y + bias

STaMP is an approximation scheme, so the oracle is the algorithm itself rather than a closed
form.  Two precisions are offered through the ``dtype`` argument of every floating-point step:

* ``np.float64``: the definition, used by the CPU tests to pin the fp32 path (and available as
  dense matrices through ``haar1d_matrix`` / ``haar2d_matrix``, which are written from the
  textbook Haar basis functions, not from the butterfly recursion).
* ``np.float32``: the bit reference.  Every add, subtract, multiply and divide below is one
  individually rounded IEEE operation on numpy arrays (numpy never fuses a multiply with an
  add), in the order written.  Quantized codes depend on these roundings, so the HIP path has
  to reproduce the same operation order for the forward transform, the scale and the rounding.

Readings of the paper where it is silent (each also listed in the design document):

* Haar matrix: orthonormal (Theorem 1 needs an orthogonal L), detail = even minus odd,
  approximations first (each step moves the energy into the leading half of the slots, section
  "Efficient Energy Concentration"), Mallat ordering: after J levels
  slot 0.. hold the coarsest approximations, then the details from coarse to fine.
* Operation order of the transform (the paper gives none): a coefficient is the inner product
  with its basis function, +-2^(-l/2) on the wavelet's two halves, so it is evaluated as
  (sum of the first half - sum of the second half) * 2^(-l/2): the sums are built level by
  level as plain pairwise sums A = x[2i] + x[2i+1], D = x[2i] - x[2i+1] (no scaling inside the
  recursion), and each finished coefficient is multiplied ONCE by norm(l) = fl(2^(-l/2)) of its
  level (exact for even l).  The inverse multiplies every coefficient by the same norm(l) first
  and then runs plain butterflies x[2i] = a + d, x[2i+1] = a - d.
* 2-D: pyramid (recursion on the low-low quarter: the same section gives a 2-D step a quarter of the
  tokens); one 2-D level
  on a 2x2 cell [[p, q], [u, v]] is t0=p+q, t1=p-q, t2=u+v, t3=u-v, LL=t0+t2, W=t1+t3,
  H=t0-t2, D=t1-t3, and a finished level-l coefficient is multiplied once by 2^(-l) (exact).
  STaMP order in 2-D: final LL block row-major, then per level from coarse to fine the blocks
  [W (top-right), H (bottom-left), D (bottom-right)], each row-major.
* Quantizer: the benchmark configurations fix the symmetric specialisation of Eq. 1:
  qmax = 2^(b-1) - 1, scale = absmax / qmax (range-based, no clipping, as in the Background
  section), code = clamp(rne(x * (qmax / absmax)), -qmax, qmax).  A zero row gets scale 0 and
  codes 0.  Rounding is round-half-to-even.
* Asymmetric quantizer (the min-max form the paper's experiments use; Background, Eq. 1 in full):
  codes in [0, 2^b - 1]; range = max - min over the token's channels, exactly as the range-setting
  sentence of the Background section defines it (a one-sided token keeps its own, narrower range:
  0 need not lie inside it); scale = range / (2^b - 1) (the printed scale is its reciprocal: Eq. 1
  divides by s, and the proof of the range bound uses range / (2^b - 1)); integer offset
  z = rne(-min / scale) (Eq. 1 adds z to a rounded value and calls the result an integer, so z is
  rounded; it is any integer, negative for an all-positive token); code = clamp(rne(x / scale) + z,
  0, 2^b - 1), evaluated as rne(fl(x * inv)) with inv = (2^b - 1) / range.
  The paper does not say what a token with max = min gets (its printed scale divides by zero): here
  such a token takes range = |value|, so that it is still reproduced to within rounding; a zero
  token gets scale 0, z 0, codes 0.
* Weights: per output channel, absmax / 7, round to nearest, no range search.
* W is [d_in, d_out] and Y = X W.

parity unpinned: the paper prints no worked numeric example of a transformed or quantized
vector, so absolute output values are pinned only through the invariants, closed forms, dense
definitions and brute-force checks in tests/ (listed in the design document).
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Tuple

import numpy as np


def haar_norm(level: int, dtype=np.float32):
    """norm(l) = 2^(-l/2) rounded to dtype: a power of two for even l, else a power of two times
    fl(1/sqrt 2) (fp32: bit pattern 0x3F3504F3 scaled)."""
    ft = np.dtype(dtype).type
    if level % 2 == 0:
        return ft(2.0 ** (-(level // 2)))
    return ft(ft(0.70710678118654752440) * ft(2.0 ** (-((level - 1) // 2))))


def _norms_1d(s: int, levels: int, dtype) -> np.ndarray:
    """Per-slot normalisation of the J-level 1-D transform in STaMP order."""
    nrm = np.empty(s, dtype=dtype)
    nrm[0:s >> levels] = haar_norm(levels, dtype)
    for l in range(levels, 0, -1):
        nrm[s >> l:s >> (l - 1)] = haar_norm(l, dtype)
    return nrm


def _is_pow2(n: int) -> bool:
    return n >= 1 and (n & (n - 1)) == 0


# --------------------------------------------------------------------------------------
# 1-D Haar DWT along axis 0 (tokens).  Section "Efficient Energy Concentration".
# --------------------------------------------------------------------------------------

def haar1d_forward(x: np.ndarray, levels: int, dtype=np.float32) -> np.ndarray:
    """J-level orthonormal Haar DWT of x[s, ...] along axis 0, result in STaMP order.

    Level l = 1..J acts on the first n = s / 2^(l-1) slots (the current block sums):
    the n/2 pair sums go to slots [0, n/2), the n/2 pair differences to [n/2, n); slots >= n
    keep the differences of the earlier (finer) levels.  Each slot is then multiplied once by
    the norm of its level.
    """
    t = np.array(x, dtype=dtype, copy=True)
    s = t.shape[0]
    if not _is_pow2(s) or levels < 0 or (1 << levels) > s:
        raise ValueError("seq_len must be a power of two and levels <= log2(seq_len)")
    n = s
    for _ in range(levels):
        even = t[0:n:2].copy()
        odd = t[1:n:2].copy()
        t[0:n // 2] = even + odd
        t[n // 2:n] = even - odd
        n //= 2
    nrm = _norms_1d(s, levels, dtype)
    return t * nrm.reshape((s,) + (1,) * (t.ndim - 1))


def haar1d_inverse(t: np.ndarray, levels: int, dtype=np.float32) -> np.ndarray:
    """Inverse (= transpose) of haar1d_forward: scale every slot by the norm of its level, then
    levels J..1 of plain butterflies x[2i] = a + d, x[2i+1] = a - d."""
    x = np.array(t, dtype=dtype, copy=True)
    s = x.shape[0]
    if not _is_pow2(s) or levels < 0 or (1 << levels) > s:
        raise ValueError("seq_len must be a power of two and levels <= log2(seq_len)")
    nrm = _norms_1d(s, levels, dtype)
    x = x * nrm.reshape((s,) + (1,) * (x.ndim - 1))
    n = s >> (levels - 1) if levels > 0 else s
    for _ in range(levels):
        a = x[0:n // 2].copy()
        d = x[n // 2:n].copy()
        x[0:n:2] = a + d
        x[1:n:2] = a - d
        n *= 2
    return x


def haar1d_matrix(s: int, levels: int) -> np.ndarray:
    """Dense fp64 L (s x s) of the J-level Haar DWT in STaMP order, from the basis functions.

    Rows [0, s/2^J): box functions of length 2^J and height 2^(-J/2).
    Row s/2^l + i (l = J..1, i < s/2^l): the wavelet of level l at position i: +2^(-l/2) on
    tokens [i 2^l, i 2^l + 2^(l-1)), -2^(-l/2) on the following 2^(l-1) tokens.
    """
    L = np.zeros((s, s), dtype=np.float64)
    J = levels
    na = s >> J
    for i in range(na):
        L[i, i << J:(i + 1) << J] = 2.0 ** (-J / 2.0)
    for l in range(J, 0, -1):
        base = s >> l
        half = 1 << (l - 1)
        h = 2.0 ** (-l / 2.0)
        for i in range(base):
            L[base + i, (i << l):(i << l) + half] = h
            L[base + i, (i << l) + half:(i + 1) << l] = -h
    return L


# --------------------------------------------------------------------------------------
# 1-D Haar DWT of any length, and with the first token left out of the transform.
#
# The paper picks the Haar wavelet for needing next to no padding (footnote to the DWT paragraph of section
# "Efficient Energy Concentration") and, for language models, keeps the first token (the attention sink) out
# of L and at 8 bits (appendix "Experimental details", LLMs, STaMP paragraph), which leaves s - 1 tokens: an odd
# number.  It does not say how an odd number of approximations is split.  Reading taken: a level pairs the
# current approximations (0,1), (2,3), ...; an odd one out is carried to the next level unchanged, as its last
# approximation (no padding, L stays orthogonal).  A carried token has a different weight than a pair sum, so
# the normalisation cannot wait until the end: every level is the textbook orthonormal butterfly
# a = (x0 + x1) * C, d = (x0 - x1) * C with C = fl(1 / sqrt 2), each operation rounded.
# STaMP order: [token 0 if it is left out] [approximations of the last level] [details coarse to fine].
# --------------------------------------------------------------------------------------

def ragged_level_sizes(n: int, levels: int):
    """Numbers of approximations n_0 = n, n_l = ceil(n_(l-1) / 2) after each level."""
    sizes = [n]
    for _ in range(levels):
        sizes.append((sizes[-1] + 1) // 2)
    return sizes


def max_ragged_levels(n: int) -> int:
    """Levels after which a single approximation is left."""
    l = 0
    while n > 1:
        n = (n + 1) // 2
        l += 1
    return l


def haar1d_ragged_forward(x: np.ndarray, levels: int, dtype=np.float32, skip_first: bool = False) -> np.ndarray:
    """J-level orthonormal Haar DWT of x[s, ...] along axis 0 for any s, result in STaMP order."""
    ft = np.dtype(dtype).type
    C = ft(0.70710678118654752440)
    t = np.array(x, dtype=dtype, copy=True)
    o = 1 if skip_first else 0
    n = t.shape[0] - o
    if levels < 0 or levels > max_ragged_levels(max(n, 1)):
        raise ValueError("more levels than the sequence allows")
    for _ in range(levels):
        m = n // 2
        w = t[o:o + n].copy()
        t[o:o + m] = (w[0:2 * m:2] + w[1:2 * m:2]) * C
        if n % 2:
            t[o + m] = w[n - 1]
        nn = (n + 1) // 2
        t[o + nn:o + nn + m] = (w[0:2 * m:2] - w[1:2 * m:2]) * C
        n = nn
    return t


def haar1d_ragged_inverse(t: np.ndarray, levels: int, dtype=np.float32, skip_first: bool = False) -> np.ndarray:
    """Inverse (= transpose) of haar1d_ragged_forward."""
    ft = np.dtype(dtype).type
    C = ft(0.70710678118654752440)
    x = np.array(t, dtype=dtype, copy=True)
    o = 1 if skip_first else 0
    sizes = ragged_level_sizes(x.shape[0] - o, levels)
    for l in range(levels, 0, -1):
        n, nn = sizes[l - 1], sizes[l]
        m = n // 2
        a = x[o:o + nn].copy()
        d = x[o + nn:o + nn + m].copy()
        x[o:o + 2 * m:2] = (a[:m] + d) * C
        x[o + 1:o + 2 * m:2] = (a[:m] - d) * C
        if n % 2:
            x[o + n - 1] = a[nn - 1]
    return x


def haar1d_ragged_matrix(s: int, levels: int, skip_first: bool = False) -> np.ndarray:
    """Dense fp64 L (s x s) of the ragged transform, as a product of one-level matrices: level l is the identity
    outside its n_(l-1) approximations, and inside them has the rows (e_2i + e_2i+1) / sqrt 2 for every pair,
    e_last for an odd one out, then (e_2i - e_2i+1) / sqrt 2 for every pair."""
    o = 1 if skip_first else 0
    L = np.eye(s)
    n = s - o
    r = 1.0 / math.sqrt(2.0)
    for _ in range(levels):
        H = np.eye(s)
        m, nn = n // 2, (n + 1) // 2
        H[o:o + n, o:o + n] = 0.0
        for i in range(m):
            H[o + i, o + 2 * i] = r
            H[o + i, o + 2 * i + 1] = r
            H[o + nn + i, o + 2 * i] = r
            H[o + nn + i, o + 2 * i + 1] = -r
        if n % 2:
            H[o + m, o + n - 1] = 1.0
        L = H @ L
        n = nn
    return L


# --------------------------------------------------------------------------------------
# Walsh-Hadamard and cosine transforms along the tokens (section "Efficient Energy Concentration": the
# Fourier-type transforms the paper compares the DWT with).
#
# WHT: orthonormal, rows in SEQUENCY order (row q changes sign q times), which is the order in which the
# rows are the signs of the cosine basis and therefore the order in which "the first k tokens" are the low
# frequencies.  Evaluated as log2(s) levels of plain butterflies (u, v) -> (u + v, u - v) at distance 1, 2, 4, ...
# (the Hadamard-ordered fast transform), then reordered, then multiplied once by 2^(-log2(s) / 2).
# DCT: the orthonormal DCT-II, T_k = c_k sum_n x_n cos(pi (2 n + 1) k / (2 s)), c_0 = sqrt(1 / s), c_k = sqrt(2 / s).
# Evaluated as the dense product in fp64, whatever `dtype` is, and then rounded to `dtype`: a product of s terms
# has no canonical fp32 order, and this way the quantized codes do not depend on one.
# --------------------------------------------------------------------------------------

def wht_sequency_permutation(s: int) -> np.ndarray:
    """perm[q] = row of the Hadamard-ordered (Sylvester) matrix that has sequency q: the bit reversal of the
    Gray code of q."""
    J = s.bit_length() - 1
    if not _is_pow2(s):
        raise ValueError("the WHT needs a power-of-two length")
    q = np.arange(s, dtype=np.int64)
    g = q ^ (q >> 1)
    rev = np.zeros_like(g)
    for b in range(J):
        rev |= ((g >> b) & 1) << (J - 1 - b)
    return rev


def wht_forward(x: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Orthonormal sequency-ordered WHT of x[s, ...] along axis 0 (its own inverse)."""
    t = np.array(x, dtype=dtype, copy=True)
    s = t.shape[0]
    J = s.bit_length() - 1
    perm = wht_sequency_permutation(s)
    h = 1
    while h < s:
        v = t.reshape((s // (2 * h), 2, h) + t.shape[1:])
        u0 = v[:, 0].copy()
        u1 = v[:, 1].copy()
        v[:, 0] = u0 + u1
        v[:, 1] = u0 - u1
        h *= 2
    return t[perm] * haar_norm(J, dtype)


def wht_inverse(t: np.ndarray, dtype=np.float32) -> np.ndarray:
    """The sequency-ordered orthonormal WHT matrix is symmetric and orthogonal: the inverse is the transform."""
    return wht_forward(t, dtype)


def dct_matrix(s: int) -> np.ndarray:
    """Dense fp64 orthonormal DCT-II matrix C[k, n]."""
    k = np.arange(s, dtype=np.float64)[:, None]
    n = np.arange(s, dtype=np.float64)[None, :]
    C = np.cos(np.pi * (2.0 * n + 1.0) * k / (2.0 * s)) * math.sqrt(2.0 / s)
    C[0, :] = math.sqrt(1.0 / s)
    return C


def dct_forward(x: np.ndarray, dtype=np.float32) -> np.ndarray:
    x64 = np.asarray(x, dtype=np.float64)
    s = x64.shape[0]
    return (dct_matrix(s) @ x64.reshape(s, -1)).reshape(x64.shape).astype(dtype)


def dct_inverse(t: np.ndarray, dtype=np.float32) -> np.ndarray:
    t64 = np.asarray(t, dtype=np.float64)
    s = t64.shape[0]
    return (dct_matrix(s).T @ t64.reshape(s, -1)).reshape(t64.shape).astype(dtype)


# --------------------------------------------------------------------------------------
# 2-D Haar pyramid over an H x W token grid, token t = r * W + c.
# --------------------------------------------------------------------------------------

def _norms_2d_grid(H: int, W: int, levels: int, dtype) -> np.ndarray:
    """Per-position normalisation 2^(-l) of the Mallat coefficient grid (level-l bands and, for
    the remaining low-low block, l = J).  Exact powers of two."""
    ft = np.dtype(dtype).type
    nrm = np.empty((H, W), dtype=dtype)
    for l in range(1, levels + 1):
        h, w = H >> (l - 1), W >> (l - 1)
        nrm[0:h, 0:w] = ft(2.0 ** (-l))     # overwritten below for the part that recurses further
    if levels == 0:
        nrm[:, :] = ft(1.0)
    return nrm


def haar2d_forward_grid(x: np.ndarray, grid_h: int, grid_w: int, levels: int, dtype=np.float32) -> np.ndarray:
    """J-level 2-D Haar pyramid; returns the coefficient grid [H, W, ...] (Mallat layout:
    LL top-left, width-difference band top-right, height-difference band bottom-left,
    diagonal band bottom-right, recursion on the top-left quarter)."""
    H, W = grid_h, grid_w
    if not (_is_pow2(H) and _is_pow2(W)) or levels < 0 or (1 << levels) > min(H, W):
        raise ValueError("grid sides must be powers of two and levels <= log2(min side)")
    g = np.array(x, dtype=dtype, copy=True).reshape((H, W) + x.shape[1:])
    h, w = H, W
    for _ in range(levels):
        p = g[0:h:2, 0:w:2].copy()
        q = g[0:h:2, 1:w:2].copy()
        u = g[1:h:2, 0:w:2].copy()
        v = g[1:h:2, 1:w:2].copy()
        t0 = p + q
        t1 = p - q
        t2 = u + v
        t3 = u - v
        g[0:h // 2, 0:w // 2] = t0 + t2
        g[0:h // 2, w // 2:w] = t1 + t3
        g[h // 2:h, 0:w // 2] = t0 - t2
        g[h // 2:h, w // 2:w] = t1 - t3
        h //= 2
        w //= 2
    return g * _norms_2d_grid(H, W, levels, dtype).reshape((H, W) + (1,) * (g.ndim - 2))


def haar2d_inverse_grid(g_in: np.ndarray, levels: int, dtype=np.float32) -> np.ndarray:
    """Inverse of haar2d_forward_grid on a coefficient grid [H, W, ...]."""
    g = np.array(g_in, dtype=dtype, copy=True)
    H, W = g.shape[0], g.shape[1]
    g = g * _norms_2d_grid(H, W, levels, dtype).reshape((H, W) + (1,) * (g.ndim - 2))
    h, w = (H >> (levels - 1), W >> (levels - 1)) if levels > 0 else (H, W)
    for _ in range(levels):
        cLL = g[0:h // 2, 0:w // 2].copy()
        cW = g[0:h // 2, w // 2:w].copy()
        cH = g[h // 2:h, 0:w // 2].copy()
        cD = g[h // 2:h, w // 2:w].copy()
        t0 = cLL + cH
        t2 = cLL - cH
        t1 = cW + cD
        t3 = cW - cD
        g[0:h:2, 0:w:2] = t0 + t1
        g[0:h:2, 1:w:2] = t0 - t1
        g[1:h:2, 0:w:2] = t2 + t3
        g[1:h:2, 1:w:2] = t2 - t3
        h *= 2
        w *= 2
    return g


def stamp_order_2d(grid_h: int, grid_w: int, levels: int) -> np.ndarray:
    """perm[p] = flat index (r * W + c) into the Mallat coefficient grid of STaMP slot p.

    Slots: the final LL block row-major, then for l = J..1 the three detail blocks of level l
    in the order top-right, bottom-left, bottom-right, each row-major.  Lowest frequencies first,
    so "the first k tokens" are the coarsest coefficients.
    """
    H, W, J = grid_h, grid_w, levels
    idx = np.arange(H * W, dtype=np.int64).reshape(H, W)
    out = [idx[0:H >> J, 0:W >> J].ravel()]
    for l in range(J, 0, -1):
        h, w = H >> l, W >> l  # size of each band of level l
        out.append(idx[0:h, w:2 * w].ravel())
        out.append(idx[h:2 * h, 0:w].ravel())
        out.append(idx[h:2 * h, w:2 * w].ravel())
    return np.concatenate(out)


def haar2d_forward(x: np.ndarray, grid_h: int, grid_w: int, levels: int, dtype=np.float32) -> np.ndarray:
    """x[s = H*W, ...] -> transformed tokens [s, ...] in STaMP order."""
    g = haar2d_forward_grid(x, grid_h, grid_w, levels, dtype)
    flat = g.reshape((grid_h * grid_w,) + g.shape[2:])
    return flat[stamp_order_2d(grid_h, grid_w, levels)]


def haar2d_inverse(t: np.ndarray, grid_h: int, grid_w: int, levels: int, dtype=np.float32) -> np.ndarray:
    """Inverse of haar2d_forward: STaMP-ordered tokens -> original token order."""
    perm = stamp_order_2d(grid_h, grid_w, levels)
    flat = np.empty(t.shape, dtype=dtype)
    flat[perm] = np.asarray(t, dtype=dtype)
    g = flat.reshape((grid_h, grid_w) + t.shape[1:])
    x = haar2d_inverse_grid(g, levels, dtype)
    return x.reshape(t.shape)


def _phi(n: int, l: int, i: int) -> np.ndarray:
    """Box function of level l at position i over n samples, unit norm."""
    f = np.zeros(n)
    f[i << l:(i + 1) << l] = 2.0 ** (-l / 2.0)
    return f


def _psi(n: int, l: int, i: int) -> np.ndarray:
    """Haar wavelet of level l at position i over n samples, unit norm (+ first half, - second)."""
    f = np.zeros(n)
    half = 1 << (l - 1)
    f[(i << l):(i << l) + half] = 2.0 ** (-l / 2.0)
    f[(i << l) + half:(i + 1) << l] = -(2.0 ** (-l / 2.0))
    return f


def haar2d_matrix(grid_h: int, grid_w: int, levels: int) -> np.ndarray:
    """Dense fp64 L (s x s) of the 2-D pyramid in STaMP order, from separable basis functions:
    LL = phi(rows) x phi(cols); W band = phi(rows) x psi(cols) (difference along the width);
    H band = psi(rows) x phi(cols); D band = psi(rows) x psi(cols)."""
    H, W, J = grid_h, grid_w, levels
    rows = []
    for i in range(H >> J):
        for j in range(W >> J):
            rows.append(np.outer(_phi(H, J, i), _phi(W, J, j)).ravel())
    for l in range(J, 0, -1):
        h, w = H >> l, W >> l
        for band in ("W", "H", "D"):
            for i in range(h):
                for j in range(w):
                    fr = _phi(H, l, i) if band == "W" else _psi(H, l, i)
                    fc = _phi(W, l, j) if band == "H" else _psi(W, l, j)
                    rows.append(np.outer(fr, fc).ravel())
    return np.stack(rows)


# --------------------------------------------------------------------------------------
# Transform dispatch
# --------------------------------------------------------------------------------------

def _is_ragged(s: int, xform: str, skip_first: bool) -> bool:
    """The 1-D Haar transform takes its ragged form when the first token is left out or the length is not a
    power of two."""
    return xform == "haar1d" and (skip_first or not _is_pow2(s))


def sequence_forward(x, xform: str, levels: int, grid_h: int = 0, grid_w: int = 0, dtype=np.float32,
                     skip_first: bool = False):
    """T = L X for one sequence x[s, ...]."""
    if skip_first and xform != "haar1d":
        raise ValueError("leaving the first token out is defined for the 1-D Haar transform")
    if xform == "identity":
        return np.array(x, dtype=dtype, copy=True)
    if xform == "haar1d":
        if _is_ragged(np.shape(x)[0], xform, skip_first):
            return haar1d_ragged_forward(x, levels, dtype, skip_first)
        return haar1d_forward(x, levels, dtype)
    if xform == "haar2d":
        return haar2d_forward(x, grid_h, grid_w, levels, dtype)
    if xform == "wht":
        return wht_forward(x, dtype)
    if xform == "dct":
        return dct_forward(x, dtype)
    raise ValueError(f"unknown transform {xform!r}")


def sequence_inverse(t, xform: str, levels: int, grid_h: int = 0, grid_w: int = 0, dtype=np.float32,
                     skip_first: bool = False):
    """X = L^-1 T for one sequence t[s, ...]."""
    if xform == "identity":
        return np.array(t, dtype=dtype, copy=True)
    if xform == "haar1d":
        if _is_ragged(np.shape(t)[0], xform, skip_first):
            return haar1d_ragged_inverse(t, levels, dtype, skip_first)
        return haar1d_inverse(t, levels, dtype)
    if xform == "haar2d":
        return haar2d_inverse(t, grid_h, grid_w, levels, dtype)
    if xform == "wht":
        return wht_inverse(t, dtype)
    if xform == "dct":
        return dct_inverse(t, dtype)
    raise ValueError(f"unknown transform {xform!r}")


# --------------------------------------------------------------------------------------
# Quantizer (Background, Eq. 1, symmetric absmax specialisation) and mixed precision
# --------------------------------------------------------------------------------------

def qmax_of(bits: int) -> int:
    return (1 << (bits - 1)) - 1


def token_bits(seq_len: int, k_hi: int, bits_hi: int = 8, bits_lo: int = 4) -> np.ndarray:
    """b_i: bits_hi for the first k transformed tokens, bits_lo for the rest."""
    b = np.full(seq_len, bits_lo, dtype=np.int32)
    b[:k_hi] = bits_hi
    return b


def effective_bits(seq_len: int, k_hi: int, bits_hi: int = 8, bits_lo: int = 4) -> float:
    """Average activation bit width of the two-level allocation."""
    return (bits_hi * k_hi + bits_lo * (seq_len - k_hi)) / seq_len


def quantize_tokens(T: np.ndarray, bits: np.ndarray, dtype=np.float32) -> Tuple[np.ndarray, np.ndarray]:
    """Per-token symmetric quantization of T[s, d] with bits[s].

    a_i = max_j |T_ij|;  scale_i = a_i / qmax_i;  inv_i = qmax_i / a_i (two separate divisions);
    code_ij = clamp(rne(T_ij * inv_i), -qmax_i, qmax_i).  Zero rows: scale = inv = 0.
    Returns (codes int8 [s, d], scale [s]).
    """
    T = np.asarray(T, dtype=dtype)
    ft = np.dtype(dtype).type
    a = np.max(np.abs(T), axis=1)
    qm = np.array([qmax_of(int(b)) for b in bits], dtype=dtype)
    nz = a > 0
    scale = np.zeros_like(a)
    inv = np.zeros_like(a)
    scale[nz] = a[nz] / qm[nz]
    inv[nz] = qm[nz] / a[nz]
    r = np.rint(T * inv[:, None])          # np.rint rounds half to even
    r = np.minimum(np.maximum(r, -qm[:, None]), qm[:, None])
    assert scale.dtype == np.dtype(dtype) and r.dtype == np.dtype(dtype) and ft is not None
    return r.astype(np.int8), scale


def dequantize_tokens(codes: np.ndarray, scale: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Q^-1: code * scale."""
    return codes.astype(dtype) * np.asarray(scale, dtype=dtype)[:, None]


def qmax_unsigned(bits: int) -> int:
    return (1 << bits) - 1


def quantize_tokens_asym(T: np.ndarray, bits: np.ndarray, dtype=np.float32) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-token asymmetric min-max quantization of T[s, d] with bits[s] (Background, Eq. 1 and the
    range-setting sentence after it).

    lo_i = min_j T_ij, hi_i = max_j T_ij, range_i = hi_i - lo_i (a token with hi = lo: range = |hi|);
    scale_i = range_i / (2^b - 1);  inv_i = (2^b - 1) / range_i (two separate divisions);
    z_i = rne(-(lo_i * inv_i));  code_ij = clamp(rne(T_ij * inv_i) + z_i, 0, 2^b - 1).
    Zero rows: scale = inv = z = 0.  Returns (codes uint8 [s, d], scale [s], z [s] as integers
    held in `dtype`; z may lie outside [0, 2^b - 1]).
    """
    T = np.asarray(T, dtype=dtype)
    zero = np.zeros((), dtype=dtype)
    lo = np.min(T, axis=1)
    hi = np.max(T, axis=1)
    rng = hi - lo
    flat = rng == 0
    rng[flat] = np.abs(hi[flat])
    qm = np.array([qmax_unsigned(int(b)) for b in bits], dtype=dtype)
    nz = rng > 0
    scale = np.zeros_like(rng)
    inv = np.zeros_like(rng)
    scale[nz] = rng[nz] / qm[nz]
    inv[nz] = qm[nz] / rng[nz]
    z = np.rint(-(lo * inv)) + zero  # + 0 turns a -0 into +0
    r = np.rint(T * inv[:, None]) + z[:, None]
    r = np.minimum(np.maximum(r, zero), qm[:, None])
    assert scale.dtype == np.dtype(dtype) and r.dtype == np.dtype(dtype) and z.dtype == np.dtype(dtype)
    return r.astype(np.uint8), scale, z


def dequantize_tokens_asym(codes: np.ndarray, scale: np.ndarray, z: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Q^-1: (code - z) * scale."""
    return (codes.astype(dtype) - np.asarray(z, dtype=dtype)[:, None]) * np.asarray(scale, dtype=dtype)[:, None]


def quantize_weight(W: np.ndarray, bits_w: int = 4, dtype=np.float32) -> Tuple[np.ndarray, np.ndarray]:
    """Per-output-channel symmetric round-to-nearest quantization of W[d_in, d_out].

    Returns (codes int8 [d_in, d_out], sw [d_out]).
    """
    codes_t, sw = quantize_tokens(np.ascontiguousarray(np.asarray(W, dtype=dtype).T),
                                  np.full(W.shape[1], bits_w, dtype=np.int32), dtype)
    return np.ascontiguousarray(codes_t.T), sw


# --------------------------------------------------------------------------------------
# Per-block (group) scales (Experiments, LVM set-up and appendix "Experimental details", LVMs: per-block
# weight and activation quantization with blocks of 64 channels, the setting of the paper's first table).
# Every token keeps its bit width; inside a token every group of `group` consecutive channels has its own
# symmetric scale (same arithmetic as quantize_tokens, per group).  Weights: per output channel, one scale
# per group of `group` consecutive input channels.  The last group may be shorter.
# --------------------------------------------------------------------------------------

def quantize_tokens_grouped(T: np.ndarray, bits: np.ndarray, group: int = 64, dtype=np.float32):
    """Returns (codes int8 [s, d], scales [s, G]) with G = ceil(d / group)."""
    T = np.asarray(T, dtype=dtype)
    s, d = T.shape
    G = (d + group - 1) // group
    codes = np.empty((s, d), dtype=np.int8)
    scales = np.empty((s, G), dtype=dtype)
    for g in range(G):
        c, sc = quantize_tokens(T[:, g * group:(g + 1) * group], bits, dtype)
        codes[:, g * group:(g + 1) * group] = c
        scales[:, g] = sc
    return codes, scales


def quantize_weight_grouped(W: np.ndarray, bits_w: int = 4, group: int = 64, dtype=np.float32):
    """W[d_in, d_out] -> (codes int8 [d_in, d_out], scales [G, d_out])."""
    W = np.asarray(W, dtype=dtype)
    d, N = W.shape
    G = (d + group - 1) // group
    codes = np.empty((d, N), dtype=np.int8)
    scales = np.empty((G, N), dtype=dtype)
    for g in range(G):
        c, sc = quantize_weight(W[g * group:(g + 1) * group], bits_w, dtype)
        codes[g * group:(g + 1) * group] = c
        scales[g] = sc
    return codes, scales


def grouped_dequant_gemm(codes: np.ndarray, sa: np.ndarray, qw: np.ndarray, swg: np.ndarray, group: int = 64,
                         dtype=np.float32) -> np.ndarray:
    """Y'[m, n] = sum_g (float(acc_g[m, n]) * sa[m, g]) * swg[g, n], acc_g the exact integer sum over the
    channels of group g, the groups added in increasing order, every operation rounded to `dtype`."""
    M, d = codes.shape
    N = qw.shape[1]
    G = (d + group - 1) // group
    Y = np.zeros((M, N), dtype=dtype)
    for g in range(G):
        acc = int_gemm(codes[:, g * group:(g + 1) * group], qw[g * group:(g + 1) * group])
        Y = Y + (acc.astype(dtype) * np.asarray(sa[:, g], dtype=dtype)[:, None]) * np.asarray(swg[g], dtype=dtype)[None, :]
    return Y


def stamp_linear_forward_grouped(X: np.ndarray, W: np.ndarray, xform: str, levels: int, k_hi: int, group: int = 64,
                                 bits_hi: int = 8, bits_lo: int = 4, bits_w: int = 4, grid_h: int = 0, grid_w: int = 0,
                                 bias: Optional[np.ndarray] = None, dtype=np.float32,
                                 skip_first: bool = False) -> Dict[str, np.ndarray]:
    """Algorithm "STaMP Linear" with per-block scales for activations and weights."""
    B, s, d = X.shape
    N = W.shape[1]
    bits = token_bits(s, k_hi, bits_hi, bits_lo)
    qw, swg = quantize_weight_grouped(W, bits_w, group, dtype)
    G = swg.shape[0]
    T = np.empty((B, s, d), dtype=dtype)
    codes = np.empty((B, s, d), dtype=np.int8)
    scales = np.empty((B, s, G), dtype=dtype)
    Yt = np.empty((B, s, N), dtype=dtype)
    Y = np.empty((B, s, N), dtype=dtype)
    for b in range(B):
        T[b] = sequence_forward(X[b], xform, levels, grid_h, grid_w, dtype, skip_first)
        codes[b], scales[b] = quantize_tokens_grouped(T[b], bits, group, dtype)
        Yt[b] = grouped_dequant_gemm(codes[b], scales[b], qw, swg, group, dtype)
        Y[b] = sequence_inverse(Yt[b], xform, levels, grid_h, grid_w, dtype, skip_first)
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=dtype)[None, None, :]
    return {"T": T, "codes": codes, "scales": scales, "bits": bits, "qw": qw, "swg": swg, "Yt": Yt, "Y": Y}


# --------------------------------------------------------------------------------------
# Integer GEMM
# --------------------------------------------------------------------------------------

def int_gemm(q: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """acc[m, n] = sum_k q[m, k] * qw[k, n], exact, returned as int32.

    Evaluated with the fp64 matrix product: every partial sum is an integer below 2^53 in
    magnitude, so each fp64 operation is exact whatever the summation order.  The result is
    checked to fit 24 bits, which the fp32 dequantization relies on."""
    K = q.shape[1]
    bound = float(K) * float(np.max(np.abs(q), initial=0)) * float(np.max(np.abs(qw), initial=0))
    assert bound < 2.0 ** 53
    acc = q.astype(np.float64) @ qw.astype(np.float64)
    assert np.max(np.abs(acc), initial=0.0) < 2.0 ** 24, "accumulator exceeds the exact fp32 integer range"
    out = acc.astype(np.int64)
    assert np.array_equal(out.astype(np.float64), acc)
    return out.astype(np.int32)


# --------------------------------------------------------------------------------------
# bf16 rounding of the output (round-to-nearest-even on the fp32 bit pattern)
# --------------------------------------------------------------------------------------

def round_to_bf16(y: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 value (ties to even), returned as fp32."""
    u = np.ascontiguousarray(y, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return (r.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(np.shape(y))


# --------------------------------------------------------------------------------------
# The whole layer
# --------------------------------------------------------------------------------------

def quantize_activation(X: np.ndarray, xform: str, levels: int, k_hi: int, bits_hi: int = 8,
                        bits_lo: int = 4, grid_h: int = 0, grid_w: int = 0,
                        dtype=np.float32, act_quant: str = "sym", skip_first: bool = False) -> Dict[str, np.ndarray]:
    """Steps 1-2 of the algorithm for X[batch, s, d]: T = L X per sequence, then per-token
    mixed-precision codes and scales, all in STaMP order.  act_quant: "sym" (absmax, signed
    codes) or "asym" (min-max, unsigned codes and integer offsets "zeros")."""
    B, s, d = X.shape
    bits = token_bits(s, k_hi, bits_hi, bits_lo)
    T = np.empty((B, s, d), dtype=dtype)
    asym = act_quant == "asym"
    assert asym or act_quant == "sym"
    codes = np.empty((B, s, d), dtype=np.uint8 if asym else np.int8)
    scales = np.empty((B, s), dtype=dtype)
    zeros = np.zeros((B, s), dtype=dtype)
    for b in range(B):
        T[b] = sequence_forward(X[b], xform, levels, grid_h, grid_w, dtype, skip_first)
        if asym:
            codes[b], scales[b], zeros[b] = quantize_tokens_asym(T[b], bits, dtype)
        else:
            codes[b], scales[b] = quantize_tokens(T[b], bits, dtype)
    out = {"T": T, "codes": codes, "scales": scales, "bits": bits}
    if asym:
        out["zeros"] = zeros
    return out


def linear_from_codes(codes: np.ndarray, scales: np.ndarray, qw: np.ndarray, sw: np.ndarray,
                      xform: str, levels: int, grid_h: int = 0, grid_w: int = 0,
                      bias: Optional[np.ndarray] = None, dtype=np.float32,
                      zeros: Optional[np.ndarray] = None, skip_first: bool = False,
                      bias_mode: str = "after") -> Dict[str, np.ndarray]:
    """Steps 3-5: integer GEMM, dequantization Y' = (float(acc) * scale_m) * sw_n, inverse
    transform per sequence and output column, bias.  With integer offsets `zeros` (asymmetric
    codes) the de-quantization (code - z) * scale of the Background section turns the sum into
    acc[m, n] - z_m * sum_c qw[c, n], an exact integer, before it is scaled.
    bias_mode: "after" adds 1 bias^T to the inverse-transformed output (the algorithm's last step);
    "transformed" adds (L 1) bias^T to the transformed output before the inverse (the third form of the
    commutation identity of section "Method"), with l = L 1 evaluated by the forward transform in `dtype`."""
    B, s, d = codes.shape
    N = qw.shape[1]
    acc = np.empty((B, s, N), dtype=np.int32)
    Yt = np.empty((B, s, N), dtype=dtype)
    Y = np.empty((B, s, N), dtype=dtype)
    sw = np.asarray(sw, dtype=dtype)
    colsum = qw.astype(np.int64).sum(axis=0)
    for b in range(B):
        acc[b] = int_gemm(codes[b], qw)
        a = acc[b].astype(np.int64)
        if zeros is not None:
            zi = np.asarray(zeros[b]).astype(np.int64)
            assert np.array_equal(zi.astype(np.float64), np.asarray(zeros[b], dtype=np.float64))
            a = a - zi[:, None] * colsum[None, :]
        Yt[b] = (a.astype(dtype) * np.asarray(scales[b], dtype=dtype)[:, None]) * sw[None, :]
        yt = Yt[b]
        if bias is not None and bias_mode == "transformed":
            ell = sequence_forward(np.ones((s, 1), dtype=dtype), xform, levels, grid_h, grid_w, dtype, skip_first)
            yt = yt + ell * np.asarray(bias, dtype=dtype)[None, :]
        Y[b] = sequence_inverse(yt, xform, levels, grid_h, grid_w, dtype, skip_first)
    assert bias_mode in ("after", "transformed")
    if bias is not None and bias_mode == "after":
        Y = Y + np.asarray(bias, dtype=dtype)[None, None, :]
    return {"acc": acc, "Yt": Yt, "Y": Y}


def stamp_linear_forward(X: np.ndarray, W: np.ndarray, xform: str, levels: int, k_hi: int,
                         bits_hi: int = 8, bits_lo: int = 4, bits_w: int = 4, grid_h: int = 0,
                         grid_w: int = 0, bias: Optional[np.ndarray] = None,
                         dtype=np.float32, act_quant: str = "sym", skip_first: bool = False,
                         bias_mode: str = "after") -> Dict[str, np.ndarray]:
    """Algorithm "STaMP Linear" end to end for X[batch, s, d_in], W[d_in, d_out]."""
    qa = quantize_activation(X, xform, levels, k_hi, bits_hi, bits_lo, grid_h, grid_w, dtype, act_quant, skip_first)
    qw, sw = quantize_weight(W, bits_w, dtype)
    out = linear_from_codes(qa["codes"], qa["scales"], qw, sw, xform, levels, grid_h, grid_w, bias, dtype,
                            zeros=qa.get("zeros"), skip_first=skip_first, bias_mode=bias_mode)
    out.update(qa)
    out.update({"qw": qw, "sw": sw})
    return out


def sqnr_db(ref: np.ndarray, approx: np.ndarray) -> float:
    """10 log10(||ref||^2 / ||ref - approx||^2) (Experiments, set-up paragraph)."""
    ref = np.asarray(ref, dtype=np.float64)
    err = ref - np.asarray(approx, dtype=np.float64)
    den = float(np.sum(err * err))
    if den == 0.0:
        return math.inf
    return 10.0 * math.log10(float(np.sum(ref * ref)) / den)
