"""Seeded synthetic inputs with the structure the paper attributes to LLM / LVM activations.

The paper evaluates on activations of diffusion transformers and language models whose
autocorrelation along the sequence is close to (block-)Toeplitz (section "Efficient Energy
Concentration"), with a few outlier feature channels (Introduction) and, for language models,
a massive first-token outlier (appendix "Experimental details", LLMs).  None of those models or
datasets is available here, so every input is drawn from a seeded generator with that structure:

* 1-D token streams: a stationary AR(1) process along the tokens, independently per channel,
  ``x_0 = e_0 / sqrt(1 - rho^2)``, ``x_t = rho * x_{t-1} + e_t`` with unit-variance Gaussian
  innovations ``e_t``.
* 2-D image-token grids: a separable AR(1) field over rows and columns with
  ``rho = exp(-1 / corr_len)`` and unit marginal variance.
* A fixed set of outlier channels multiplied by a constant, the same channels for every sequence.
* Optionally the first token of every sequence multiplied by a constant.
* Weights ``W[d_in, d_out]`` are i.i.d. Gaussian with a given standard deviation, drawn from an
  independent stream ``default_rng(seed + 1000)``.  A bias, when requested, is drawn after W
  from that same stream.

Draw order for X (``default_rng(seed)``): the innovations of the whole tensor in one
``standard_normal`` call, then the outlier channel indices (``choice`` without replacement).

bf16 tensors are carried as ``uint16`` bit patterns (numpy has no bf16); the fp32 values are
rounded to bf16 once, round-to-nearest-even, and both consumers read those bits.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    seq_len: int
    d_in: int
    d_out: int
    xform: str            # "haar1d", "haar2d", "wht", "dct" or "identity"
    levels: int
    grid_h: int = 0       # haar2d only; token t = r * grid_w + c
    grid_w: int = 0
    k_hi: int = 64
    bits_hi: int = 8
    bits_lo: int = 4
    bits_w: int = 4
    x_dtype: str = "bf16"  # "bf16" or "f32"
    rho: float = 0.9       # 1-D AR(1) coefficient
    corr_len: float = 8.0  # 2-D correlation length in tokens
    n_outlier_channels: int = 0
    outlier_scale: float = 1.0
    first_token_scale: float = 1.0
    w_std: float = 0.02
    seed: int = 0
    act_quant: str = "sym"   # "sym" (absmax, signed codes) or "asym" (min-max, unsigned codes + offsets)
    mean_shift: float = 0.0   # constant added to every activation (skews the per-token ranges)
    skip_first: bool = False  # the first token is left out of the sequence transform
    bias_mode: str = "after"  # "after" or "transformed"
    group_size: int = 0       # 64: per-block scales

    @property
    def tokens(self) -> int:
        return self.batch * self.seq_len


# The five benchmark configurations, smallest first; cfg5 is the one the benchmark times.
WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", 1, 256, 512, 512, "haar1d", 8, k_hi=8, x_dtype="f32", rho=0.95,
                     n_outlier_channels=4, outlier_scale=20.0, w_std=0.02, seed=0),
    "cfg2": Workload("cfg2", 1, 2048, 4096, 11008, "haar1d", 11, k_hi=64, rho=0.9,
                     n_outlier_channels=41, outlier_scale=50.0, first_token_scale=100.0,
                     w_std=0.02, seed=1),
    "cfg3": Workload("cfg3", 8, 4096, 4096, 4096, "haar1d", 12, k_hi=64, rho=0.9,
                     n_outlier_channels=41, outlier_scale=30.0, w_std=0.02, seed=2),
    "cfg4": Workload("cfg4", 2, 4096, 1152, 4608, "haar2d", 6, grid_h=64, grid_w=64, k_hi=64,
                     corr_len=8.0, n_outlier_channels=6, outlier_scale=40.0, w_std=0.02, seed=3),
    "cfg5": Workload("cfg5", 4, 8192, 8192, 28672, "haar1d", 13, k_hi=128, rho=0.95,
                     n_outlier_channels=82, outlier_scale=50.0, w_std=0.01, seed=4),
}


def get_workload(name: str, **overrides) -> Workload:
    """Look a configuration up by name, optionally overriding fields (e.g. a smaller d_out)."""
    return replace(WORKLOADS[name], **overrides)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _ar1_along_axis1(e: np.ndarray, rho: float, stationary_start: bool, innovation_gain: float) -> None:
    """In place: e[:, t] <- rho * e[:, t-1] + innovation_gain * e[:, t] along axis 1."""
    r = np.float32(rho)
    g = np.float32(innovation_gain)
    if stationary_start:
        e[:, 0] *= np.float32(1.0 / np.sqrt(1.0 - rho * rho))
    for t in range(1, e.shape[1]):
        if innovation_gain != 1.0:
            e[:, t] *= g
        e[:, t] += r * e[:, t - 1]


def make_activation(w: Workload) -> np.ndarray:
    """fp32 activation [batch, seq_len, d_in] (before any cast to the storage dtype)."""
    rng = np.random.default_rng(w.seed)
    x = rng.standard_normal((w.batch, w.seq_len, w.d_in), dtype=np.float32)
    if w.xform == "haar2d":
        rho = float(np.exp(-1.0 / w.corr_len))
        gain = float(np.sqrt(1.0 - rho * rho))
        g = x.reshape(w.batch, w.grid_h, w.grid_w, w.d_in)
        # along rows (axis 1), then along columns (axis 2); unit marginal variance throughout
        _ar1_along_axis1(g, rho, stationary_start=False, innovation_gain=gain)
        gt = g.transpose(0, 2, 1, 3)
        _ar1_along_axis1(gt, rho, stationary_start=False, innovation_gain=gain)
    else:
        _ar1_along_axis1(x, w.rho, stationary_start=True, innovation_gain=1.0)
    if w.n_outlier_channels > 0:
        ch = rng.choice(w.d_in, size=w.n_outlier_channels, replace=False)
        x[:, :, ch] *= np.float32(w.outlier_scale)
    if w.first_token_scale != 1.0:
        x[:, 0, :] *= np.float32(w.first_token_scale)
    if w.mean_shift != 0.0:
        x += np.float32(w.mean_shift)
    return x


def make_weight(w: Workload, with_bias: bool = False) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """fp32 weight W[d_in, d_out] and, optionally, a bias [d_out]."""
    rng = np.random.default_rng(w.seed + 1000)
    W = rng.standard_normal((w.d_in, w.d_out), dtype=np.float32)
    W *= np.float32(w.w_std)
    bias = None
    if with_bias:
        bias = rng.standard_normal((w.d_out,), dtype=np.float32)
    return W, bias


def make_inputs(w: Workload, with_bias: bool = False, need_weight: bool = True) -> dict:
    """All inputs of one workload.

    Returns a dict with
      "X_f32":  fp32 values the method sees (already rounded to bf16 when x_dtype is bf16),
      "X_store": what is uploaded: fp32 array, or uint16 bf16 bit patterns,
      "W": fp32 [d_in, d_out] (None if need_weight is False), "bias": fp32 [d_out] or None.
    """
    x = make_activation(w)
    if w.x_dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        x = bf16_bits_to_f32(bits)
        store = bits
    elif w.x_dtype == "f32":
        store = x
    else:
        raise ValueError(f"unknown x_dtype {w.x_dtype!r}")
    W = bias = None
    if need_weight:
        W, bias = make_weight(w, with_bias)
    return {"X_f32": x, "X_store": store, "W": W, "bias": bias}
