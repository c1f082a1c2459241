"""Argument marshalling shared by the benchmark, the smoke check and the tests: a workload description
(any object with the fields of gen.Workload) -> plan description, and host arrays -> device tensors.
No arithmetic of the method happens here."""
from __future__ import annotations

from .binding import PlanDesc, STAMP_BF16, STAMP_F32

XFORM_CODE = {"identity": 0, "haar1d": 1, "haar2d": 2, "wht": 3, "dct": 4}


def plan_desc_for(w, y_dtype: str = "f32") -> PlanDesc:
    return PlanDesc(batch=w.batch, seq_len=w.seq_len, d_in=w.d_in, d_out=w.d_out, xform=XFORM_CODE[w.xform],
                    levels=w.levels, grid_h=w.grid_h, grid_w=w.grid_w, k_hi=w.k_hi, bits_hi=w.bits_hi,
                    bits_lo=w.bits_lo, bits_w=w.bits_w,
                    x_dtype=STAMP_BF16 if w.x_dtype == "bf16" else STAMP_F32,
                    y_dtype=STAMP_BF16 if y_dtype == "bf16" else STAMP_F32,
                    act_quant=1 if w.act_quant == "asym" else 0,
                    skip_first=int(getattr(w, "skip_first", False)),
                    bias_mode=1 if getattr(w, "bias_mode", "after") == "transformed" else 0,
                    group_size=int(getattr(w, "group_size", 0)))


def to_device_x(inp: dict, w):
    """The stored activation (fp32 array, or uint16 bf16 bit patterns) as a GPU tensor of its dtype."""
    import numpy as np
    import torch
    if w.x_dtype == "bf16":
        return torch.from_numpy(inp["X_store"].view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(inp["X_store"]).cuda()
