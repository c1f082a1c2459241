"""stamp_linear_forward_static (the entry point that allocates nothing: scratch memory in a static device array
of the library) against stamp_linear_forward with a caller workspace, through the C ABI.  Same kernels, same
inputs: the outputs must be bit-identical, and equal to the oracle within the usual bar.  Two calls in a row, the
second on a smaller input, share the array."""
import numpy as np
import pytest

from gen import Workload, make_inputs
from oracle import stamp_oracle as so

import stamp_testlib as tl

pytestmark = pytest.mark.gpu


def _wl(name, **kw):
    base = dict(name=name, batch=1, seq_len=256, d_in=256, d_out=256, xform="haar1d", levels=8, k_hi=8,
                x_dtype="bf16", rho=0.9, n_outlier_channels=3, outlier_scale=30.0, w_std=0.02, seed=11)
    base.update(kw)
    return Workload(**base)


def _run(w, y_dtype):
    import torch
    import paper_2510_26771_amd as st
    inp = make_inputs(w, with_bias=True)
    plan = st.StampPlan(st.plan_desc_for(w, y_dtype), torch.from_numpy(inp["W"]).cuda(), torch.from_numpy(inp["bias"]).cuda())
    assert plan.workspace_bytes() <= st.binding.STAMP_STATIC_SCRATCH_BYTES
    X = st.to_device_x(inp, w)
    ydt = torch.int16 if y_dtype == "bf16" else torch.float32
    Y_ws = torch.zeros((w.batch, w.seq_len, w.d_out), dtype=ydt, device="cuda")
    plan.linear_forward(X, Y_ws, plan.alloc_workspace())
    torch.cuda.synchronize()
    Y = torch.full_like(Y_ws, -1)
    plan.linear_forward_static(X, Y)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_ws), f"{w.name}: static scratch and caller workspace disagree"
    ora = so.stamp_linear_forward(inp["X_f32"], inp["W"], w.xform, w.levels, w.k_hi, grid_h=w.grid_h, grid_w=w.grid_w,
                                  bias=inp["bias"], act_quant=w.act_quant)
    tl.check_output(tl.y_to_numpy(Y, y_dtype == "bf16"), ora["Y"], y_dtype == "bf16", w.name)
    plan.destroy()


def test_static_scratch_two_calls_second_smaller():
    import torch
    assert torch.cuda.is_available()
    # first a larger layer (several row tiles, split channels of the 8-bit rows' GEMM, top levels), then a smaller
    # one on a 2-D grid with the asymmetric quantizer: the second call finds the first call's leftovers in the array
    _run(_wl("static_big", batch=4, seq_len=2048, levels=11, k_hi=64, d_in=1024, d_out=1536, seed=95), "bf16")
    _run(_wl("static_small", batch=1, seq_len=256, xform="haar2d", levels=4, grid_h=16, grid_w=16, k_hi=4, d_in=96,
             d_out=136, corr_len=4.0, seed=96, act_quant="asym", mean_shift=0.4), "f32")
    _run(_wl("static_big", batch=4, seq_len=2048, levels=11, k_hi=64, d_in=1024, d_out=1536, seed=95), "bf16")


def test_static_scratch_refuses_plans_beyond_its_size():
    import torch
    import paper_2510_26771_amd as st
    w = _wl("static_too_big", batch=8, seq_len=4096, levels=12, k_hi=64, d_in=4096, d_out=256, seed=97)
    W = torch.zeros((w.d_in, w.d_out), dtype=torch.float32, device="cuda")
    plan = st.StampPlan(st.plan_desc_for(w, "bf16"), W)
    assert plan.workspace_bytes() > st.binding.STAMP_STATIC_SCRATCH_BYTES
    X = torch.zeros((w.batch, w.seq_len, w.d_in), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((w.batch, w.seq_len, w.d_out), dtype=torch.int16, device="cuda")
    with pytest.raises(st.StampError) as e:
        plan.linear_forward_static(X, Y)
    assert e.value.status == 4
    plan.destroy()
