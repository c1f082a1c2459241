"""Host-side tests of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2510_26771_amd as st
from paper_2510_26771_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(st.lib_path()):
        from paper_2510_26771_amd.build import build
        build(verbose=False)
    return st.load_library()


def test_header_symbols_are_exported(lib):
    header = open(os.path.join(ROOT, "include", "stamp.h")).read()
    declared = set(re.findall(r"\b(stamp_[a-z_0-9]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    for code in range(7):
        s = lib.stamp_status_string(code)
        assert s and len(s) > 1


def _create(lib, desc, W=1):
    h = C.c_void_p()
    # W is a fake non-null pointer: validation must fail before it is ever dereferenced
    rc = lib.stamp_plan_create(C.byref(desc.to_c()), C.c_void_p(W) if W else None, None, None, C.byref(h))
    assert not h.value
    return rc


def _good(**kw):
    d = dict(batch=1, seq_len=256, d_in=512, d_out=512, xform=st.STAMP_L_HAAR1D, levels=8, k_hi=8,
             x_dtype=st.STAMP_F32, y_dtype=st.STAMP_F32)
    d.update(kw)
    return st.PlanDesc(**d)


@pytest.mark.parametrize("kw,expect", [
    (dict(seq_len=250, levels=9), 2),                         # 250 tokens halve (odd ones carried) 8 times at most
    (dict(seq_len=256, levels=9, skip_first=1), 2),           # 255 tokens after the first: 8 levels exist, 9 do not
    (dict(skip_first=2), 2),
    (dict(xform=st.STAMP_L_HAAR2D, grid_h=16, grid_w=16, levels=3, skip_first=1), 2),   # only the 1-D Haar transform skips
    (dict(xform=st.STAMP_L_WHT, seq_len=250, levels=0), 2),   # Walsh-Hadamard needs a power of two
    (dict(xform=st.STAMP_L_WHT, levels=3), 2),                # WHT and DCT take no level count
    (dict(xform=st.STAMP_L_DCT, levels=1), 2),
    (dict(xform=st.STAMP_L_DCT, levels=0, seq_len=32768), 3), # dense DCT matrix beyond 16384 tokens
    (dict(bias_mode=2), 2),
    (dict(group_size=-64), 2),
    (dict(group_size=32), 3),                                 # blocks of 64 channels only
    (dict(group_size=64, d_in=96), 3),
    (dict(group_size=64, act_quant=1), 3),
    (dict(levels=9), 2),                                      # more levels than log2(seq_len)
    (dict(levels=0), 2),
    (dict(k_hi=257), 2),                                      # k > s
    (dict(k_hi=-1), 2),
    (dict(d_in=511), 2),                                      # odd d_in cannot be packed
    (dict(batch=0), 2),
    (dict(xform=7), 2),
    (dict(bits_hi=9), 2),
    (dict(xform=st.STAMP_L_HAAR2D, grid_h=16, grid_w=8, levels=3), 2),   # grid != seq_len
    (dict(xform=st.STAMP_L_HAAR2D, grid_h=16, grid_w=16, levels=5), 2),  # too many levels
    (dict(bits_lo=3), 3),
    (dict(d_in=48), 3),                                       # d_in not a multiple of 32
    (dict(d_in=32800), 3),                                    # wider than the channel splits go
    (dict(d_out=(1 << 21) + 2), 3),                           # 256 output rows no longer fit 32-bit byte offsets
    (dict(xform=st.STAMP_L_IDENTITY, levels=2), 2),          # no transform has no levels
    (dict(xform=st.STAMP_L_HAAR2D, grid_h=32, grid_w=8, levels=4, k_hi=16), 2),   # more levels than the short side has
    (dict(w_dtype=7), 2),
    # batch and batch * (top rows) are grid dimensions of the transform kernels: beyond 65535 the plan is refused
    (dict(batch=65536, seq_len=64, levels=6, k_hi=8), 3),
    (dict(batch=512, seq_len=1024, levels=10, k_hi=128), 3),
    (dict(xform=st.STAMP_L_IDENTITY, levels=0, batch=512, k_hi=128, seq_len=256), 3),
])
def test_plan_create_rejects_before_any_device_call(lib, kw, expect):
    assert _create(lib, _good(**kw)) == expect


@pytest.mark.parametrize("kw", [
    dict(seq_len=500, levels=3, k_hi=300),                      # more than 256 8-bit tokens
    dict(seq_len=4096, levels=3),                               # 512 approximations: more than the fast path's top part holds
    dict(k_hi=12),                                              # k not a power of two
    dict(k_hi=128),                                             # blocks of 2 tokens
    dict(xform=st.STAMP_L_IDENTITY, levels=0, k_hi=300, seq_len=512),
    dict(xform=st.STAMP_L_HAAR2D, grid_h=16, grid_w=16, levels=4, k_hi=8),    # k not a power of four
    dict(xform=st.STAMP_L_HAAR2D, grid_h=32, grid_w=8, levels=3, k_hi=16),    # rectangular grid
    dict(seq_len=250, levels=8),                                # not a power of two
    dict(w_dtype=st.STAMP_BF16),
])
def test_settings_outside_the_fast_path_are_accepted(lib, kw):
    """Valid STaMP settings without the fast path's block structure are served by the general path: validation
    passes, and without a GPU the first device allocation is what fails."""
    assert _create(lib, _good(**kw)) == 5


def test_null_arguments(lib):
    assert lib.stamp_plan_create(None, None, None, None, None) == 1
    assert _create(lib, _good(), W=0) == 1
    assert lib.stamp_plan_destroy(None) == 1
    assert lib.stamp_plan_workspace_bytes(None) == 0
    assert lib.stamp_plan_row_of_coeff(None, None) == 1
    assert lib.stamp_quantize_act(None, None, None, None, None, None, 0, None) == 1
    assert lib.stamp_linear_forward(None, None, None, None, 0, None) == 1
    assert lib.stamp_linear_forward_static(None, None, None, None) == 1
    assert lib.stamp_linear_forward_q(None, None, None, None, None, None, 0, None) == 1
    assert lib.stamp_inverse(None, None, 1, None, None, 0, None) == 1
    assert lib.stamp_debug_gemm_acc(None, None, None, None, None) == 1
    assert lib.stamp_debug_weight_codes(None, None, None) == 1
    assert lib.stamp_debug_run_stage(None, 0, None, None, None, None, None, None, 0, None) == 1
    assert lib.stamp_plan_set_unfused(None, 1) == 1
    assert lib.stamp_plan_set_gemm_engine(None, 1) == 1
    assert lib.stamp_debug_mfma_rate(0, None) == 1
    assert lib.stamp_debug_mfma_rate(7, None) == 1  # the null check comes first


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.load_library()
