"""ctypes binding of include/stamp.h.  Same entry-point names as the C ABI, argument marshalling only.

There is no CPU fallback: if libstamp_hip.so has not been built (python -m paper_2510_26771_amd.build)
loading raises, and every compute call needs CUDA/HIP tensors.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libstamp_hip.so"

STAMP_F32, STAMP_BF16 = 0, 1
STAMP_L_IDENTITY, STAMP_L_HAAR1D, STAMP_L_HAAR2D, STAMP_L_WHT, STAMP_L_DCT = 0, 1, 2, 3, 4
STAMP_STATIC_SCRATCH_BYTES = 64 << 20  # include/stamp.h
STATUS_NAMES = {0: "STAMP_OK", 1: "STAMP_ERR_NULL", 2: "STAMP_ERR_SHAPE", 3: "STAMP_ERR_UNSUPPORTED",
                4: "STAMP_ERR_WORKSPACE", 5: "STAMP_ERR_ALLOC", 6: "STAMP_ERR_DEVICE"}

# every symbol include/stamp.h declares
EXPORTS = ["stamp_plan_create", "stamp_plan_destroy", "stamp_plan_workspace_bytes", "stamp_plan_hi_rows",
           "stamp_plan_row_of_coeff",
           "stamp_quantize_act", "stamp_linear_forward", "stamp_linear_forward_static", "stamp_linear_forward_q", "stamp_inverse",
           "stamp_debug_gemm_acc", "stamp_debug_weight_codes", "stamp_debug_run_stage", "stamp_plan_set_unfused", "stamp_plan_set_gemm_engine",
           "stamp_debug_mfma_rate", "stamp_status_string"]


class StampError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}")


class _Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "seq_len", "d_in", "d_out", "xform", "levels", "grid_h", "grid_w", "k_hi", "bits_hi", "bits_lo",
        "bits_w", "x_dtype", "y_dtype", "w_dtype", "w_is_out_by_in", "act_quant", "skip_first", "bias_mode", "group_size")]


@dataclass
class PlanDesc:
    batch: int
    seq_len: int
    d_in: int
    d_out: int
    xform: int = STAMP_L_HAAR1D
    levels: int = 0
    grid_h: int = 0
    grid_w: int = 0
    k_hi: int = 64
    bits_hi: int = 8
    bits_lo: int = 4
    bits_w: int = 4
    x_dtype: int = STAMP_BF16
    y_dtype: int = STAMP_BF16
    w_dtype: int = STAMP_F32
    w_is_out_by_in: int = 0
    act_quant: int = 0  # 0 symmetric absmax, 1 asymmetric min-max
    skip_first: int = 0  # 1: the first token is left out of the transform (HAAR1D)
    bias_mode: int = 0   # 1: transformed bias (L 1) bias^T added before the inverse
    group_size: int = 0  # 64: per-block scales

    def to_c(self) -> _Desc:
        return _Desc(**{n: int(getattr(self, n)) for n, _ in _Desc._fields_})


_lib = None


def lib_path() -> str:
    """The in-tree library; STAMP_LIB_PATH names another build of it (kernel variants under measurement)."""
    return os.environ.get("STAMP_LIB_PATH") or os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load libstamp_hip.so (built in-tree).  Raises if it is missing: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_2510_26771_amd.build` "
                           "(the STaMP path has no CPU or PyTorch fallback)")
    # PyTorch supplies the device memory this library works on, so both must talk to ONE HIP runtime: PyTorch's.
    # The dynamic loader binds this library's HIP dependency to whichever runtime the process loaded first; loaded
    # before torch, it would bring in the system's runtime next to torch's own, and allocations then fail.
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.stamp_plan_create.argtypes = [C.POINTER(_Desc), vp, vp, vp, C.POINTER(vp)]
    lib.stamp_plan_create.restype = C.c_int
    lib.stamp_plan_destroy.argtypes = [vp]
    lib.stamp_plan_destroy.restype = C.c_int
    lib.stamp_plan_workspace_bytes.argtypes = [vp]
    lib.stamp_plan_workspace_bytes.restype = sz
    lib.stamp_plan_hi_rows.argtypes = [vp]
    lib.stamp_plan_hi_rows.restype = i32
    lib.stamp_plan_row_of_coeff.argtypes = [vp, C.POINTER(i32)]
    lib.stamp_plan_row_of_coeff.restype = C.c_int
    lib.stamp_quantize_act.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stamp_quantize_act.restype = C.c_int
    lib.stamp_linear_forward.argtypes = [vp, vp, vp, vp, sz, vp]
    lib.stamp_linear_forward.restype = C.c_int
    lib.stamp_linear_forward_static.argtypes = [vp, vp, vp, vp]
    lib.stamp_linear_forward_static.restype = C.c_int
    lib.stamp_linear_forward_q.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stamp_linear_forward_q.restype = C.c_int
    lib.stamp_inverse.argtypes = [vp, vp, i32, vp, vp, sz, vp]
    lib.stamp_inverse.restype = C.c_int
    lib.stamp_debug_gemm_acc.argtypes = [vp, vp, vp, vp, vp]
    lib.stamp_debug_gemm_acc.restype = C.c_int
    lib.stamp_debug_weight_codes.argtypes = [vp, vp, vp]
    lib.stamp_debug_weight_codes.restype = C.c_int
    lib.stamp_debug_run_stage.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stamp_debug_run_stage.restype = C.c_int
    lib.stamp_plan_set_unfused.argtypes = [vp, i32]
    lib.stamp_plan_set_unfused.restype = C.c_int
    lib.stamp_plan_set_gemm_engine.argtypes = [vp, i32]
    lib.stamp_plan_set_gemm_engine.restype = C.c_int
    lib.stamp_debug_mfma_rate.argtypes = [i32, C.POINTER(C.c_double)]
    lib.stamp_debug_mfma_rate.restype = C.c_int
    lib.stamp_status_string.argtypes = [C.c_int]
    lib.stamp_status_string.restype = C.c_char_p
    _lib = lib
    return lib


def _check(status: int, where: str):
    if status != 0:
        raise StampError(status, where)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream or None


def mfma_rate(engine) -> float:
    """Sustained rate (1e12 op/s) of the matrix pipeline of `engine` ("int8" / "fp6") on random 4-bit codes, no memory traffic."""
    lib = load_library()
    code = {"int8": 0, "fp6": 1}[engine] if isinstance(engine, str) else int(engine)
    out = C.c_double(0.0)
    _check(lib.stamp_debug_mfma_rate(code, C.byref(out)), "stamp_debug_mfma_rate")
    return out.value


class StampPlan:
    """Owns a stamp_plan_t.  Methods mirror the C entry points; tensors must live on the GPU."""

    def __init__(self, desc: PlanDesc, W, bias=None, stream=None):
        self.lib = load_library()
        self.desc = desc
        self._h = C.c_void_p()
        if W is not None and not W.is_cuda:
            raise ValueError("W must be a GPU tensor: the library has no host path")
        _check(self.lib.stamp_plan_create(C.byref(desc.to_c()), _ptr(W), _ptr(bias), _stream(stream), C.byref(self._h)),
               "stamp_plan_create")

    # -- lifetime --
    def destroy(self):
        if self._h:
            self.lib.stamp_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- queries --
    def workspace_bytes(self) -> int:
        return int(self.lib.stamp_plan_workspace_bytes(self._h))

    def hi_rows(self) -> int:
        """Rows per sequence of the q_hi buffer (k_hi, or the number of approximations if that is larger)."""
        return int(self.lib.stamp_plan_hi_rows(self._h))

    def row_of_coeff(self):
        import numpy as np
        out = np.empty(self.desc.seq_len, dtype=np.int32)
        _check(self.lib.stamp_plan_row_of_coeff(self._h, out.ctypes.data_as(C.POINTER(C.c_int32))), "stamp_plan_row_of_coeff")
        return out

    def set_gemm_engine(self, engine):
        """engine: "fp6" (default) or "int8": the matrix pipeline that multiplies the 4-bit rows."""
        code = {"int8": 0, "fp6": 1}[engine] if isinstance(engine, str) else int(engine)
        _check(self.lib.stamp_plan_set_gemm_engine(self._h, code), "stamp_plan_set_gemm_engine")

    def set_unfused(self, unfused: bool):
        _check(self.lib.stamp_plan_set_unfused(self._h, int(bool(unfused))), "stamp_plan_set_unfused")

    def alloc_workspace(self, device="cuda"):
        import torch
        return torch.empty(max(self.workspace_bytes(), 256), dtype=torch.uint8, device=device)

    # -- compute (asynchronous on the stream) --
    def quantize_act(self, X, q_hi, q_lo, scales, workspace, stream=None):
        _check(self.lib.stamp_quantize_act(self._h, _ptr(X), _ptr(q_hi), _ptr(q_lo), _ptr(scales), _ptr(workspace),
                                           workspace.numel(), _stream(stream)), "stamp_quantize_act")

    def linear_forward(self, X, Y, workspace, stream=None):
        _check(self.lib.stamp_linear_forward(self._h, _ptr(X), _ptr(Y), _ptr(workspace), workspace.numel(),
                                             _stream(stream)), "stamp_linear_forward")

    def linear_forward_static(self, X, Y, stream=None):
        """stamp_linear_forward on the library's static scratch array (no workspace, no allocation)."""
        _check(self.lib.stamp_linear_forward_static(self._h, _ptr(X), _ptr(Y), _stream(stream)),
               "stamp_linear_forward_static")

    def linear_forward_q(self, q_hi, q_lo, scales, Y, workspace, stream=None):
        _check(self.lib.stamp_linear_forward_q(self._h, _ptr(q_hi), _ptr(q_lo), _ptr(scales), _ptr(Y), _ptr(workspace),
                                               workspace.numel(), _stream(stream)), "stamp_linear_forward_q")

    def inverse(self, Yt, n_cols, Y, workspace, stream=None):
        _check(self.lib.stamp_inverse(self._h, _ptr(Yt), int(n_cols), _ptr(Y), _ptr(workspace), workspace.numel(),
                                      _stream(stream)), "stamp_inverse")

    def debug_gemm_acc(self, q_hi, q_lo, acc, stream=None):
        _check(self.lib.stamp_debug_gemm_acc(self._h, _ptr(q_hi), _ptr(q_lo), _ptr(acc), _stream(stream)),
               "stamp_debug_gemm_acc")

    def debug_run_stage(self, stage, X, q_hi, q_lo, scales, Y, workspace, stream=None):
        _check(self.lib.stamp_debug_run_stage(self._h, int(stage), _ptr(X), _ptr(q_hi), _ptr(q_lo), _ptr(scales),
                                              _ptr(Y), _ptr(workspace), workspace.numel(), _stream(stream)),
               "stamp_debug_run_stage")

    def debug_weight_codes(self):
        import numpy as np
        qw = np.empty((self.desc.d_in, self.desc.d_out), dtype=np.int8)
        # per-block scales: one per block of input channels and output column
        sw = np.empty((self.desc.d_in // self.desc.group_size, self.desc.d_out) if self.desc.group_size
                      else self.desc.d_out, dtype=np.float32)
        _check(self.lib.stamp_debug_weight_codes(self._h, qw.ctypes.data, sw.ctypes.data), "stamp_debug_weight_codes")
        return qw, sw

    # -- convenience allocators for the activation buffers (layouts of include/stamp.h) --
    def alloc_act_buffers(self, device="cuda"):
        import torch
        d = self.desc
        # at least one row, so that the pointer is valid when a plan keeps no 8-bit token at all
        q_hi = torch.empty((d.batch, max(self.hi_rows(), 1), d.d_in), dtype=torch.int8, device=device)
        if d.group_size:
            # per-block scales: q_hi holds every token's codes, q_lo is not used
            return (q_hi, torch.zeros(16, dtype=torch.uint8, device=device),
                    torch.zeros((d.batch, d.seq_len, d.d_in // d.group_size), dtype=torch.float32, device=device))
        mp = -(-(d.batch * d.seq_len) // 256) * 256
        kp = -(-d.d_in // 128) * 128
        q_lo = torch.zeros(mp * kp // 2, dtype=torch.uint8, device=device)  # tiled, see include/stamp.h
        # asymmetric plans: [2][batch, seq_len] = scales, then the integer offsets
        shape = (2, d.batch, d.seq_len) if d.act_quant else (d.batch, d.seq_len)
        scales = torch.zeros(shape, dtype=torch.float32, device=device)
        return q_hi, q_lo, scales
