"""MI355X (gfx950) STaMP quantized linear layer: thin Python binding over the C-ABI library.

All computation happens in the HIP kernels of libstamp_hip.so; this package only marshals
arguments (torch tensors serve as device memory, torch streams as HIP streams).
"""
from .binding import (  # noqa: F401
    StampError,
    StampPlan,
    PlanDesc,
    lib_path,
    mfma_rate,
    load_library,
    STATUS_NAMES,
    STAMP_F32,
    STAMP_BF16,
    STAMP_L_IDENTITY,
    STAMP_L_HAAR1D,
    STAMP_L_HAAR2D,
    STAMP_L_WHT,
    STAMP_L_DCT,
)
from .marshal import plan_desc_for, to_device_x, XFORM_CODE  # noqa: F401
