"""smha: masked multi-head attention for MI355X (gfx950) behind a C ABI.

The compute lives in libsmha.so (HIP); this package is the thin ctypes binding
(`binding`) and the in-tree build step (`build`).  There is no CPU fallback: if
the library is missing or no GPU is usable, calls raise.
"""
from .binding import (  # noqa: F401
    SMHA_BF16, SMHA_F16, SMHA_F32, SMHA_KERNEL_AUTO, SMHA_KERNEL_BLOCK, SMHA_KERNEL_ROW,
    SMHA_SELECTOR_CALIBRATED, SMHA_SELECTOR_PAPER_EQ1, Plan, SmhaError, library_path,
    smha_forward, smha_forward_static, smha_kernel_name, smha_plan_destroy, smha_plan_export, smha_plan_from_dense,
    smha_plan_from_dense_rect,
    smha_plan_from_desc, smha_plan_info, smha_plan_prepare, smha_plan_work_order, smha_status_string)
