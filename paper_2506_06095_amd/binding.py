"""ctypes binding of include/smha.h: argument marshalling only.

Function names mirror the C ABI.  torch is used for device memory and streams;
numpy for host index arrays.  Nothing here computes attention.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

from . import build as _build

SMHA_F16, SMHA_BF16, SMHA_F32 = 0, 1, 2
SMHA_KERNEL_AUTO, SMHA_KERNEL_ROW, SMHA_KERNEL_BLOCK = 0, 1, 2
SMHA_SELECTOR_CALIBRATED, SMHA_SELECTOR_PAPER_EQ1 = 0, 1

EXPORTS = {
    "row_ptr": (0, np.int32), "col_idx": (1, np.int32),
    "load_row_ptr": (2, np.int32), "load_col_idx": (3, np.int32),
    "flags": (4, np.uint8), "bitmap": (5, np.uint64),
    "full_row_ptr": (6, np.int32), "full_col_idx": (7, np.int32),
    "part_row_ptr": (8, np.int32), "part_col_idx": (9, np.int32),
    "bitmap_it8": (10, np.uint64),
    "kernel_items": (11, np.int32), "kernel_items_fine": (15, np.int32), "kernel_entries": (12, np.int32),
    "kernel_bitmaps": (13, np.uint64), "kernel_gather_keys": (14, np.int32),
}


class SmhaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {smha_status_string(status)} (status {status})")


class PlanOpts(C.Structure):
    _fields_ = [("block", C.c_int), ("force", C.c_int), ("selector", C.c_int),
                ("build_both", C.c_int), ("device_id", C.c_int), ("head_dim", C.c_int),
                ("no_gather", C.c_int), ("block_form", C.c_int)]


class MaskDesc(C.Structure):
    _fields_ = [("flags", C.c_uint32), ("window_left", C.c_int), ("window_right", C.c_int),
                ("n_global", C.c_int), ("stride", C.c_int), ("stride_phase", C.c_int),
                ("block", C.c_int), ("keep_p", C.c_double), ("n_window_blocks", C.c_int),
                ("n_global_blocks", C.c_int), ("n_random_blocks", C.c_int), ("seed", C.c_uint64),
                ("per_head", C.c_int), ("valid_len", C.POINTER(C.c_int32))]


class PlanInfo(C.Structure):
    _fields_ = [("S", C.c_int), ("Bm", C.c_int), ("Hm", C.c_int), ("block", C.c_int),
                ("kernel", C.c_int), ("has_row_format", C.c_int),
                ("has_block_kernel_lists", C.c_int), ("on_device", C.c_int),
                ("nnz", C.c_int64), ("n_valid", C.c_int64), ("n_full", C.c_int64),
                ("n_part", C.c_int64), ("n_valid16", C.c_int64), ("n_tiles64", C.c_int64), ("n_union", C.c_int64),
                ("n_items", C.c_int64), ("n_split_rows", C.c_int64),
                ("eq1_threshold", C.c_double), ("model_row_us", C.c_double),
                ("model_block_us", C.c_double), ("Sk", C.c_int), ("n_gathered", C.c_int64)]


_lib = None


def library_path() -> str:
    return _build.LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_library(force=True)  # raises if hipcc is missing or the build fails
    lib = C.CDLL(_build.LIB)
    vp = C.c_void_p
    lib.smha_plan_from_dense.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int,
                                         C.POINTER(PlanOpts), C.POINTER(vp)]
    lib.smha_plan_from_dense.restype = C.c_int
    lib.smha_plan_from_dense_rect.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                              C.POINTER(PlanOpts), C.POINTER(vp)]
    lib.smha_plan_from_dense_rect.restype = C.c_int
    lib.smha_plan_from_desc.argtypes = [C.POINTER(MaskDesc), C.c_int, C.c_int, C.c_int,
                                        C.POINTER(PlanOpts), C.POINTER(vp)]
    lib.smha_plan_from_desc.restype = C.c_int
    lib.smha_plan_info.argtypes = [vp, C.POINTER(PlanInfo)]
    lib.smha_plan_info.restype = C.c_int
    lib.smha_plan_export.argtypes = [vp, C.c_int, C.c_int, vp, C.c_size_t, C.POINTER(C.c_size_t)]
    lib.smha_plan_export.restype = C.c_int
    lib.smha_forward.argtypes = [vp, vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                 C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                 C.POINTER(C.c_int64), C.c_float, C.c_int, vp]
    lib.smha_forward.restype = C.c_int
    lib.smha_forward_static.argtypes = lib.smha_forward.argtypes
    lib.smha_forward_static.restype = C.c_int
    lib.smha_plan_prepare.argtypes = [vp, C.c_int, C.c_int, C.c_int]
    lib.smha_plan_prepare.restype = C.c_int
    lib.smha_plan_work_order.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_size_t,
                                         C.POINTER(C.c_size_t), C.POINTER(C.c_int)]
    lib.smha_plan_work_order.restype = C.c_int
    lib.smha_plan_destroy.argtypes = [vp]
    lib.smha_plan_destroy.restype = None
    lib.smha_status_string.argtypes = [C.c_int]
    lib.smha_status_string.restype = C.c_char_p
    lib.smha_kernel_name.argtypes = [vp, C.c_int, C.c_int, C.c_int]
    lib.smha_kernel_name.restype = C.c_char_p
    _lib = lib
    return lib


def smha_status_string(status: int) -> str:
    return _load().smha_status_string(int(status)).decode()


def _opts(block=0, force=SMHA_KERNEL_AUTO, selector=SMHA_SELECTOR_CALIBRATED, build_both=False,
          device_id=-1, head_dim=0, no_gather=False, block_form=0) -> PlanOpts:
    return PlanOpts(int(block), int(force), int(selector), int(bool(build_both)), int(device_id),
                    int(head_dim), int(bool(no_gather)), int(block_form))


def smha_plan_from_dense(mask, **opts) -> int:
    """mask: numpy uint8 [Bm,Hm,S,S] (host) or a torch uint8/bool CUDA tensor (device).
    Returns the plan handle (an integer address)."""
    if mask.ndim != 4 or mask.shape[2] != mask.shape[3]:
        raise ValueError("mask must be [Bm,Hm,S,S]")
    return _plan_from_dense(mask, False, **opts)


def smha_plan_from_dense_rect(mask, **opts) -> int:
    """mask: [Bm,Hm,Sq,Sk], numpy uint8 (host) or a 1-byte torch CUDA tensor (device)."""
    if mask.ndim != 4:
        raise ValueError("mask must be [Bm,Hm,Sq,Sk]")
    return _plan_from_dense(mask, True, **opts)


def _plan_from_dense(mask, rect: bool, **opts) -> int:
    lib = _load()
    if isinstance(mask, np.ndarray):
        if mask.dtype != np.uint8:
            raise ValueError("mask must be uint8")
        m = np.ascontiguousarray(mask)
        ptr, on_dev = m.ctypes.data, 0
    else:  # torch tensor on the GPU
        if mask.element_size() != 1:
            raise ValueError("mask must be a 1-byte tensor")
        m = mask.contiguous()
        ptr, on_dev = m.data_ptr(), (1 if m.is_cuda else 0)
    Bm, Hm, Sq, Sk = m.shape
    out = C.c_void_p()
    o = _opts(**opts)
    if rect:
        st = lib.smha_plan_from_dense_rect(C.c_void_p(ptr), on_dev, Bm, Hm, Sq, Sk, C.byref(o), C.byref(out))
    else:
        st = lib.smha_plan_from_dense(C.c_void_p(ptr), on_dev, Bm, Hm, Sq, C.byref(o), C.byref(out))
    if st != 0:
        raise SmhaError(st, "smha_plan_from_dense_rect" if rect else "smha_plan_from_dense")
    return out.value


def smha_plan_from_desc(spec, B: int, H: int, S: int, **opts) -> int:
    """spec: any object with the fields of smha_mask_desc_t (e.g. workloads.MaskSpec)."""
    lib = _load()
    vl = getattr(spec, "valid_len", None)
    arr = None
    d = MaskDesc(int(spec.flags), int(spec.window_left), int(spec.window_right), int(spec.n_global),
                 int(spec.stride), int(spec.stride_phase), int(spec.block), float(spec.keep_p),
                 int(spec.n_window_blocks), int(spec.n_global_blocks), int(spec.n_random_blocks),
                 int(spec.seed), int(bool(spec.per_head)), None)
    if vl is not None:
        arr = (C.c_int32 * len(vl))(*[int(v) for v in vl])
        d.valid_len = C.cast(arr, C.POINTER(C.c_int32))
    out = C.c_void_p()
    o = _opts(**opts)
    st = lib.smha_plan_from_desc(C.byref(d), B, H, S, C.byref(o), C.byref(out))
    if st != 0:
        raise SmhaError(st, "smha_plan_from_desc")
    return out.value


def smha_plan_info(plan: int) -> dict:
    info = PlanInfo()
    st = _load().smha_plan_info(C.c_void_p(plan), C.byref(info))
    if st != 0:
        raise SmhaError(st, "smha_plan_info")
    return {name: getattr(info, name) for name, _ in PlanInfo._fields_}


def smha_plan_export(plan: int, which: str, mask_index: int = 0) -> np.ndarray:
    code, dtype = EXPORTS[which]
    lib = _load()
    need = C.c_size_t(0)
    st = lib.smha_plan_export(C.c_void_p(plan), mask_index, code, None, 0, C.byref(need))
    if st != 0:
        raise SmhaError(st, "smha_plan_export")
    out = np.empty(need.value // np.dtype(dtype).itemsize, dtype=dtype)
    if need.value:
        st = lib.smha_plan_export(C.c_void_p(plan), mask_index, code, C.c_void_p(out.ctypes.data),
                                  need.value, C.byref(need))
        if st != 0:
            raise SmhaError(st, "smha_plan_export")
    return out


def smha_plan_work_order(plan: int, B: int, H: int, workgroups_per_xcd: int, fine: bool = False):
    """(table, per_xcd): int32 table = 8 list starts, 8 list lengths, then (batch*head, item) pairs."""
    lib = _load()
    need, per = C.c_size_t(0), C.c_int(0)
    st = lib.smha_plan_work_order(C.c_void_p(plan), B, H, workgroups_per_xcd, int(fine), None, 0, C.byref(need),
                                  C.byref(per))
    if st != 0:
        raise SmhaError(st, "smha_plan_work_order")
    out = np.empty(need.value, dtype=np.int32)
    st = lib.smha_plan_work_order(C.c_void_p(plan), B, H, workgroups_per_xcd, int(fine),
                                  C.c_void_p(out.ctypes.data), need.value, C.byref(need), C.byref(per))
    if st != 0:
        raise SmhaError(st, "smha_plan_work_order")
    return out, per.value


def smha_plan_prepare(plan: int, B: int, H: int, d: int) -> None:
    """Make the work order and workspaces for calls with this batch size, head count and head size."""
    st = _load().smha_plan_prepare(C.c_void_p(plan), B, H, d)
    if st != 0:
        raise SmhaError(st, "smha_plan_prepare")


def smha_plan_destroy(plan: Optional[int]) -> None:
    if plan:
        _load().smha_plan_destroy(C.c_void_p(plan))


def smha_kernel_name(plan: int, d: int, in_dtype: int, kernel: int = SMHA_KERNEL_AUTO) -> str:
    return _load().smha_kernel_name(C.c_void_p(plan), d, in_dtype, kernel).decode()


def _strides3(t):
    """NULL (= packed) for a contiguous tensor, else the three leading strides in elements."""
    if t.is_contiguous():
        return None
    st = t.stride()
    if st[3] != 1:
        raise ValueError("head_dim must be contiguous")
    return (C.c_int64 * 3)(st[0], st[1], st[2])


_DTYPE_CODES = None


def _current_raw_stream(torch, device) -> int:
    """The handle of torch's current stream on `device` (the short way when torch offers it)."""
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    if raw is not None and device.index is not None:
        return raw(device.index)
    return torch.cuda.current_stream(device).cuda_stream


def smha_forward_static(plan: int, Q, K, V, O, scale: float = 0.0, kernel: int = SMHA_KERNEL_AUTO,
                        stream=None, _dims=None) -> None:
    """smha_forward through the entry point that allocates nothing (the shape must be prepared)."""
    smha_forward(plan, Q, K, V, O, scale, kernel, stream, _dims, _entry="smha_forward_static")


def smha_forward(plan: int, Q, K, V, O, scale: float = 0.0, kernel: int = SMHA_KERNEL_AUTO,
                 stream=None, _dims=None, _entry="smha_forward") -> None:
    """Q, O: torch CUDA tensors [B,H,S,d]; K, V: [B,H,Sk,d] (S and Sk as in the plan); O in the
    input dtype or float32.  Enqueues on `stream` (default: torch's current stream); does not
    synchronise.  (_dims: the plan's (S, Sk) if the caller already holds them.)"""
    import torch
    global _DTYPE_CODES
    if _DTYPE_CODES is None:
        _DTYPE_CODES = {torch.float16: SMHA_F16, torch.bfloat16: SMHA_BF16, torch.float32: SMHA_F32}
    lib = _load()
    B, H, S, d = Q.shape
    if _dims is None:
        info = PlanInfo()
        st = lib.smha_plan_info(plan, C.byref(info))
        if st != 0:
            raise SmhaError(st, "smha_plan_info")
        _dims = (info.S, info.Sk)
    if O.shape != Q.shape or K.shape != V.shape or K.shape[:2] != Q.shape[:2] or K.shape[3] != d:
        raise ValueError("Q, O must be [B,H,S,d] and K, V [B,H,Sk,d]")
    if S != _dims[0] or K.shape[2] != _dims[1]:
        raise ValueError(f"the plan is for {_dims[0]} queries and {_dims[1]} keys per sequence")
    in_code = _DTYPE_CODES.get(Q.dtype)
    if in_code is None or in_code == SMHA_F32 or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V must be float16 or bfloat16")
    out_code = _DTYPE_CODES.get(O.dtype)
    if out_code is None:
        raise ValueError("O must be float16, bfloat16 or float32")
    if not (Q.is_cuda and K.is_cuda and V.is_cuda and O.is_cuda):
        raise ValueError("tensors must be on the GPU")
    if stream is None:
        handle = _current_raw_stream(torch, Q.device)
    else:
        handle = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    st = getattr(lib, _entry)(plan, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, d,
                              in_code, out_code, _strides3(Q), _strides3(K), _strides3(V), _strides3(O),
                              float(scale), int(kernel), handle)
    if st != 0:
        raise SmhaError(st, _entry)


class Plan:
    """Owns one smha_plan_t handle."""

    def __init__(self, handle: int):
        self.handle = handle
        self._dims = None  # (S, Sk), read from the plan at the first forward

    @classmethod
    def from_dense(cls, mask, **opts) -> "Plan":
        return cls(smha_plan_from_dense(mask, **opts))

    @classmethod
    def from_dense_rect(cls, mask, **opts) -> "Plan":
        return cls(smha_plan_from_dense_rect(mask, **opts))

    @classmethod
    def from_desc(cls, spec, B: int, H: int, S: int, **opts) -> "Plan":
        return cls(smha_plan_from_desc(spec, B, H, S, **opts))

    def info(self) -> dict:
        return smha_plan_info(self.handle)

    def export(self, which: str, mask_index: int = 0) -> np.ndarray:
        return smha_plan_export(self.handle, which, mask_index)

    def work_order(self, B: int, H: int, workgroups_per_xcd: int, fine: bool = False):
        return smha_plan_work_order(self.handle, B, H, workgroups_per_xcd, fine)

    def prepare(self, B: int, H: int, d: int) -> None:
        smha_plan_prepare(self.handle, B, H, d)

    def forward_static(self, Q, K, V, out, scale: float = 0.0, kernel: int = SMHA_KERNEL_AUTO, stream=None):
        if self._dims is None:
            info = self.info()
            self._dims = (info["S"], info["Sk"])
        smha_forward_static(self.handle, Q, K, V, out, scale, kernel, stream, self._dims)
        return out

    def forward(self, Q, K, V, out=None, out_dtype=None, scale: float = 0.0,
                kernel: int = SMHA_KERNEL_AUTO, stream=None):
        import torch
        if out is None:
            out = torch.empty(Q.shape, dtype=out_dtype or Q.dtype, device=Q.device)
        if self._dims is None:
            info = self.info()
            self._dims = (info["S"], info["Sk"])
        smha_forward(self.handle, Q, K, V, out, scale, kernel, stream, self._dims)
        return out

    def close(self) -> None:
        if self.handle:
            smha_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
