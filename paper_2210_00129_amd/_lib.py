"""ctypes loader of libsbp.so: argument marshalling only.

The library is loaded lazily and must exist: there is no fallback path.  Build it with
``python -m paper_2210_00129_amd.build``.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsbp.so")

c_i32, c_i64, c_u32, c_u64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint64
c_vp, c_sz, c_dbl = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_double


class SampleDesc(ctypes.Structure):
    """Mirror of sbp_sample_desc in include/sbp.h."""
    _fields_ = [("B", c_i32), ("P", c_i32), ("H", c_i32), ("W", c_i32), ("cell", c_i32), ("k", c_i32),
                ("mode", c_i32), ("per_sample", c_i32), ("seed", c_u64), ("stream_id", c_u64)]


class LinearLayer(ctypes.Structure):
    """Mirror of sbp_linear_layer in include/sbp.h."""
    _fields_ = [("dY", c_vp), ("idx", c_vp), ("inv", c_vp), ("X_k", c_vp), ("W", c_vp), ("M", c_i64), ("K", c_i64),
                ("Cin", c_i32), ("Cout", c_i32), ("dW", c_vp), ("db", c_vp), ("dX", c_vp), ("flags", c_u32),
                ("reserved", c_u32)]


class GatherItem(ctypes.Structure):
    """Mirror of sbp_gather_item in include/sbp.h."""
    _fields_ = [("X", c_vp), ("idx", c_vp), ("X_k", c_vp), ("M", c_i64), ("K", c_i64), ("C", c_i32), ("layout", c_i32)]


# name -> (restype, argtypes); every symbol include/sbp.h declares
PROTOTYPES = {
    "sbp_status_string": (ctypes.c_char_p, [c_i32]),
    "sbp_last_error": (ctypes.c_char_p, []),
    "sbp_k_from_ratio": (c_i32, [c_dbl, c_i32]),
    "sbp_keep_count": (c_i64, [ctypes.POINTER(SampleDesc)]),
    "sbp_sample_indices": (c_i32, [ctypes.POINTER(SampleDesc), c_vp, c_i64, c_vp, c_vp]),
    "sbp_sample_indices_batch": (c_i32, [ctypes.POINTER(SampleDesc), c_i32, ctypes.POINTER(c_vp), ctypes.POINTER(c_i64),
                                         ctypes.POINTER(c_vp), c_vp]),
    "sbp_forward_cache": (c_i32, [c_vp, c_vp, c_i64, c_i64, c_i32, c_i32, c_vp, c_vp]),
    "sbp_forward_cache_batch": (c_i32, [ctypes.POINTER(GatherItem), c_i32, c_i32, c_vp]),
    "sbp_backward_linear_workspace": (c_sz, [c_i64, c_i64, c_i32, c_i32, c_i32, c_u32]),
    "sbp_forward_cache_patches": (c_i32, [c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i64, c_i32, c_vp, c_vp]),
    "sbp_scatter_patches_workspace": (c_sz, [c_i32, c_i32, c_i32, c_i32]),
    "sbp_scatter_patches": (c_i32, [c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i64, c_i32, c_vp, c_vp, c_sz, c_vp]),
    "sbp_act_forward_rows": (c_i32, [c_vp, c_i64, c_i32, c_i32, c_i32, c_vp, c_vp]),
    "sbp_act_backward_rows": (c_i32, [c_vp, c_vp, c_i64, c_i32, c_i32, c_i32, c_vp, c_vp]),
    "sbp_backward_layernorm_workspace": (c_sz, [c_i64, c_i64, c_i32, c_i32, c_u32]),
    "sbp_backward_layernorm": (c_i32, [c_vp, c_vp, c_vp, ctypes.c_float, c_vp, c_vp, c_i64, c_i64, c_i32, c_i32,
                                       c_vp, c_vp, c_vp, c_vp, c_sz, c_u32, c_vp]),
    "sbp_backward_layerscale_workspace": (c_sz, [c_i64, c_i32]),
    "sbp_backward_layerscale": (c_i32, [c_vp, c_vp, c_vp, c_i64, c_i32, c_i32, c_vp, c_vp, c_vp, c_sz, c_u32, c_vp]),
    "sbp_backward_attention_engine": (c_i32, [c_i32, c_i32, c_i32]),
    "sbp_backward_attention": (c_i32, [c_vp, c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, ctypes.c_float, c_i32, c_vp, c_vp]),
    "sbp_backward_linear_engine": (c_i32, [c_i64, c_i64, c_i32, c_i32, c_i32, c_u32, ctypes.POINTER(c_i32)]),
    "sbp_backward_linear": (c_i32, [c_vp, c_vp, c_vp, c_vp, c_vp, c_i64, c_i64, c_i32, c_i32, c_i32,
                                    c_vp, c_vp, c_vp, c_vp, c_sz, c_u32, c_vp]),
    "sbp_backward_linear_batch_workspace": (c_sz, [ctypes.POINTER(LinearLayer), c_i32, c_i32]),
    "sbp_backward_linear_batch": (c_i32, [ctypes.POINTER(LinearLayer), c_i32, c_i32, c_vp, c_sz, c_vp]),
    "sbp_static_scratch_bytes": (c_sz, []),
    "sbp_backward_linear_static": (c_i32, [c_vp, c_vp, c_vp, c_vp, c_vp, c_i64, c_i64, c_i32, c_i32, c_i32,
                                           c_vp, c_vp, c_vp, c_u32, c_vp]),
    "sbp_backward_dwconv_workspace": (c_sz, [c_i32, c_i32, c_i32, c_i32, c_i32, c_i64, c_i32, c_u32]),
    "sbp_backward_dwconv": (c_i32, [c_vp, c_vp, c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32,
                                    c_i64, c_i32, c_vp, c_vp, c_vp, c_vp, c_sz, c_u32, c_vp]),
    "sbp_set_option": (c_i32, [ctypes.c_char_p, ctypes.c_char_p]),
    "sbp_profile_enable": (c_i32, [c_i32]),
    "sbp_profile_timeline": (c_i32, [c_vp, c_i64]),
    "sbp_profile_read": (c_i32, [c_i32, ctypes.POINTER(c_dbl), ctypes.POINTER(c_i64)]),
}

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2210_00129_amd.build` "
                "(there is no fallback implementation)")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in PROTOTYPES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


class SbpError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libsbp status {status}: {message}")
        self.status = status


def check(status: int) -> int:
    if status < 0:
        L = lib()
        text = L.sbp_last_error().decode() or L.sbp_status_string(int(status)).decode()
        raise SbpError(int(status), text)
    return status
