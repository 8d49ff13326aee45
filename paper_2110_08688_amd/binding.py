"""Thin ctypes binding of libmggcn.so: same names as include/mggcn.h, argument marshalling only.

Tensors are PyTorch-ROCm device tensors used purely as device memory; every computation runs
in the library's HIP kernels.  There is no fallback: if the library has not been built the
import of a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmggcn.so")

OK = 0
E_INVALID_ARG, E_BAD_CSR, E_OVERFLOW, E_WORKSPACE, E_HIP, E_UNSUPPORTED, E_NO_MEMORY = -1, -2, -3, -4, -5, -6, -7
NORM_SYM_SELFLOOP, NORM_MEAN_IN = 0, 1
OP_N, OP_T = 0, 1
EPI_NONE, EPI_RELU, EPI_RELU_MASK = 0, 1, 2
ORDER_AUTO, ORDER_GEMM_FIRST, ORDER_SPMM_FIRST = -1, 0, 1
MODEL_CACHE_INPUT, MODEL_GATHER_BF16, MODEL_GEMM_BF16X3 = 1, 2, 4

_vp, _i32, _i64, _sz, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float

# name -> (restype, argtypes); mirrors include/mggcn.h one to one
SIGNATURES = {
    "mggcn_last_error": (C.c_char_p, []),
    "mggcn_version": (C.c_int, []),
    "mggcn_csr_normalize_workspace_bytes": (_sz, [_i32, _i32]),
    "mggcn_csr_normalize_count": (C.c_int, [_i32, _i32, _vp, _vp, C.c_int, _vp, C.POINTER(_i64), _vp, _sz, _vp]),
    "mggcn_csr_normalize": (C.c_int, [_i32, _i32, _vp, _vp, C.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mggcn_csr_normalize_count64": (C.c_int, [_i32, _i32, _vp, _vp, C.c_int, _vp, C.POINTER(_i64), _vp, _sz, _vp]),
    "mggcn_csr_normalize64": (C.c_int, [_i32, _i32, _vp, _vp, C.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mggcn_csr_transpose_workspace_bytes": (_sz, [_i32, _i32, _i64]),
    "mggcn_csr_transpose": (C.c_int, [_i32, _i32, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mggcn_csr_transpose64": (C.c_int, [_i32, _i32, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mggcn_graph_create": (C.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, C.POINTER(_vp)]),
    "mggcn_graph_create64": (C.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, C.POINTER(_vp)]),
    "mggcn_graph_workspace_bytes": (_sz, [_vp, _i32]),
    "mggcn_graph_bind": (C.c_int, [_vp, _i32, _vp, _sz, _vp]),
    "mggcn_graph_destroy": (C.c_int, [_vp]),
    "mggcn_graph_panels": (C.c_int, [_vp, C.c_int, _i32]),
    "mggcn_graph_tune": (C.c_int, [_vp, _i32, _i32]),
    "mggcn_graph_tables": (C.c_int, [_vp, C.c_int, _i32, C.POINTER(_i32), C.POINTER(_i64), C.POINTER(_vp), C.POINTER(_i64),
                                     C.POINTER(_i64), C.POINTER(_vp), C.POINTER(_i64), C.POINTER(_i64)]),
    "mggcn_spmm": (C.c_int, [_vp, C.c_int, _vp, _i64, _i32, _f32, C.c_int, _vp, _i64, _vp]),
    "mggcn_spmm_bf16": (C.c_int, [_vp, C.c_int, _vp, _i64, _i32, _f32, C.c_int, _vp, _i64, _vp]),
    "mggcn_f32_to_bf16": (C.c_int, [_i64, _i32, _vp, _i64, _vp, _i64, _vp]),
    "mggcn_gemm_workspace_bytes": (_sz, [C.c_int, C.c_int, _i64, _i64, _i64]),
    "mggcn_gemm": (C.c_int, [C.c_int, C.c_int, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _f32, C.c_int, _vp, _i64,
                             _vp, _sz, _vp]),
    "mggcn_gemm_bf16x3": (C.c_int, [C.c_int, C.c_int, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _f32, C.c_int, _vp, _i64,
                             _vp, _sz, _vp]),
    "mggcn_relu_bwd": (C.c_int, [_i64, _i32, _vp, _i64, _vp, _i64, _vp]),
    "mggcn_adam_step": (C.c_int, [_i64, _vp, _vp, _vp, _vp, _i32, _f32, _f32, _f32, _f32, _vp]),
    "mggcn_softmax_ce_workspace_bytes": (_sz, [_i64]),
    "mggcn_softmax_ce": (C.c_int, [_i64, _i32, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "mggcn_softmax_ce_static": (C.c_int, [_i64, _i32, _vp, _i64, _vp, _vp, _vp, _i64, _vp]),
    "mggcn_model_create": (C.c_int, [_vp, _i32, _vp, _vp, _i32, C.POINTER(_vp)]),
    "mggcn_model_cache_input": (C.c_int, [_vp, _vp, _i64, _vp]),
    "mggcn_model_destroy": (C.c_int, [_vp]),
    "mggcn_model_spmm_width_max": (_i32, [_vp, _vp, _i32, _i32]),
    "mggcn_model_arena_bytes": (_sz, [_vp]),
    "mggcn_model_bind": (C.c_int, [_vp, _vp, _sz]),
    "mggcn_model_order": (C.c_int, [_vp, _i32]),
    "mggcn_model_activation": (C.c_int, [_vp, _i32, C.POINTER(_vp), C.POINTER(_i64)]),
    "mggcn_model_gather_operand": (C.c_int, [_vp, _i32, C.POINTER(_vp), C.POINTER(_i64)]),
    "mggcn_layer_fwd": (C.c_int, [_vp, _i32, _vp, _i64, _vp, _i64, C.c_int, _vp, _i64, _vp]),
    "mggcn_layer_bwd": (C.c_int, [_vp, _i32, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64,
                                  C.c_int, _vp]),
    "mggcn_probe_sink_floats": (_i32, []),
    "mggcn_probe_read": (C.c_int, [_vp, _i64, _vp, _vp]),
    "mggcn_probe_write": (C.c_int, [_vp, _i64, _f32, _vp]),
    "mggcn_probe_mfma": (_i64, [_i32, _vp, _vp]),
    "mggcn_probe_gather": (C.c_int, [_vp, _i64, _i32, _i64, _vp, _i64, _vp, _vp]),
    "mggcn_epoch": (C.c_int, [_vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp]),
}

_lib = None


class MggcnError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"mggcn error {code}: {message}")
        self.code = code


def lib():
    """Load libmggcn.so (built by `python -m paper_2110_08688_amd.build`); no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2110_08688_amd.build` "
                "(there is no CPU or PyTorch fallback for the HIP path)"
            )
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def last_error() -> str:
    return lib().mggcn_last_error().decode()


def check(rc: int) -> int:
    if rc < 0:
        raise MggcnError(rc, last_error())
    return rc


def ptr(t):
    """Device (or host) address of a tensor / numpy array / None / int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def current_stream():
    import torch

    return torch.cuda.current_stream().cuda_stream


def ld_of(t) -> int:
    """Leading dimension (elements) of a row-major 2-D tensor, possibly a column slice."""
    assert t.dim() == 2
    if t.numel() == 0:
        return max(int(t.shape[1]), 1)
    assert t.shape[1] <= 1 or t.stride(1) == 1, "need unit column stride"
    return max(int(t.stride(0)), int(t.shape[1]), 1) if t.shape[0] > 1 else max(int(t.shape[1]), 1)
