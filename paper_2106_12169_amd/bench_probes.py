"""ctypes binding over libapnn_bench.so (include/apnn_bench.h): the measurement probes the benchmark uses.
Argument marshalling only; nothing of the method is computed by these calls."""

from __future__ import annotations

import ctypes as C
import os

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libapnn_bench.so")
EXPORTS = ("apnn_probe_valu", "apnn_probe_copy", "apnn_probe_issue")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2106_12169_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.apnn_probe_valu.argtypes = [C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
        L.apnn_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.apnn_probe_issue.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _check(rc: int, who: str):
    if rc != 0:
        raise RuntimeError(f"{who} failed with status {rc}")


def apnn_probe_valu(blocks: int, iters: int, out: torch.Tensor) -> float:
    """Returns the lane-operation count of the launch."""
    ops = C.c_double(0.0)
    _check(lib().apnn_probe_valu(blocks, iters, out.data_ptr(), C.byref(ops), torch.cuda.current_stream().cuda_stream),
           "apnn_probe_valu")
    return ops.value


def apnn_probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    _check(lib().apnn_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(),
                                 torch.cuda.current_stream().cuda_stream), "apnn_probe_copy")


def apnn_probe_issue(vector_per_matrix: int, with_matrix: bool, waves_per_simd: int, iters: int, out: torch.Tensor) -> None:
    _check(lib().apnn_probe_issue(vector_per_matrix, int(with_matrix), waves_per_simd, iters, out.data_ptr(),
                                  torch.cuda.current_stream().cuda_stream), "apnn_probe_issue")
