"""Thin ctypes binding over libapnn.so: argument marshalling only.

Every function has the name of the C entry point it calls (``include/apnn.h``);
tensors are PyTorch device tensors used purely as device memory, the stream is
PyTorch's current stream.  No computation of the method happens in Python.
The library must have been built (``python -m paper_2106_12169_amd.build``);
a missing library is an error, there is no fallback path.
"""

from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

ENC_UNSIGNED, ENC_PM1 = 0, 1
LAYOUT_NHWC, LAYOUT_NCHW = 0, 1
POOL_NONE, POOL_MAX2, POOL_SUM2 = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libapnn.so")

EXPORTS = (
    "apnn_last_error", "apnn_row_words", "apnn_packed_words", "apnn_fmap_words",
    "apnn_pack", "apnn_pack_fmap", "apnn_pack_conv_weights", "apnn_pack_patches",
    "apnn_pack_patch_weights", "apnn_quantize", "apnn_gemm", "apnn_conv2d", "apnn_layer",
    "apnn_layer_pair", "apnn_input_weight_bytes", "apnn_pack_input_weights", "apnn_input_layer",
    "apnn_fold_bn", "apnn_maxpool", "apnn_sumpool", "apnn_sumpool_fc", "apnn_workspace_bytes",
    "apnn_debug_force", "apnn_debug_reset", "apnn_debug_tile_choice",
)


class ApnnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"apnn status {status}: {text}")
        self.status = status


class ConvDesc(C.Structure):
    _fields_ = [("N", C.c_int64), ("H", C.c_int64), ("W", C.c_int64), ("Cin", C.c_int64), ("Cout", C.c_int64),
                ("R", C.c_int), ("S", C.c_int), ("stride", C.c_int), ("pad", C.c_int),
                ("p", C.c_int), ("q", C.c_int), ("encW", C.c_int), ("encX", C.c_int)]


class LayerDesc(C.Structure):
    _fields_ = [("conv", ConvDesc), ("is_gemm", C.c_int), ("q_out", C.c_int),
                ("scale_dev", C.c_void_p), ("bias_dev", C.c_void_p),
                ("residual_dev", C.c_void_p), ("q_res", C.c_int), ("res_scale", C.c_float),
                ("acc_out_dev", C.c_void_p), ("float_out_dev", C.c_void_p), ("pool", C.c_int)]


_lib = None


def lib():
    """Load libapnn.so (once) and declare the prototypes of include/apnn.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2106_12169_amd.build`")
    L = C.CDLL(LIB_PATH)
    i64, i32, vp, f32 = C.c_int64, C.c_int, C.c_void_p, C.c_float
    L.apnn_last_error.restype = C.c_char_p
    L.apnn_row_words.restype = i64
    L.apnn_row_words.argtypes = [i64]
    L.apnn_packed_words.restype = C.c_size_t
    L.apnn_packed_words.argtypes = [i64, i64, i32]
    L.apnn_fmap_words.restype = C.c_size_t
    L.apnn_fmap_words.argtypes = [i64, i64, i32]
    L.apnn_pack.argtypes = [vp, i64, i64, i32, i32, vp, vp]
    L.apnn_pack_fmap.argtypes = [vp, i32, i64, i64, i64, i64, i32, i32, vp, vp]
    L.apnn_pack_conv_weights.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp]
    L.apnn_pack_patches.argtypes = [vp, i64, i64, i64, i64, i32, i32, i32, i32, i32, vp, vp]
    L.apnn_pack_patch_weights.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp]
    L.apnn_quantize.argtypes = [vp, i64, i64, f32, f32, i32, vp, vp]
    L.apnn_gemm.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, vp]
    L.apnn_conv2d.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp]
    L.apnn_layer.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp]
    L.apnn_layer_pair.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, C.POINTER(LayerDesc), vp, vp, vp, vp]
    L.apnn_input_weight_bytes.restype = C.c_size_t
    L.apnn_input_weight_bytes.argtypes = [i64, i64, i32, i32]
    L.apnn_pack_input_weights.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp]
    L.apnn_input_layer.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp]
    L.apnn_fold_bn.argtypes = [vp, vp, vp, vp, C.c_double, C.c_double, C.c_double, i64, vp, vp]
    L.apnn_maxpool.argtypes = [vp, i64, i64, i64, i64, i32, i32, i32, i32, vp, vp]
    L.apnn_sumpool.argtypes = [vp, i64, i64, i64, i64, i32, i32, vp, vp]
    L.apnn_sumpool_fc.argtypes = [vp, i64, i64, i64, i64, i32, vp, i64, i32, i32, vp, vp]
    L.apnn_workspace_bytes.restype = C.c_size_t
    L.apnn_workspace_bytes.argtypes = [C.POINTER(LayerDesc)]
    L.apnn_debug_force.argtypes = [C.c_char_p, i32]
    L.apnn_debug_reset.restype = None
    L.apnn_debug_reset.argtypes = []
    L.apnn_debug_tile_choice.argtypes = [i64, i64, i32, i32]
    for name in EXPORTS:
        if name not in ("apnn_last_error", "apnn_row_words", "apnn_packed_words", "apnn_fmap_words",
                        "apnn_input_weight_bytes", "apnn_workspace_bytes", "apnn_debug_reset"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        raise ApnnError(status, lib().apnn_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return t.data_ptr()


def _words(n: int, device) -> torch.Tensor:
    # int32 storage for uint32 words; at least one element so data_ptr() is valid
    return torch.empty(max(int(n), 1), dtype=torch.int32, device=device)


def apnn_row_words(K: int) -> int:
    return lib().apnn_row_words(K)


def apnn_packed_words(rows: int, K: int, bits: int) -> int:
    return lib().apnn_packed_words(rows, K, bits)


def apnn_fmap_words(pixels: int, Cc: int, bits: int) -> int:
    return lib().apnn_fmap_words(pixels, Cc, bits)


def apnn_pack(src: torch.Tensor, bits: int, enc: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """src: rows x K uint8/int8 device tensor -> packed matrix operand (int32 words)."""
    rows, K = src.shape
    if out is None:
        out = _words(apnn_packed_words(rows, K, bits), src.device)
    _check(lib().apnn_pack(_ptr(src), rows, K, bits, enc, _ptr(out), _stream()))
    return out


def apnn_pack_fmap(src: torch.Tensor, layout: int, bits: int, enc: int,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if layout == LAYOUT_NHWC:
        N, H, W, Cc = src.shape
    else:
        N, Cc, H, W = src.shape
    if out is None:
        out = _words(apnn_fmap_words(N * H * W, Cc, bits), src.device)
    _check(lib().apnn_pack_fmap(_ptr(src), layout, N, H, W, Cc, bits, enc, _ptr(out), _stream()))
    return out


def apnn_pack_conv_weights(src: torch.Tensor, bits: int, enc: int) -> torch.Tensor:
    Cout, Cin, R, S = src.shape
    out = _words(Cout * bits * R * S * ((Cin + 31) // 32), src.device)
    _check(lib().apnn_pack_conv_weights(_ptr(src), Cout, Cin, R, S, bits, enc, _ptr(out), _stream()))
    return out


def apnn_pack_patches(img: torch.Tensor, R: int, S: int, stride: int, pad: int, bits: int,
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
    N, Cc, H, W = img.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if out is None:
        out = _words(apnn_packed_words(N * Ho * Wo, 32 * R, bits), img.device)
    _check(lib().apnn_pack_patches(_ptr(img), N, Cc, H, W, R, S, stride, pad, bits, _ptr(out), _stream()))
    return out


def apnn_pack_patch_weights(src: torch.Tensor, bits: int, enc: int) -> torch.Tensor:
    Cout, Cin, R, S = src.shape
    out = _words(apnn_packed_words(Cout, 32 * R, bits), src.device)
    _check(lib().apnn_pack_patch_weights(_ptr(src), Cout, Cin, R, S, bits, enc, _ptr(out), _stream()))
    return out


def apnn_quantize(src: torch.Tensor, zero: float, step: float, bits: int,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    rows, K = src.shape
    assert src.dtype == torch.float32
    if out is None:
        out = _words(apnn_packed_words(rows, K, bits), src.device)
    _check(lib().apnn_quantize(_ptr(src), rows, K, zero, step, bits, _ptr(out), _stream()))
    return out


def apnn_gemm(W: torch.Tensor, X: torch.Tensor, M: int, N: int, K: int, p: int, q: int,
              encW: int, encX: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=W.device)
    _check(lib().apnn_gemm(_ptr(W), _ptr(X), _ptr(out) if out.numel() else None, M, N, K, p, q, encW, encX, _stream()))
    return out


@dataclass
class Conv:
    """Plain description of a convolution (or, with is_gemm, a matrix layer)."""
    N: int
    H: int
    W: int
    Cin: int
    Cout: int
    R: int = 1
    S: int = 1
    stride: int = 1
    pad: int = 0
    p: int = 1
    q: int = 2
    encW: int = ENC_PM1
    encX: int = ENC_UNSIGNED

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def c(self) -> ConvDesc:
        return ConvDesc(self.N, self.H, self.W, self.Cin, self.Cout, self.R, self.S, self.stride, self.pad,
                        self.p, self.q, self.encW, self.encX)


def apnn_conv2d(d: Conv, W: torch.Tensor, X: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty((d.N, d.Ho, d.Wo, d.Cout), dtype=torch.int32, device=X.device)
    desc = d.c()
    _check(lib().apnn_conv2d(C.byref(desc), _ptr(W), _ptr(X), _ptr(out), _stream()))
    return out


def apnn_layer(d: Conv, W: torch.Tensor, X: torch.Tensor, *, is_gemm: bool = False, q_out: int = 0,
               scale: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None,
               residual: Optional[torch.Tensor] = None, q_res: int = 0, res_scale: float = 0.0,
               acc_out: Optional[torch.Tensor] = None, float_out: Optional[torch.Tensor] = None,
               out: Optional[torch.Tensor] = None, pool: int = 0) -> Optional[torch.Tensor]:
    """Returns the packed output codes (or None when q_out == 0).  pool: POOL_NONE / POOL_MAX2 / POOL_SUM2."""
    pixels = d.N * (1 if is_gemm else ((d.Ho // 2) * (d.Wo // 2) if pool else d.Ho * d.Wo))
    if q_out > 0 and out is None:
        out = _words(apnn_fmap_words(pixels, d.Cout, q_out), X.device)
    L = LayerDesc(d.c(), int(is_gemm), q_out, _ptr(scale), _ptr(bias), _ptr(residual), q_res, res_scale,
                  _ptr(acc_out), _ptr(float_out), pool)
    _check(lib().apnn_layer(C.byref(L), _ptr(W), _ptr(X), _ptr(out) if q_out > 0 else None, _stream()))
    return out if q_out > 0 else None


def apnn_layer_pair(a: dict, b: dict) -> None:
    """Two independent layers, one launch where the library can share it.  a, b: the arguments of apnn_layer as
    dicts with keys d, W, X and optionally q_out, scale, bias, residual, q_res, res_scale, acc_out, float_out, out,
    pool; packed outputs must be preallocated (out)."""
    def desc(k):
        q_out = k.get("q_out", 0)
        assert q_out == 0 or k.get("out") is not None, "preallocate the packed output"
        L = LayerDesc(k["d"].c(), 0, q_out, _ptr(k.get("scale")), _ptr(k.get("bias")), _ptr(k.get("residual")),
                      k.get("q_res", 0), k.get("res_scale", 0.0), _ptr(k.get("acc_out")), _ptr(k.get("float_out")),
                      k.get("pool", 0))
        return L, _ptr(k["W"]), _ptr(k["X"]), (_ptr(k["out"]) if q_out > 0 else None)
    La, Wa, Xa, Oa = desc(a)
    Lb, Wb, Xb, Ob = desc(b)
    _check(lib().apnn_layer_pair(C.byref(La), Wa, Xa, Oa, C.byref(Lb), Wb, Xb, Ob, _stream()))


def apnn_pack_input_weights(src: torch.Tensor, bits: int, enc: int) -> torch.Tensor:
    """src: Cout x Cin x R x S values, one per byte -> the input layer's signed-byte weight rows."""
    Cout, Cin, R, S = src.shape
    out = torch.empty(max(lib().apnn_input_weight_bytes(Cout, Cin, R, S), 16), dtype=torch.uint8, device=src.device)
    _check(lib().apnn_pack_input_weights(_ptr(src), Cout, Cin, R, S, bits, enc, _ptr(out), _stream()))
    return out


def apnn_input_layer(d: Conv, W: torch.Tensor, image: torch.Tensor, *, q_out: int = 0,
                     scale: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None,
                     residual: Optional[torch.Tensor] = None, q_res: int = 0, res_scale: float = 0.0,
                     acc_out: Optional[torch.Tensor] = None, float_out: Optional[torch.Tensor] = None,
                     out: Optional[torch.Tensor] = None) -> Optional[torch.Tensor]:
    """Convolution of the N x Cin x H x W uint8 image with weights from apnn_pack_input_weights, fused epilogue
    as in apnn_layer.  Returns the packed output codes (or None when q_out == 0)."""
    if q_out > 0 and out is None:
        out = _words(apnn_fmap_words(d.N * d.Ho * d.Wo, d.Cout, q_out), image.device)
    L = LayerDesc(d.c(), 0, q_out, _ptr(scale), _ptr(bias), _ptr(residual), q_res, res_scale,
                  _ptr(acc_out), _ptr(float_out), 0)
    _check(lib().apnn_input_layer(C.byref(L), _ptr(W), _ptr(image), _ptr(out) if q_out > 0 else None, _stream()))
    return out if q_out > 0 else None


def apnn_maxpool(X: torch.Tensor, N: int, H: int, W: int, Cc: int, bits: int, k: int, stride: int, pad: int,
                 out: Optional[torch.Tensor] = None) -> torch.Tensor:
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    if out is None:
        out = _words(apnn_fmap_words(N * Ho * Wo, Cc, bits), X.device)
    _check(lib().apnn_maxpool(_ptr(X), N, H, W, Cc, bits, k, stride, pad, _ptr(out), _stream()))
    return out


def apnn_sumpool(X: torch.Tensor, N: int, H: int, W: int, Cc: int, bits: int, out_bits: int,
                 out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = _words(apnn_packed_words(N, Cc, out_bits), X.device)
    _check(lib().apnn_sumpool(_ptr(X), N, H, W, Cc, bits, out_bits, _ptr(out), _stream()))
    return out


def apnn_sumpool_fc(X: torch.Tensor, N: int, H: int, W: int, Cc: int, bits: int, Wp: torch.Tensor, Cout: int, p: int,
                    encW: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Global sum pooling + fully connected layer in one launch -> int32 [N][Cout]."""
    if out is None:
        out = torch.empty((N, Cout), dtype=torch.int32, device=X.device)
    _check(lib().apnn_sumpool_fc(_ptr(X), N, H, W, Cc, bits, _ptr(Wp), Cout, p, encW, _ptr(out), _stream()))
    return out


def apnn_fold_bn(gamma, beta, mean, var, eps: float, zero: float, step: float):
    """Host helper: numpy float64 arrays in, fp32 numpy (scale, bias) out."""
    import numpy as np
    g, b, m, v = (np.ascontiguousarray(a, np.float64) for a in (gamma, beta, mean, var))
    scale, bias = np.empty(g.shape, np.float32), np.empty(g.shape, np.float32)
    _check(lib().apnn_fold_bn(g.ctypes.data, b.ctypes.data, m.ctypes.data, v.ctypes.data, eps, zero, step,
                              g.size, scale.ctypes.data, bias.ctypes.data))
    return scale, bias


def apnn_workspace_bytes(d: Conv, *, is_gemm: bool = False, q_out: int = 0, pool: int = 0) -> int:
    L = LayerDesc(d.c(), int(is_gemm), q_out, None, None, None, 0, 0.0, None, None, pool)
    return lib().apnn_workspace_bytes(C.byref(L))


def apnn_debug_force(name: str, value: int) -> None:
    """Force a kernel choice (include/apnn_debug.h); value < 0 clears it."""
    _check(lib().apnn_debug_force(name.encode(), int(value)))


def apnn_debug_reset() -> None:
    lib().apnn_debug_reset()


def apnn_debug_tile_choice(M: int, N: int, is_conv: bool = False, matrix_form: bool = True) -> int:
    """Block tile edge the dispatch would take for an M x N output (Sec. 4.3 heuristic); host only."""
    return lib().apnn_debug_tile_choice(int(M), int(N), int(is_conv), int(matrix_form))
