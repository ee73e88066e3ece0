"""ctypes binding of libflatquant.so: argument marshalling only.

Functions have the names of the C entry points (see include/flatquant.h).  They
accept raw device addresses (ints) or objects with ``data_ptr()`` (torch
tensors); nothing is computed in Python.  There is no fallback: if the shared
library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libflatquant.so")

FQ_OK, FQ_INVALID_ARG, FQ_UNSUPPORTED_SHAPE, FQ_MISALIGNED, FQ_LAUNCH_FAILED = range(5)

EXPORTS = (
    "flatquant_transform_quant", "flatquant_kv_transform_quant", "flatquant_kv_transform_quant_bits",
    "flatquant_dequant", "flatquant_dequant_bits", "flatquant_stream_probe", "flatquant_transform_mxfp4", "flatquant_transform_mxfp4_tiled", "fq_mxfp4_tiled_scale_bytes",
    "flatquant_dequant_mxfp4", "flatquant_mxfp4_gemm",
    "flatquant_weight_transform_quant", "fq_inverse_transpose", "flatquant_head_transform", "flatquant_w4a4_gemm",
    "fq_supported", "fq_choose_factors", "fq_default_design_fits", "fq_lds_bytes",
    "fq_status_string", "fq_last_hip_error", "fq_abi_version", "fq_set_tuning",
)

_lib = None


class FlatQuantError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status}, hip error {last_hip_error()})")


def lib() -> ctypes.CDLL:
    """Load the shared library once.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_09426_amd.build` "
                "(there is no CPU fallback for the FlatQuant kernels)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float
        L.flatquant_transform_quant.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i64, vp, vp, vp]
        L.flatquant_transform_quant.restype = i32
        L.flatquant_transform_mxfp4.argtypes = L.flatquant_transform_quant.argtypes
        L.flatquant_transform_mxfp4.restype = i32
        L.flatquant_transform_mxfp4_tiled.argtypes = L.flatquant_transform_quant.argtypes
        L.flatquant_transform_mxfp4_tiled.restype = i32
        L.fq_mxfp4_tiled_scale_bytes.argtypes = [i64, i64]
        L.fq_mxfp4_tiled_scale_bytes.restype = i64
        L.flatquant_mxfp4_gemm.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, i64, vp]
        L.flatquant_mxfp4_gemm.restype = i32
        L.flatquant_dequant_mxfp4.argtypes = [vp, vp, i64, i32, vp, vp]
        L.flatquant_dequant_mxfp4.restype = i32
        L.flatquant_kv_transform_quant.argtypes = [vp, vp, i32, f32, i64, i32, i32, vp, vp, vp, vp]
        L.flatquant_kv_transform_quant.restype = i32
        L.flatquant_dequant.argtypes = [vp, vp, vp, i64, i32, vp, vp]
        L.flatquant_dequant.restype = i32
        L.flatquant_kv_transform_quant_bits.argtypes = [vp, vp, i32, f32, i32, i64, i32, i32, vp, vp, vp, vp]
        L.flatquant_kv_transform_quant_bits.restype = i32
        L.flatquant_dequant_bits.argtypes = [vp, vp, vp, i64, i32, i32, vp, vp]
        L.flatquant_dequant_bits.restype = i32
        L.flatquant_weight_transform_quant.argtypes = L.flatquant_transform_quant.argtypes
        L.flatquant_weight_transform_quant.restype = i32
        L.flatquant_w4a4_gemm.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, i64, vp]
        L.flatquant_w4a4_gemm.restype = i32
        L.flatquant_head_transform.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp]
        L.flatquant_head_transform.restype = i32
        L.fq_inverse_transpose.argtypes = [vp, i32, vp, ctypes.POINTER(ctypes.c_double)]
        L.fq_inverse_transpose.restype = i32
        L.flatquant_stream_probe.argtypes = [vp, i64, i32, i64, vp, vp]
        L.flatquant_stream_probe.restype = i32
        L.fq_supported.argtypes = [i32, i32]
        L.fq_supported.restype = i32
        L.fq_choose_factors.argtypes = [i64, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.fq_choose_factors.restype = i32
        L.fq_default_design_fits.argtypes = [i32, i32, i64]
        L.fq_default_design_fits.restype = i32
        L.fq_lds_bytes.argtypes = [i32, i32]
        L.fq_lds_bytes.restype = i64
        L.fq_status_string.argtypes = [i32]
        L.fq_status_string.restype = ctypes.c_char_p
        L.fq_last_hip_error.argtypes = []
        L.fq_last_hip_error.restype = i32
        L.fq_set_tuning.argtypes = [ctypes.c_char_p, i32, i32]
        L.fq_set_tuning.restype = i32
        L.fq_abi_version.argtypes = []
        L.fq_abi_version.restype = i32
        _lib = L
    return _lib


def _ptr(obj) -> Optional[int]:
    if obj is None:
        return None
    if isinstance(obj, int):
        return obj
    return int(obj.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None      # torch.cuda.Stream


def status_string(status: int) -> str:
    return lib().fq_status_string(int(status)).decode()


def last_hip_error() -> int:
    return int(lib().fq_last_hip_error())


def flatquant_transform_quant(x, P1, P2, clip, clip_mode: int, T: int, n1: int, n2: int, x_stride: int,
                              out_codes, out_scales, stream=None, check: bool = True) -> int:
    st = lib().flatquant_transform_quant(_ptr(x), _ptr(P1), _ptr(P2), _ptr(clip), int(clip_mode), int(T), int(n1),
                                         int(n2), int(x_stride), _ptr(out_codes), _ptr(out_scales), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_transform_quant")
    return st


def flatquant_kv_transform_quant(kv, P, Hp: int, clip: float, T: int, H: int, D: int, out_codes, out_scales, out_zeros,
                                 stream=None, check: bool = True) -> int:
    st = lib().flatquant_kv_transform_quant(_ptr(kv), _ptr(P), int(Hp), float(clip), int(T), int(H), int(D),
                                            _ptr(out_codes), _ptr(out_scales), _ptr(out_zeros), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_kv_transform_quant")
    return st


def flatquant_transform_mxfp4(x, P1, P2, clip, clip_mode: int, T: int, n1: int, n2: int, x_stride: int, out_codes, out_scales,
                              stream=None, check: bool = True) -> int:
    st = lib().flatquant_transform_mxfp4(_ptr(x), _ptr(P1), _ptr(P2), _ptr(clip), int(clip_mode), int(T), int(n1), int(n2),
                                         int(x_stride), _ptr(out_codes), _ptr(out_scales), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_transform_mxfp4")
    return st


def flatquant_transform_mxfp4_tiled(x, P1, P2, clip, clip_mode: int, T: int, n1: int, n2: int, x_stride: int, out_codes,
                                    out_scales, stream=None, check: bool = True) -> int:
    st = lib().flatquant_transform_mxfp4_tiled(_ptr(x), _ptr(P1), _ptr(P2), _ptr(clip), int(clip_mode), int(T), int(n1), int(n2),
                                               int(x_stride), _ptr(out_codes), _ptr(out_scales), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_transform_mxfp4_tiled")
    return st


def fq_mxfp4_tiled_scale_bytes(rows: int, n: int) -> int:
    return int(lib().fq_mxfp4_tiled_scale_bytes(int(rows), int(n)))


def flatquant_mxfp4_gemm(x_codes, x_scales, w_codes, w_scales, T: int, m: int, n: int, out, out_stride: int,
                         stream=None, check: bool = True) -> int:
    st = lib().flatquant_mxfp4_gemm(_ptr(x_codes), _ptr(x_scales), _ptr(w_codes), _ptr(w_scales), int(T), int(m), int(n),
                                    _ptr(out), int(out_stride), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_mxfp4_gemm")
    return st


def flatquant_dequant_mxfp4(codes, scales, rows: int, n: int, out, stream=None, check: bool = True) -> int:
    st = lib().flatquant_dequant_mxfp4(_ptr(codes), _ptr(scales), int(rows), int(n), _ptr(out), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_dequant_mxfp4")
    return st


def flatquant_kv_transform_quant_bits(kv, P, Hp: int, clip: float, bits: int, T: int, H: int, D: int, out_codes, out_scales,
                                      out_zeros, stream=None, check: bool = True) -> int:
    st = lib().flatquant_kv_transform_quant_bits(_ptr(kv), _ptr(P), int(Hp), float(clip), int(bits), int(T), int(H), int(D),
                                                 _ptr(out_codes), _ptr(out_scales), _ptr(out_zeros), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_kv_transform_quant_bits")
    return st


def flatquant_dequant_bits(codes, scales, zeros, rows: int, n: int, bits: int, out, stream=None, check: bool = True) -> int:
    st = lib().flatquant_dequant_bits(_ptr(codes), _ptr(scales), _ptr(zeros), int(rows), int(n), int(bits), _ptr(out),
                                      _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_dequant_bits")
    return st


def flatquant_dequant(codes, scales, zeros, rows: int, n: int, out, stream=None, check: bool = True) -> int:
    st = lib().flatquant_dequant(_ptr(codes), _ptr(scales), _ptr(zeros), int(rows), int(n), _ptr(out), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_dequant")
    return st


def flatquant_weight_transform_quant(w, A1, A2, clip, clip_mode: int, m: int, n1: int, n2: int, w_stride: int,
                                     out_codes, out_scales, stream=None, check: bool = True) -> int:
    st = lib().flatquant_weight_transform_quant(_ptr(w), _ptr(A1), _ptr(A2), _ptr(clip), int(clip_mode), int(m), int(n1),
                                                int(n2), int(w_stride), _ptr(out_codes), _ptr(out_scales), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_weight_transform_quant")
    return st


def flatquant_w4a4_gemm(x_codes, x_scales, w_codes, w_scales, T: int, m: int, n: int, out, out_stride: int,
                        stream=None, check: bool = True) -> int:
    st = lib().flatquant_w4a4_gemm(_ptr(x_codes), _ptr(x_scales), _ptr(w_codes), _ptr(w_scales), int(T), int(m), int(n),
                                   _ptr(out), int(out_stride), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_w4a4_gemm")
    return st


def flatquant_head_transform(x, P, Hp: int, T: int, H: int, D: int, out, stream=None, check: bool = True) -> int:
    st = lib().flatquant_head_transform(_ptr(x), _ptr(P), int(Hp), int(T), int(H), int(D), _ptr(out), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_head_transform")
    return st


def fq_inverse_transpose(P):
    """Host helper: fp16 [n, n] numpy array -> (fp16 (P^-1)^T, max |P^T out - I|).  Raises on a singular matrix."""
    import numpy as np
    P = np.ascontiguousarray(P, dtype=np.float16)
    n = P.shape[0]
    if P.ndim != 2 or P.shape != (n, n):
        raise ValueError("fq_inverse_transpose expects a square matrix")
    out = np.empty((n, n), dtype=np.float16)
    res = ctypes.c_double(0.0)
    st = lib().fq_inverse_transpose(P.ctypes.data, n, out.ctypes.data, ctypes.byref(res))
    if st != FQ_OK:
        raise FlatQuantError(st, "fq_inverse_transpose")
    return out, res.value


def flatquant_stream_probe(x, T: int, n: int, x_stride: int, out, stream=None, check: bool = True) -> int:
    st = lib().flatquant_stream_probe(_ptr(x), int(T), int(n), int(x_stride), _ptr(out), _stream(stream))
    if check and st != FQ_OK:
        raise FlatQuantError(st, "flatquant_stream_probe")
    return st


def fq_supported(n1: int, n2: int) -> bool:
    return bool(lib().fq_supported(int(n1), int(n2)))


def fq_choose_factors(n: int):
    a, b = ctypes.c_int(0), ctypes.c_int(0)
    st = lib().fq_choose_factors(int(n), ctypes.byref(a), ctypes.byref(b))
    if st != FQ_OK:
        raise FlatQuantError(st, "fq_choose_factors")
    return a.value, b.value


def fq_default_design_fits(n1: int, n2: int, m_bytes: int) -> bool:
    return bool(lib().fq_default_design_fits(int(n1), int(n2), int(m_bytes)))


def fq_lds_bytes(n1: int, n2: int) -> int:
    return int(lib().fq_lds_bytes(int(n1), int(n2)))


def fq_set_tuning(name: str, value: Optional[int]) -> None:
    """Set a tuning override (value) or remove it (None)."""
    st = lib().fq_set_tuning(name.encode(), 0 if value is None else int(value), 0 if value is None else 1)
    if st != FQ_OK:
        raise FlatQuantError(st, f"fq_set_tuning({name})")


def fq_abi_version() -> int:
    return int(lib().fq_abi_version())
