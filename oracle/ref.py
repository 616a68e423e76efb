"""ctypes front end of the C oracle (oracle/amxfp4_ref.c).

Test infrastructure: only tests, the smoke check and the benchmark's cpu_baseline leg import this module.
It works on host numpy arrays and shares nothing with the GPU library.

Scale kinds: 0 = E8M0 floor (Appendix B, Algorithm 1), 1 = E8M0 round (Appendix B, "Floor vs. Round"),
2 = FP8 E5M2 (Sec. 4.2 "FP8"), 3 = FP8 E4M3 (Sec. 4.2 ablation).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "amxfp4_ref.c")
_LIB = os.path.join(_HERE, "libamxfp4_ref.so")

E8M0_FLOOR, E8M0_ROUND, FP8_E5M2, FP8_E4M3 = 0, 1, 2, 3


class RefFormat(ctypes.Structure):
    _fields_ = [("group_size", ctypes.c_int32), ("elem", ctypes.c_int32), ("scale", ctypes.c_int32),
                ("asymmetric", ctypes.c_int32)]


def build(force=False):
    """Compile the oracle with gcc (plain C11 + OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
                               _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, u8p = ctypes.c_int64, ctypes.c_void_p
        L.amxfp4_quantize_ref.argtypes = [ctypes.POINTER(RefFormat), ctypes.c_void_p, i64, i64, i64, i64, u8p, u8p]
        L.amxfp4_quantize_ref.restype = ctypes.c_int
        L.amxfp4_dequantize_ref.argtypes = [ctypes.POINTER(RefFormat), u8p, u8p, i64, i64, ctypes.c_void_p]
        L.amxfp4_dequantize_ref.restype = ctypes.c_int
        L.amxfp4_gemm_ref.argtypes = [ctypes.POINTER(RefFormat), i64, i64, i64, u8p, u8p, u8p, u8p, ctypes.c_void_p,
                                      i64, i64]
        L.amxfp4_gemm_ref.restype = ctypes.c_int
        f32 = ctypes.c_float
        L.amxfp4_quantize_scaled_ref.argtypes = [ctypes.POINTER(RefFormat), ctypes.c_void_p, i64, i64, i64, i64, f32,
                                                 u8p, u8p]
        L.amxfp4_quantize_scaled_ref.restype = ctypes.c_int
        L.amxfp4_quantize_f32_ref.argtypes = [ctypes.POINTER(RefFormat), ctypes.c_void_p, i64, i64, u8p, u8p]
        L.amxfp4_quantize_f32_ref.restype = ctypes.c_int
        L.amxfp4_gemm_scaled_ref.argtypes = [ctypes.POINTER(RefFormat), i64, i64, i64, u8p, u8p, f32, u8p, u8p, f32,
                                             ctypes.c_void_p, i64, i64]
        L.amxfp4_gemm_scaled_ref.restype = ctypes.c_int
        L.amxfp4_tensor_scale_ref.argtypes = [ctypes.c_void_p, i64, i64, i64, i64, ctypes.c_void_p]
        L.amxfp4_tensor_scale_ref.restype = ctypes.c_int
        L.amxfp4_scale_encode_ref.argtypes = [ctypes.c_int32, ctypes.c_double]
        L.amxfp4_scale_encode_ref.restype = ctypes.c_uint8
        L.amxfp4_scale_decode_ref.argtypes = [ctypes.c_int32, ctypes.c_uint8]
        L.amxfp4_scale_decode_ref.restype = ctypes.c_double
        L.amxfp4_elem_encode_ref.argtypes = [ctypes.c_double, ctypes.c_double]
        L.amxfp4_elem_encode_ref.restype = ctypes.c_uint8
        L.amxfp4_ref_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _fmt(group_size, scale, asymmetric):
    return RefFormat(int(group_size), 0, int(scale), int(bool(asymmetric)))


def _groups(K, group_size):
    return 1 if group_size == -1 else K // group_size


def tensor_scale(x_bf16):
    """Tensor-wise scale pair (S_t, R_t = 1 / S_t) of the double-scaling scheme (Sec. 5.3), as numpy float32."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2
    out = np.zeros(2, np.float32)
    rc = lib().amxfp4_tensor_scale_ref(x_bf16.ctypes.data, x_bf16.shape[0], x_bf16.shape[1], x_bf16.strides[0] // 2,
                                       x_bf16.strides[1] // 2, out.ctypes.data)
    if rc:
        raise ValueError("amxfp4_tensor_scale_ref failed: %d" % rc)
    return out[0], out[1]


def quantize(x_bf16, group_size=32, scale=FP8_E5M2, asymmetric=True, k_axis=-1, tensor_rcp=1.0):
    """x_bf16: 2-D uint16 array of BF16 bit patterns, any strides. Groups run along `k_axis` (-1: along rows'
    elements; 0: down the columns, i.e. the operand is x.T). tensor_rcp: the factor R_t of a tensor-wise scale
    (Sec. 5.3), 1 for none. Returns (codes [rows, K/2] u8, scales u8)."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2
    xv = x_bf16 if k_axis in (-1, 1) else x_bf16.T
    rows, K = xv.shape
    rs, ks = xv.strides[0] // 2, xv.strides[1] // 2
    G = _groups(K, group_size)
    ns = 2 if asymmetric else 1
    codes = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, G, ns) if asymmetric else (rows, G), np.uint8)
    f = _fmt(group_size, scale, asymmetric)
    rc = lib().amxfp4_quantize_scaled_ref(ctypes.byref(f), xv.ctypes.data, rows, K, rs, ks,
                                          ctypes.c_float(float(np.float32(tensor_rcp))), codes.ctypes.data,
                                          scales.ctypes.data)
    if rc:
        raise ValueError("amxfp4_quantize_scaled_ref failed: %d" % rc)
    return codes, scales


def quantize_f32(y, group_size=32, scale=FP8_E5M2, asymmetric=True):
    """The group-wise cast of single-precision values: y 2-D float32, groups along each row. Returns (codes, scales)."""
    y = np.ascontiguousarray(y, np.float32)
    assert y.ndim == 2
    rows, K = y.shape
    G = _groups(K, group_size)
    codes = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, G, 2) if asymmetric else (rows, G), np.uint8)
    f = _fmt(group_size, scale, asymmetric)
    rc = lib().amxfp4_quantize_f32_ref(ctypes.byref(f), y.ctypes.data, rows, K, codes.ctypes.data, scales.ctypes.data)
    if rc:
        raise ValueError("amxfp4_quantize_f32_ref failed: %d" % rc)
    return codes, scales


def dequantize(codes, scales, group_size=32, scale=FP8_E5M2, asymmetric=True, tensor_scale=1.0):
    """Returns float64 [rows, K] (times the tensor-wise scale S_t of Sec. 5.3, exact in float64)."""
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.uint8)
    rows, K = codes.shape[0], codes.shape[1] * 2
    out = np.empty((rows, K), np.float64)
    f = _fmt(group_size, scale, asymmetric)
    rc = lib().amxfp4_dequantize_ref(ctypes.byref(f), codes.ctypes.data, scales.ctypes.data, rows, K, out.ctypes.data)
    if rc:
        raise ValueError("amxfp4_dequantize_ref failed: %d" % rc)
    return out if tensor_scale == 1.0 else out * np.float64(np.float32(tensor_scale))


def gemm(a_codes, a_scales, b_codes, b_scales, group_size=32, scale=FP8_E5M2, asymmetric=True, a_tensor_scale=1.0,
         b_tensor_scale=1.0):
    """a_codes [M, K/2] or [batch, M, K/2]; b_codes [N, K/2] or [batch, N, K/2]. Returns float32 C = A_hat.B_hat^T
    (operands times their tensor-wise scales S_t of Sec. 5.3, 1 for none)."""
    a_codes = np.ascontiguousarray(a_codes, np.uint8)
    b_codes = np.ascontiguousarray(b_codes, np.uint8)
    a_scales = np.ascontiguousarray(a_scales, np.uint8)
    b_scales = np.ascontiguousarray(b_scales, np.uint8)
    batched = a_codes.ndim == 3
    batch = a_codes.shape[0] if batched else 1
    M, K = a_codes.shape[-2], a_codes.shape[-1] * 2
    N = b_codes.shape[-2]
    C = np.empty((batch, M, N), np.float32)
    f = _fmt(group_size, scale, asymmetric)
    rc = lib().amxfp4_gemm_scaled_ref(ctypes.byref(f), M, N, K, a_codes.ctypes.data, a_scales.ctypes.data,
                                      ctypes.c_float(float(np.float32(a_tensor_scale))), b_codes.ctypes.data,
                                      b_scales.ctypes.data, ctypes.c_float(float(np.float32(b_tensor_scale))),
                                      C.ctypes.data, N, batch)
    if rc:
        raise ValueError("amxfp4_gemm_scaled_ref failed: %d" % rc)
    return C if batched else C[0]


def scale_encode(kind, amax):
    return int(lib().amxfp4_scale_encode_ref(kind, float(amax)))


def scale_decode(kind, byte):
    return float(lib().amxfp4_scale_decode_ref(kind, int(byte)))


def elem_encode(absx, S):
    return int(lib().amxfp4_elem_encode_ref(float(absx), float(S)))


def num_threads():
    return int(lib().amxfp4_ref_num_threads())
