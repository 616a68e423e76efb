"""Thin ctypes binding of libamxfp4.so: the same entry points as include/amxfp4.h and include/amxfp4_layer.h, taking
torch CUDA tensors.

Only argument marshalling happens here (pointers, sizes, the current HIP stream); every step of the path runs in
the library's kernels. There is no fallback: if the library has not been built, or no GPU is present, calls raise.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libamxfp4.so")

E8M0_FLOOR, E8M0_ROUND, FP8_E5M2, FP8_E4M3 = 0, 1, 2, 3


class AmxFormat(ctypes.Structure):
    _fields_ = [("group_size", ctypes.c_int32), ("elem", ctypes.c_int32), ("scale", ctypes.c_int32),
                ("asymmetric", ctypes.c_int32)]


class AmxGemmOptions(ctypes.Structure):
    _fields_ = [("e5m2_kernel", ctypes.c_int32), ("pot_kernel", ctypes.c_int32), ("tile", ctypes.c_int32),
                ("few_rows", ctypes.c_int32)]


class AmxError(RuntimeError):
    pass


_lib = None


def load():
    """Loads the built library (does not compile it) and declares the signatures of include/amxfp4.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise AmxError("libamxfp4.so is not built: run `python -m paper_2411_09909_amd.build` (needs hipcc)")
    L = ctypes.CDLL(LIB_PATH)
    i64, vp, fp = ctypes.c_int64, ctypes.c_void_p, ctypes.POINTER(AmxFormat)
    L.amxfp4_last_error.restype = ctypes.c_char_p
    for name in ("amxfp4_codes_bytes", "amxfp4_scales_bytes"):
        getattr(L, name).argtypes = [fp, i64, i64]
        getattr(L, name).restype = ctypes.c_size_t
    L.amxfp4_gemm_workspace_bytes.argtypes = [fp, i64, i64, i64, i64]
    L.amxfp4_gemm_workspace_bytes.restype = ctypes.c_size_t
    for p in ("amxfp4", "mxfp4"):
        q, d, g = getattr(L, p + "_quantize"), getattr(L, p + "_dequantize"), getattr(L, p + "_gemm")
        q.argtypes = [fp, vp, i64, i64, i64, i64, vp, vp, vp]
        d.argtypes = [fp, vp, vp, i64, i64, vp, ctypes.c_int32, vp]
        g.argtypes = [fp, i64, i64, i64, vp, vp, vp, vp, vp, i64, i64, vp, ctypes.c_size_t, vp]
        q.restype = d.restype = g.restype = ctypes.c_int
    L.amxfp4_gemm_silu_mul_workspace_bytes.argtypes = [fp, i64, i64, i64]
    L.amxfp4_gemm_silu_mul_workspace_bytes.restype = ctypes.c_size_t
    L.amxfp4_gemm_silu_mul.argtypes = [fp, i64, i64, i64, vp, vp, vp, vp, vp, i64, vp, ctypes.c_size_t, vp]
    L.amxfp4_gemm_silu_mul.restype = ctypes.c_int
    L.amxfp4_gemm_silu_mul_prepared_workspace_bytes.argtypes = [fp, i64, i64, i64]
    L.amxfp4_gemm_silu_mul_prepared_workspace_bytes.restype = ctypes.c_size_t
    L.amxfp4_gemm_silu_mul_prepared.argtypes = [fp, i64, i64, i64, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, i64, vp,
                                                ctypes.c_size_t, vp]
    L.amxfp4_gemm_silu_mul_prepared.restype = ctypes.c_int
    L.amxfp4_quantize_batched.argtypes = [fp, vp, i64, i64, i64, i64, i64, i64, vp, vp, vp]
    L.amxfp4_quantize_batched.restype = ctypes.c_int
    L.amxfp4_profile_next_gemm.argtypes = [vp, vp]
    L.amxfp4_profile_next_gemm.restype = ctypes.c_int
    op = ctypes.POINTER(AmxGemmOptions)
    L.amxfp4_gemm_workspace_bytes_ex.argtypes = [fp, op, i64, i64, i64, i64]
    L.amxfp4_gemm_workspace_bytes_ex.restype = ctypes.c_size_t
    L.amxfp4_gemm_ex.argtypes = [fp, op, i64, i64, i64, vp, vp, vp, vp, vp, i64, i64, vp, ctypes.c_size_t, vp]
    L.amxfp4_gemm_ex.restype = ctypes.c_int
    L.amxfp4_gemm_static.argtypes = [fp, i64, i64, i64, vp, vp, vp, vp, vp, i64, i64, vp]
    L.amxfp4_gemm_static.restype = ctypes.c_int
    L.amxfp4_weights_prepared_bytes.argtypes = [fp, i64, i64]
    L.amxfp4_weights_prepared_bytes.restype = ctypes.c_size_t
    L.amxfp4_prepare_weights.argtypes = [fp, i64, i64, vp, vp, vp, ctypes.c_size_t, vp]
    L.amxfp4_prepare_weights.restype = ctypes.c_int
    L.amxfp4_gemm_prepared_workspace_bytes.argtypes = [fp, i64, i64, i64]
    L.amxfp4_gemm_prepared_workspace_bytes.restype = ctypes.c_size_t
    L.amxfp4_gemm_prepared.argtypes = [fp, i64, i64, i64, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, i64, vp,
                                       ctypes.c_size_t, vp]
    L.amxfp4_gemm_prepared.restype = ctypes.c_int
    f32, f64, i32 = ctypes.c_float, ctypes.c_double, ctypes.c_int32
    L.amxfp4_tensor_scale.argtypes = [vp, i64, i64, i64, vp, vp]
    L.amxfp4_quantize_scaled.argtypes = [fp, vp, i64, i64, i64, i64, vp, vp, vp, vp]
    L.amxfp4_dequantize_scaled.argtypes = [fp, vp, vp, i64, i64, vp, vp, vp]
    L.amxfp4_gemm_scaled.argtypes = [fp, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, i64, i64, vp, ctypes.c_size_t, vp]
    for name in ("amxfp4_tensor_scale", "amxfp4_quantize_scaled", "amxfp4_dequantize_scaled", "amxfp4_gemm_scaled"):
        getattr(L, name).restype = ctypes.c_int
    L.amxfp4_gemm_scaled_workspace_bytes.argtypes = [fp, i64, i64, i64, i64]
    L.amxfp4_gemm_scaled_workspace_bytes.restype = ctypes.c_size_t
    L.amxfp4_attention_workspace_bytes.argtypes = [fp, i64, i64, i64, i64, i64]
    L.amxfp4_attention_workspace_bytes.restype = ctypes.c_size_t
    L.amxfp4_attention.argtypes = [fp, i64, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, f32, i32, vp, vp,
                                   ctypes.c_size_t, vp]
    L.amxfp4_attention.restype = ctypes.c_int
    L.amxfp4_attention_merged.argtypes = L.amxfp4_attention.argtypes
    L.amxfp4_attention_merged.restype = ctypes.c_int
    L.amxfp4_attention_decode_workspace_bytes.argtypes = [fp, i64, i64, i64, i64, i64, i64]
    L.amxfp4_attention_decode_workspace_bytes.restype = ctypes.c_size_t
    L.amxfp4_attention_decode.argtypes = [fp, i64, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, f32, i32, i64, vp, vp,
                                          ctypes.c_size_t, vp]
    L.amxfp4_attention_decode.restype = ctypes.c_int
    L.amxfp4_peak_mfma.argtypes = [i32, vp, i32, vp, ctypes.POINTER(f64), vp]
    L.amxfp4_peak_mfma.restype = ctypes.c_int
    L.amxfp4_peak_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.amxfp4_peak_copy.restype = ctypes.c_int
    for name, args in (("amxfp4_rmsnorm", [vp, vp, i64, i64, f32, vp, vp]),
                       ("amxfp4_split_heads_rope", [vp, i64, i64, i64, i64, i64, i32, i64, f64, vp, vp]),
                       ("amxfp4_split_heads_rope_quantize", [fp, vp, i64, i64, i64, i64, i64, i64, f64, vp, vp, vp]),
                       ("amxfp4_softmax_causal", [vp, i64, i64, i64, f32, vp, vp]),
                       ("amxfp4_silu_mul", [vp, i64, i64, vp, vp]),
                       ("amxfp4_residual_add", [vp, vp, i64, vp, vp]),
                       ("amxfp4_merge_heads", [vp, i64, i64, i64, i64, vp, vp]),
                       ("amxfp4_rmsnorm_quantize", [fp, vp, vp, vp, vp, i64, i64, f32, vp, vp, vp])):
        getattr(L, name).argtypes = args
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise AmxError("libamxfp4 error %d: %s" % (rc, load().amxfp4_last_error().decode()))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need_cuda(*ts):
    for t in ts:
        if not t.is_cuda:
            raise AmxError("libamxfp4 works on device memory only")


def make_format(scale=FP8_E5M2, asymmetric=True, group_size=32):
    return AmxFormat(int(group_size), 0, int(scale), int(bool(asymmetric)))


def _groups(fmt, K):
    """Groups along a row of K elements (group_size -1: the whole row is one group)."""
    return 1 if fmt.group_size == -1 else K // fmt.group_size


def codes_bytes(fmt, rows, K):
    return load().amxfp4_codes_bytes(ctypes.byref(fmt), rows, K)


def scales_bytes(fmt, rows, K):
    return load().amxfp4_scales_bytes(ctypes.byref(fmt), rows, K)


E5M2_KERNELS = {"panel": 0, "hybrid": 1, "fused": 2}
POT_KERNELS = {"merged_fp6": 0, "split": 1, "merged_fp8": 2}
TILES = {"auto": 0, "256x256": 1, "256x128": 2, "64x256": 3}


def gemm_options(e5m2_kernel="panel", pot_kernel="merged_fp6", tile="auto", few_rows=0):
    """The per-call kernel choice of amxfp4_gemm_ex (names or the header's integers); few_rows: 0 = where it applies,
    -1 = never, n > 0 = with n outer K slices."""
    return AmxGemmOptions(E5M2_KERNELS.get(e5m2_kernel, e5m2_kernel), POT_KERNELS.get(pot_kernel, pot_kernel),
                          TILES.get(tile, tile), int(few_rows))


def gemm_workspace_bytes(fmt, M, N, K, batch=1, options=None):
    if options is None:
        return load().amxfp4_gemm_workspace_bytes(ctypes.byref(fmt), M, N, K, batch)
    return load().amxfp4_gemm_workspace_bytes_ex(ctypes.byref(fmt), ctypes.byref(options), M, N, K, batch)


def profile_next_gemm(start_event, stop_event):
    """Arms raw hipEvent_t handles (ints) around the matrix-multiply kernel of the next gemm() call."""
    _check(load().amxfp4_profile_next_gemm(start_event, stop_event))


PEAK_MFMA = {"bf16": 0, "fp8": 1, "fp4": 2, "f16": 3, "fp6": 4}


def peak_mfma(mfma, operand, iterations, sink):
    """Launches the register-resident MFMA loop ("bf16" | "f16" | "fp8" | "fp6" | "fp4") on the current stream; operand: 16384-byte
    CUDA tensor, sink: float32 CUDA tensor of 512 * 256 elements. Returns the floating-point operations it performs."""
    _need_cuda(operand, sink)
    if operand.numel() * operand.element_size() < 16384 or sink.numel() < 512 * 256 or sink.dtype != torch.float32:
        raise AmxError("peak_mfma: operand needs 16384 bytes, sink 512 * 256 float32")
    flops = ctypes.c_double()
    _check(load().amxfp4_peak_mfma(PEAK_MFMA[mfma], operand.data_ptr(), int(iterations), sink.data_ptr(),
                                   ctypes.byref(flops), _stream()))
    return flops.value


def peak_copy(src, dst):
    """Streaming copy src -> dst (CUDA tensors of equal byte size, a multiple of 16) on the current stream."""
    _need_cuda(src, dst)
    n = src.numel() * src.element_size()
    if n != dst.numel() * dst.element_size() or not (src.is_contiguous() and dst.is_contiguous()):
        raise AmxError("peak_copy: contiguous buffers of equal size needed")
    _check(load().amxfp4_peak_copy(src.data_ptr(), dst.data_ptr(), n, _stream()))


def _fn(fmt, name, baseline):
    return getattr(load(), ("mxfp4_" if baseline else "amxfp4_") + name)


def tensor_scale(x, out=None):
    """Tensor-wise scale of the double-scaling scheme: x 2-D BF16 CUDA tensor with contiguous rows -> float32 CUDA
    tensor {S_t, 1 / S_t} (computed on the device, stream-ordered)."""
    _need_cuda(x)
    assert x.dim() == 2 and x.element_size() == 2 and x.stride(1) == 1
    if out is None:
        out = torch.empty(2, dtype=torch.float32, device=x.device)
    _check(load().amxfp4_tensor_scale(x.data_ptr(), x.shape[0], x.shape[1], x.stride(0), out.data_ptr(), _stream()))
    return out


def _pair_ptr(pair):
    _need_cuda(pair)
    if pair.dtype != torch.float32 or pair.numel() < 2 or not pair.is_contiguous():
        raise AmxError("a tensor-scale pair is a contiguous float32 CUDA tensor of two elements")
    return pair.data_ptr()


def quantize(fmt, x, k_axis=-1, codes=None, scales=None, baseline=False, tensor_pair=None):
    """x: 2-D BF16 (or uint16 bit pattern) CUDA tensor. k_axis=-1: groups along each row (rows contiguous in K);
    k_axis=0: groups run down the columns (operand = x.T, strided cast). tensor_pair: result of tensor_scale() for
    the double-scaling cast. Returns (codes u8 [rows, K/2], scales u8)."""
    _need_cuda(x)
    assert x.dim() == 2 and x.element_size() == 2
    if k_axis in (-1, 1):
        rows, K = x.shape
        row_stride, k_stride = x.stride(0), x.stride(1)
    else:
        K, rows = x.shape
        k_stride, row_stride = x.stride(0), x.stride(1)
    asym = bool(fmt.asymmetric) and not baseline
    if codes is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
    if scales is None:
        shape = (rows, _groups(fmt, K), 2) if asym else (rows, _groups(fmt, K))
        scales = torch.empty(shape, dtype=torch.uint8, device=x.device)
    if tensor_pair is not None:
        if baseline:
            raise AmxError("the mxfp4_* baseline calls take no tensor-wise scale; clear fmt.asymmetric instead")
        _check(load().amxfp4_quantize_scaled(ctypes.byref(fmt), x.data_ptr(), rows, K, row_stride, k_stride,
                                             _pair_ptr(tensor_pair), codes.data_ptr(), scales.data_ptr(), _stream()))
        return codes, scales
    _check(_fn(fmt, "quantize", baseline)(ctypes.byref(fmt), x.data_ptr(), rows, K, row_stride, k_stride,
                                          codes.data_ptr(), scales.data_ptr(), _stream()))
    return codes, scales


def quantize_batched(fmt, x, k_axis=-1, codes=None, scales=None):
    """x: 3-D BF16 CUDA tensor [batch, ., .]; every x[b] is cast as quantize(fmt, x[b], k_axis) would, in one launch.
    Returns (codes u8 [batch, rows, K/2], scales u8 [batch, rows, K/group_size(, 2)])."""
    _need_cuda(x)
    assert x.dim() == 3 and x.element_size() == 2
    batch = x.shape[0]
    if k_axis in (-1, 2):
        rows, K = x.shape[1], x.shape[2]
        row_stride, k_stride = x.stride(1), x.stride(2)
    else:
        K, rows = x.shape[1], x.shape[2]
        k_stride, row_stride = x.stride(1), x.stride(2)
    asym = bool(fmt.asymmetric)
    if codes is None:
        codes = torch.empty((batch, rows, K // 2), dtype=torch.uint8, device=x.device)
    if scales is None:
        shape = (batch, rows, _groups(fmt, K), 2) if asym else (batch, rows, _groups(fmt, K))
        scales = torch.empty(shape, dtype=torch.uint8, device=x.device)
    _check(load().amxfp4_quantize_batched(ctypes.byref(fmt), x.data_ptr(), batch, x.stride(0), rows, K, row_stride,
                                          k_stride, codes.data_ptr(), scales.data_ptr(), _stream()))
    return codes, scales


def interleave_gate_up(gate, up):
    """Rows of the two [width, K] projection matrices interleaved in blocks of 32, the order gemm_silu_mul() wants."""
    width, K = gate.shape
    assert up.shape == gate.shape and width % 32 == 0
    return torch.stack([gate.view(width // 32, 32, K), up.view(width // 32, 32, K)], 1).reshape(2 * width, K)


def gemm_silu_mul_workspace_bytes(fmt, M, width, K):
    return int(load().amxfp4_gemm_silu_mul_workspace_bytes(ctypes.byref(fmt), M, width, K))


def gemm_silu_mul(fmt, a_codes, a_scales, b_codes, b_scales, out=None, workspace=None, prepared=None):
    """bf16(silu(g) * u) of the fused gate / up projection (g | u) = A . B^T, B's rows interleaved as by
    interleave_gate_up() before they were cast. prepared: prepare_weights() of those interleaved weights
    (amxfp4_gemm_silu_mul_prepared). Returns [M, width] BF16."""
    _need_cuda(a_codes, a_scales, b_codes, b_scales)
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    width = b_codes.shape[0] // 2
    if out is None:
        out = torch.empty((M, width), dtype=torch.bfloat16, device=a_codes.device)
    if prepared is not None:
        need = int(load().amxfp4_gemm_silu_mul_prepared_workspace_bytes(ctypes.byref(fmt), M, width, K))
        if need and (workspace is None or workspace.numel() < need):
            workspace = torch.empty(need, dtype=torch.uint8, device=a_codes.device)
        n_prep = prepared.numel() * prepared.element_size()
        _check(load().amxfp4_gemm_silu_mul_prepared(
            ctypes.byref(fmt), M, width, K, a_codes.data_ptr(), a_scales.data_ptr(), b_codes.data_ptr(),
            b_scales.data_ptr(), prepared.data_ptr() if n_prep else None, n_prep, out.data_ptr(), out.stride(0),
            workspace.data_ptr() if need else None, workspace.numel() if need else 0, _stream()))
        return out
    need = gemm_silu_mul_workspace_bytes(fmt, M, width, K)
    if need and (workspace is None or workspace.numel() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=a_codes.device)
    _check(load().amxfp4_gemm_silu_mul(ctypes.byref(fmt), M, width, K, a_codes.data_ptr(), a_scales.data_ptr(),
                                       b_codes.data_ptr(), b_scales.data_ptr(), out.data_ptr(), out.stride(0),
                                       workspace.data_ptr() if need else None, workspace.numel() if need else 0,
                                       _stream()))
    return out


def dequantize(fmt, codes, scales, out_dtype=torch.float32, baseline=False, tensor_pair=None):
    _need_cuda(codes, scales)
    rows, K = codes.shape[0], codes.shape[1] * 2
    out = torch.empty((rows, K), dtype=out_dtype, device=codes.device)
    if tensor_pair is not None:
        if baseline or out_dtype != torch.float32:
            raise AmxError("the scaled dequantize writes float32 and has no mxfp4_* twin")
        _check(load().amxfp4_dequantize_scaled(ctypes.byref(fmt), codes.data_ptr(), scales.data_ptr(), rows, K,
                                               _pair_ptr(tensor_pair), out.data_ptr(), _stream()))
        return out
    _check(_fn(fmt, "dequantize", baseline)(ctypes.byref(fmt), codes.data_ptr(), scales.data_ptr(), rows, K,
                                            out.data_ptr(), 1 if out_dtype == torch.bfloat16 else 0, _stream()))
    return out


def gemm(fmt, a_codes, a_scales, b_codes, b_scales, out=None, workspace=None, baseline=False, a_pair=None,
         b_pair=None, options=None):
    """a_codes [M, K/2] or [batch, M, K/2]; b_codes [N, K/2] or [batch, N, K/2] (contiguous). a_pair / b_pair: the
    operands' tensor_scale() results (both or neither). options: gemm_options() for amxfp4_gemm_ex. out: FP32
    [.., M, ldc >= N] with contiguous rows. Returns FP32 C."""
    _need_cuda(a_codes, a_scales, b_codes, b_scales)
    batched = a_codes.dim() == 3
    batch = a_codes.shape[0] if batched else 1
    M, K = a_codes.shape[-2], a_codes.shape[-1] * 2
    N = b_codes.shape[-2]
    for t in (a_codes, a_scales, b_codes, b_scales):
        assert t.is_contiguous()
    if out is None:
        out = torch.empty((batch, M, N) if batched else (M, N), dtype=torch.float32, device=a_codes.device)
    scaled = a_pair is not None or b_pair is not None
    if scaled and (a_pair is None or b_pair is None or baseline):
        raise AmxError("the scaled GEMM needs both tensor-scale pairs and has no mxfp4_* twin")
    if options is not None and (scaled or baseline):
        raise AmxError("kernel options go with the plain amxfp4_gemm only (clear fmt.asymmetric for the baseline)")
    need = (load().amxfp4_gemm_scaled_workspace_bytes(ctypes.byref(fmt), M, N, K, batch) if scaled
            else gemm_workspace_bytes(fmt, M, N, K, batch, options))
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=a_codes.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if scaled:
        _check(load().amxfp4_gemm_scaled(ctypes.byref(fmt), M, N, K, a_codes.data_ptr(), a_scales.data_ptr(),
                                         _pair_ptr(a_pair), b_codes.data_ptr(), b_scales.data_ptr(), _pair_ptr(b_pair),
                                         out.data_ptr(), out.stride(-2), batch, ws_ptr, ws_len, _stream()))
        return out
    if options is not None:
        _check(load().amxfp4_gemm_ex(ctypes.byref(fmt), ctypes.byref(options), M, N, K, a_codes.data_ptr(),
                                     a_scales.data_ptr(), b_codes.data_ptr(), b_scales.data_ptr(), out.data_ptr(),
                                     out.stride(-2), batch, ws_ptr, ws_len, _stream()))
        return out
    _check(_fn(fmt, "gemm", baseline)(ctypes.byref(fmt), M, N, K, a_codes.data_ptr(), a_scales.data_ptr(),
                                      b_codes.data_ptr(), b_scales.data_ptr(), out.data_ptr(), out.stride(-2), batch,
                                      ws_ptr, ws_len, _stream()))
    return out


GEMM_STATIC_BYTES = 16 << 20  # AMXFP4_GEMM_STATIC_BYTES of include/amxfp4.h


def gemm_static(fmt, a_codes, a_scales, b_codes, b_scales, out):
    """amxfp4_gemm_static: the product into the caller's `out` (FP32 [.., M, ldc >= N], rows contiguous) with the
    library's static scratch; nothing is allocated here or in the library."""
    _need_cuda(a_codes, a_scales, b_codes, b_scales, out)
    batch = a_codes.shape[0] if a_codes.dim() == 3 else 1
    M, K = a_codes.shape[-2], a_codes.shape[-1] * 2
    N = b_codes.shape[-2]
    _check(load().amxfp4_gemm_static(ctypes.byref(fmt), M, N, K, a_codes.data_ptr(), a_scales.data_ptr(),
                                     b_codes.data_ptr(), b_scales.data_ptr(), out.data_ptr(), out.stride(-2), batch,
                                     _stream()))
    return out


def attention_decode(fmt, q_codes, q_scales, k_codes, k_scales, v_codes, v_scales, scale, causal=True, key_splits=1,
                     out=None, workspace=None):
    """amxfp4_attention_decode: few queries ((Hq / Hkv) * Sq <= 32) against many keys, the keys cut into `key_splits`
    ranges. Shapes as attention(); returns FP32 [Hq, Sq, D]."""
    _need_cuda(q_codes, q_scales, k_codes, k_scales, v_codes, v_scales)
    Hq, Sq, D = q_codes.shape[0], q_codes.shape[1], q_codes.shape[2] * 2
    Hkv, Sk = k_codes.shape[0], k_codes.shape[1]
    assert k_codes.shape[2] * 2 == D and tuple(v_codes.shape) == (Hkv, D, Sk // 2)
    for t in (q_codes, q_scales, k_codes, k_scales, v_codes, v_scales):
        assert t.is_contiguous()
    if out is None:
        out = torch.empty((Hq, Sq, D), dtype=torch.float32, device=q_codes.device)
    need = int(load().amxfp4_attention_decode_workspace_bytes(ctypes.byref(fmt), Hq, Hkv, Sq, Sk, D, key_splits))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q_codes.device)
    _check(load().amxfp4_attention_decode(ctypes.byref(fmt), Hq, Hkv, Sq, Sk, D, q_codes.data_ptr(), q_scales.data_ptr(),
                                          k_codes.data_ptr(), k_scales.data_ptr(), v_codes.data_ptr(),
                                          v_scales.data_ptr(), float(scale), 1 if causal else 0, int(key_splits),
                                          out.data_ptr(), workspace.data_ptr(),
                                          workspace.numel() * workspace.element_size(), _stream()))
    return out


def prepare_weights(fmt, b_codes, b_scales):
    """amxfp4_prepare_weights: the prepared form of static weights b_codes [N, K/2] (a uint8 tensor, empty for formats
    whose kernels read the weights as stored); pass it to gemm_prepared()."""
    _need_cuda(b_codes, b_scales)
    N, K = b_codes.shape[0], b_codes.shape[1] * 2
    need = int(load().amxfp4_weights_prepared_bytes(ctypes.byref(fmt), N, K))
    prepared = torch.empty(need, dtype=torch.uint8, device=b_codes.device)
    _check(load().amxfp4_prepare_weights(ctypes.byref(fmt), N, K, b_codes.data_ptr(), b_scales.data_ptr(),
                                         prepared.data_ptr() if need else None, need, _stream()))
    return prepared


def gemm_prepared(fmt, a_codes, a_scales, b_codes, b_scales, prepared, out=None, workspace=None):
    """amxfp4_gemm_prepared: C = A . B^T with the weights' prepared form (prepare_weights()). One problem per call."""
    _need_cuda(a_codes, a_scales, b_codes, b_scales)
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    N = b_codes.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_codes.device)
    need = int(load().amxfp4_gemm_prepared_workspace_bytes(ctypes.byref(fmt), M, N, K))
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=a_codes.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    n_prep = prepared.numel() * prepared.element_size()
    _check(load().amxfp4_gemm_prepared(ctypes.byref(fmt), M, N, K, a_codes.data_ptr(), a_scales.data_ptr(),
                                       b_codes.data_ptr(), b_scales.data_ptr(), prepared.data_ptr() if n_prep else None,
                                       n_prep, out.data_ptr(), out.stride(-2), ws_ptr, ws_len, _stream()))
    return out


def attention_workspace_bytes(fmt, q_heads, kv_heads, Sq, Sk, head_dim=128):
    return int(load().amxfp4_attention_workspace_bytes(ctypes.byref(fmt), q_heads, kv_heads, Sq, Sk, head_dim))


def attention(fmt, q_codes, q_scales, k_codes, k_scales, v_codes, v_scales, scale, causal=True, out=None,
              workspace=None, merged=False):
    """Fused quantized attention. q_codes [Hq, Sq, D/2], k_codes [Hkv, Sk, D/2] (cast along D), v_codes
    [Hkv, D, Sk/2] (each head's V cast along the keys, k_axis=0), scales to match. Returns FP32 [Hq, Sq, D], or with
    merged=True the same values as BF16 [Sq, Hq * D] (token-major, heads side by side)."""
    ts = (q_codes, q_scales, k_codes, k_scales, v_codes, v_scales)
    _need_cuda(*ts)
    for t in ts:
        assert t.is_contiguous()
    Hq, Sq, D = q_codes.shape[0], q_codes.shape[1], q_codes.shape[2] * 2
    Hkv, Sk = k_codes.shape[0], k_codes.shape[1]
    assert k_codes.shape[2] * 2 == D and tuple(v_codes.shape) == (Hkv, D, Sk // 2)
    if out is None:
        out = (_bf16_out((Sq, Hq * D), q_codes.device) if merged
               else torch.empty((Hq, Sq, D), dtype=torch.float32, device=q_codes.device))
    assert out.is_contiguous() and out.dtype == (torch.bfloat16 if merged else torch.float32)
    need = attention_workspace_bytes(fmt, Hq, Hkv, Sq, Sk, D)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q_codes.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    call = load().amxfp4_attention_merged if merged else load().amxfp4_attention
    _check(call(ctypes.byref(fmt), Hq, Hkv, Sq, Sk, D, q_codes.data_ptr(), q_scales.data_ptr(), k_codes.data_ptr(),
                k_scales.data_ptr(), v_codes.data_ptr(), v_scales.data_ptr(), float(scale), int(bool(causal)),
                out.data_ptr(), ws_ptr, ws_len, _stream()))
    return out


# ---- glue operators of the decoder-layer workload (include/amxfp4_layer.h) ------------------------------------------

def _bf16_out(shape, device):
    return torch.empty(shape, dtype=torch.bfloat16, device=device)


def rmsnorm(x, weight, eps):
    """x [rows, dim] BF16, weight [dim] FP32 -> BF16 [rows, dim]."""
    _need_cuda(x, weight)
    assert x.is_contiguous() and x.dtype == torch.bfloat16 and weight.dtype == torch.float32
    out = _bf16_out(x.shape, x.device)
    _check(load().amxfp4_rmsnorm(x.data_ptr(), weight.data_ptr(), x.shape[0], x.shape[1], eps, out.data_ptr(),
                                 _stream()))
    return out


def rmsnorm_quantize(fmt, x, weight, eps, y=None):
    """quantize(fmt, rmsnorm(x, weight, eps)) in one pass; with y (FP32, the shape of x) the residual addition first:
    returns (codes, scales), or (x + y as BF16, codes, scales) when y is given."""
    _need_cuda(x, weight)
    assert x.is_contiguous() and x.dtype == torch.bfloat16 and weight.dtype == torch.float32 and x.dim() == 2
    rows, dim = x.shape
    codes = torch.empty((rows, dim // 2), dtype=torch.uint8, device=x.device)
    shape = (rows, _groups(fmt, dim), 2) if fmt.asymmetric else (rows, _groups(fmt, dim))
    scales = torch.empty(shape, dtype=torch.uint8, device=x.device)
    total = None
    if y is not None:
        _need_cuda(y)
        assert y.is_contiguous() and y.dtype == torch.float32 and y.shape == x.shape
        total = _bf16_out(x.shape, x.device)
    _check(load().amxfp4_rmsnorm_quantize(ctypes.byref(fmt), x.data_ptr(), y.data_ptr() if y is not None else None,
                                          total.data_ptr() if y is not None else None, weight.data_ptr(), rows, dim,
                                          eps, codes.data_ptr(), scales.data_ptr(), _stream()))
    return (codes, scales) if y is None else (total, codes, scales)


def split_heads_rope(proj, col0, heads, head_dim, rotate, pos0=0, theta=10000.0):
    """proj [seq, ld] FP32 (a projection output) -> BF16 [heads, seq, head_dim], rotary embedding if `rotate`."""
    _need_cuda(proj)
    assert proj.dtype == torch.float32 and proj.dim() == 2 and proj.stride(1) == 1
    seq = proj.shape[0]
    out = _bf16_out((heads, seq, head_dim), proj.device)
    _check(load().amxfp4_split_heads_rope(proj.data_ptr(), seq, proj.stride(0), col0, heads, head_dim,
                                          1 if rotate else 0, pos0, theta, out.data_ptr(), _stream()))
    return out


def split_heads_rope_quantize(fmt, proj, col0, heads, head_dim, pos0=0, theta=10000.0):
    """split_heads_rope(rotate=True) followed by quantize() along head_dim, in one launch: (codes [heads, seq,
    head_dim / 2], scales [heads, seq, head_dim / 32(, 2)]), the Q or K operand of attention()."""
    _need_cuda(proj)
    assert proj.dtype == torch.float32 and proj.dim() == 2 and proj.stride(1) == 1
    seq = proj.shape[0]
    codes = torch.empty((heads, seq, head_dim // 2), dtype=torch.uint8, device=proj.device)
    scales = torch.empty((heads, seq, head_dim // 32) + ((2,) if fmt.asymmetric else ()), dtype=torch.uint8,
                         device=proj.device)
    _check(load().amxfp4_split_heads_rope_quantize(ctypes.byref(fmt), proj.data_ptr(), seq, proj.stride(0), col0, heads,
                                                   head_dim, pos0, theta, codes.data_ptr(), scales.data_ptr(),
                                                   _stream()))
    return codes, scales


def softmax_causal(scores, scale):
    """scores [batch, rows, cols] FP32 (row r = query position r % cols) -> BF16 probabilities, masked entries 0."""
    _need_cuda(scores)
    assert scores.dtype == torch.float32 and scores.dim() == 3 and scores.is_contiguous()
    out = _bf16_out(scores.shape, scores.device)
    _check(load().amxfp4_softmax_causal(scores.data_ptr(), scores.shape[0], scores.shape[1], scores.shape[2], scale,
                                        out.data_ptr(), _stream()))
    return out


def silu_mul(gate_up):
    """gate_up [rows, 2 * width] FP32 (gate | up) -> BF16 [rows, width] = silu(gate) * up."""
    _need_cuda(gate_up)
    assert gate_up.dtype == torch.float32 and gate_up.is_contiguous()
    rows, width = gate_up.shape[0], gate_up.shape[1] // 2
    out = _bf16_out((rows, width), gate_up.device)
    _check(load().amxfp4_silu_mul(gate_up.data_ptr(), rows, width, out.data_ptr(), _stream()))
    return out


def residual_add(x, y):
    """BF16 x + FP32 y -> BF16, same shape."""
    _need_cuda(x, y)
    assert x.dtype == torch.bfloat16 and y.dtype == torch.float32 and x.is_contiguous() and y.is_contiguous()
    out = _bf16_out(x.shape, x.device)
    _check(load().amxfp4_residual_add(x.data_ptr(), y.data_ptr(), x.numel(), out.data_ptr(), _stream()))
    return out


def merge_heads(o, groups, per_group, seq, head_dim):
    """o [groups, per_group * seq, head_dim] FP32 -> BF16 [seq, groups * per_group * head_dim] (token-major)."""
    _need_cuda(o)
    assert o.dtype == torch.float32 and o.is_contiguous()
    out = _bf16_out((seq, groups * per_group * head_dim), o.device)
    _check(load().amxfp4_merge_heads(o.data_ptr(), groups, per_group, seq, head_dim, out.data_ptr(), _stream()))
    return out
