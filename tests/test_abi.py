"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header declares, and
rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2411_09909_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in ("amxfp4.h", "amxfp4_layer.h")]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2411_09909_amd import build
        build.build(verbose=False)
    return binding.load()


def declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:amxfp4|mxfp4)_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"amxfp4_quantize", "amxfp4_dequantize", "amxfp4_gemm", "mxfp4_quantize", "mxfp4_dequantize",
            "mxfp4_gemm", "amxfp4_last_error", "amxfp4_codes_bytes", "amxfp4_scales_bytes",
            "amxfp4_gemm_workspace_bytes", "amxfp4_rmsnorm", "amxfp4_split_heads_rope", "amxfp4_softmax_causal",
            "amxfp4_silu_mul", "amxfp4_residual_add", "amxfp4_merge_heads", "amxfp4_rmsnorm_quantize",
            "amxfp4_gemm_silu_mul", "amxfp4_attention", "amxfp4_attention_merged"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_size_queries(lib):
    f = binding.make_format(binding.FP8_E5M2, True)
    assert binding.codes_bytes(f, 64, 1024) == 64 * 512
    assert binding.scales_bytes(f, 64, 1024) == 64 * 32 * 2
    g = binding.make_format(binding.E8M0_FLOOR, False)
    assert binding.scales_bytes(g, 64, 1024) == 64 * 32
    assert binding.codes_bytes(f, 0, 1024) == 0
    # workspace: BF16 panels padded to 256 rows / 128 columns of K
    assert binding.gemm_workspace_bytes(f, 300, 1024, 1024) == (512 + 1024) * 1024 * 2
    assert binding.gemm_workspace_bytes(f, 300, 10, 96, 2) == 2 * (512 + 256) * 128 * 2
    # power-of-two scales with K % 128 == 0 run on the FP4 MFMA with the codes read in place; the workspace holds the
    # scale bytes re-laid per 128 rows (padded to 256) and K stage of 256: 1 KiB each
    assert binding.gemm_workspace_bytes(g, 300, 1024, 1024) == (512 + 1024) // 128 * 4 * 1024
    assert binding.gemm_workspace_bytes(g, 300, 1024, 384, 3) == 3 * (512 + 1024) // 128 * 2 * 1024
    assert binding.gemm_workspace_bytes(g, 64, 1024, 96) == (256 + 1024) * 128 * 2
    # M <= 256 with K % 256 == 0, any scale format: only A's panel (rows padded to 32) and, when K is cut into outer
    # slices (here 4 blocks of 256 -> 4 slices, 8 workgroups each), the partial tiles
    for fmt in (f, g):
        assert binding.gemm_workspace_bytes(fmt, 64, 1024, 1024) == 64 * 1024 * 2 + 4 * 64 * 1024 * 4
        assert binding.gemm_workspace_bytes(fmt, 5, 28672 * 4, 256) == 32 * 256 * 2   # one K block: no slices
        assert binding.gemm_workspace_bytes(fmt, 100, 1024, 1024) == 128 * 1024 * 2 + 4 * 128 * 1024 * 4
        assert binding.gemm_workspace_bytes(fmt, 130, 1024, 1024) == 192 * 1024 * 2 + 4 * 192 * 1024 * 4  # 5 -> 6 row tiles


def test_kernel_options_are_per_call_and_the_workspace_query_is_pure(lib):
    """The kernel choice travels with the call (amx_gemm_options_t): the workspace query is a function of its arguments
    alone, and a query with other options in between does not change what the default query returns."""
    f = binding.make_format(binding.FP8_E5M2, True)
    default = (512 + 1024) * 1024 * 2
    assert binding.gemm_workspace_bytes(f, 300, 1024, 1024) == default
    hybrid = binding.gemm_options(e5m2_kernel="hybrid")   # only the A panel (FP16) lives in the workspace
    assert binding.gemm_workspace_bytes(f, 300, 1024, 1024, options=hybrid) == 512 * 1024 * 2
    assert binding.gemm_workspace_bytes(f, 300, 1024, 96, options=hybrid) == (512 + 1024) * 128 * 2  # K % 128 != 0: panel
    assert binding.gemm_workspace_bytes(f, 300, 1024, 1024, options=binding.gemm_options(e5m2_kernel="fused")) == 0
    assert binding.gemm_workspace_bytes(f, 300, 1024, 1024) == default
    assert binding.gemm_workspace_bytes(f, 300, 1024, 1024, options=binding.gemm_options()) == default
    # asymmetric power-of-two scales: merged FP6 panels sized for the worst case (every group position split in both
    # operands: 2 G K steps of 1536 bytes per 32 rows, padded to a multiple of 12) + anchors + split flags + plan;
    # merged FP8 panels (1 byte per element + anchors); or the sign-split FP4 kernel
    g = binding.make_format(binding.E8M0_FLOOR, True)
    fp6 = 48 * 72 * 1536 + 48 * 18 * 256 + 256 + 256
    assert binding.gemm_workspace_bytes(g, 300, 1024, 1024) == fp6
    merged = (512 + 1024) * 1024 + (512 + 1024) // 32 * (1024 // 256) * 256
    assert binding.gemm_workspace_bytes(g, 300, 1024, 1024, options=binding.gemm_options(pot_kernel="merged_fp8")) == merged
    assert (binding.gemm_workspace_bytes(g, 300, 1024, 1024, options=binding.gemm_options(pot_kernel="split"))
            == (512 + 1024) // 128 * 4 * 2048)   # the sign-split FP4 kernel: re-laid scale pairs only
    # few rows: without that kernel the panel path's workspace; with a forced slice count its partial tiles
    assert binding.gemm_workspace_bytes(f, 64, 1024, 1024, options=binding.gemm_options(few_rows=-1)) == (256 + 1024) * 1024 * 2
    assert binding.gemm_workspace_bytes(f, 64, 1024, 1024, options=binding.gemm_options(few_rows=2)) == 64 * 1024 * 2 + 2 * 64 * 1024 * 4
    assert binding.gemm_workspace_bytes(f, 64, 1024, 1024, options=binding.gemm_options(few_rows=1)) == 64 * 1024 * 2
    # unknown option values: no size, and the call itself is an invalid-argument error before anything is touched
    p = ctypes.c_void_p(0x1000)
    for bad in (binding.AmxGemmOptions(3, 0, 0, 0), binding.AmxGemmOptions(0, 3, 0, 0), binding.AmxGemmOptions(0, 0, 4, 0),
                binding.AmxGemmOptions(0, 0, 0, 17), binding.AmxGemmOptions(0, 0, 0, -2), binding.AmxGemmOptions(-1, 0, 0, 0)):
        assert binding.gemm_workspace_bytes(f, 300, 1024, 1024, options=bad) == 0
        assert lib.amxfp4_gemm_ex(ctypes.byref(f), ctypes.byref(bad), 64, 64, 64, p, p, p, p, p, 64, 1, p, 1 << 30,
                                  None) == -1
        assert b"options" in lib.amxfp4_last_error()
    # NULL options = defaults
    assert lib.amxfp4_gemm_workspace_bytes_ex(ctypes.byref(f), None, 300, 1024, 1024, 1) == default


def test_no_environment_reads_and_no_process_wide_selectors():
    """The boundary keeps no process-wide choice: the sources read no environment variable and export no selector."""
    import glob
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for path in glob.glob(os.path.join(root, "paper_2411_09909_amd", "csrc", "*")):
        text = open(path).read()
        assert "getenv" not in text and "std::atomic" not in text, path
    header = open(os.path.join(root, "include", "amxfp4.h")).read()
    assert "amxfp4_select_" not in header


def _q(lib, fmt, x, rows, K, rs, ks, codes, scales):
    return lib.amxfp4_quantize(ctypes.byref(fmt), x, rows, K, rs, ks, codes, scales, None)


def test_invalid_arguments_are_rejected_on_the_host(lib):
    ok = binding.make_format(binding.FP8_E5M2, True)
    p = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    assert _q(lib, ok, None, 4, 64, 64, 1, p, p) == -1
    assert _q(lib, ok, p, 0, 64, 64, 1, p, p) == -1
    assert _q(lib, ok, p, 4, 48, 48, 1, p, p) == -1          # K not a multiple of the group size
    assert _q(lib, ok, p, 4, 64, 32, 1, p, p) == -1          # row stride shorter than a row
    assert _q(lib, ok, p, 4, 64, 64, 1, ctypes.c_void_p(0x1001), p) == -1   # misaligned codes
    assert _q(lib, ok, p, 4, 64, 3, 2, p, p) == -1           # unsupported stride combination
    assert b"stride" in lib.amxfp4_last_error()
    for bad, code in [(binding.AmxFormat(8, 0, 2, 1), -2), (binding.AmxFormat(48, 0, 2, 1), -2),
                      (binding.AmxFormat(-2, 0, 2, 1), -1),
                      (binding.AmxFormat(32, 1, 2, 1), -1), (binding.AmxFormat(32, 0, 7, 1), -1),
                      (binding.AmxFormat(0, 0, 2, 1), -1), (binding.AmxFormat(32, 0, 2, 5), -1)]:
        assert _q(lib, bad, p, 4, 64, 64, 1, p, p) == code
    assert _q(lib, binding.AmxFormat(128, 0, 2, 1), p, 4, 64, 64, 1, p, p) == -1   # K smaller than one group of 128
    assert _q(lib, binding.AmxFormat(16, 0, 2, 1), p, 4, 48, 48, 1, p, p) == -1    # whole groups of 16, but K % 32 != 0
    assert lib.amxfp4_quantize(None, p, 4, 64, 64, 1, p, p, None) == -1
    # one group per row: along contiguous rows only
    whole = binding.AmxFormat(-1, 0, 2, 1)
    assert _q(lib, whole, p, 4, 64, 1, 4, p, p) == -2 and b"whole-row" in lib.amxfp4_last_error()
    assert lib.amxfp4_scales_bytes(ctypes.byref(whole), 5, 96) == 10
    # size limits: K, rows of a cast, M / N / batch of a GEMM
    big_k = (1 << 20) + 32
    assert _q(lib, ok, p, 4, big_k, big_k, 1, p, p) == -1 and b"maximum" in lib.amxfp4_last_error()
    assert _q(lib, ok, p, 1 << 31, 64, 64, 1, p, p) == -1
    gg = lib.amxfp4_gemm
    assert gg(ctypes.byref(ok), 1 << 21, 64, 64, p, p, p, p, p, 64, 1, p, 1 << 40, None) == -1
    assert gg(ctypes.byref(ok), 64, 1 << 21, 64, p, p, p, p, p, 1 << 21, 1, p, 1 << 40, None) == -1
    assert gg(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 64, 65536, p, 1 << 40, None) == -1
    assert lib.amxfp4_dequantize(ctypes.byref(ok), p, p, 4, 64, p, 2, None) == -1      # bad out_dtype
    # GEMM: workspace too small / missing, ldc < N
    g = lib.amxfp4_gemm
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 64, 1, None, 0, None) == -3
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 64, 1, p, 16, None) == -3
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 32, 1, p, 1 << 30, None) == -1
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 64, 0, p, 1 << 30, None) == -1
    assert lib.mxfp4_gemm(ctypes.byref(ok), 64, 64, 40, p, p, p, p, p, 64, 1, p, 1 << 30, None) == -1


def test_binding_refuses_host_tensors(lib):
    import torch
    f = binding.make_format()
    with pytest.raises(binding.AmxError):
        binding.quantize(f, torch.zeros(4, 64, dtype=torch.bfloat16))


def test_batched_cast_rejects_bad_arguments(lib):
    ok = binding.make_format(binding.FP8_E5M2, True, 32)
    p = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    q = lib.amxfp4_quantize_batched
    assert q(None, p, 2, 4096, 4, 64, 64, 1, p, p, None) == -1
    assert q(ctypes.byref(ok), p, 0, 4096, 4, 64, 64, 1, p, p, None) == -1        # no operand
    assert q(ctypes.byref(ok), p, 65536, 4096, 4, 64, 64, 1, p, p, None) == -1    # too many
    assert b"batch" in lib.amxfp4_last_error()
    assert q(ctypes.byref(ok), p, 2, -8, 4, 64, 64, 1, p, p, None) == -1          # negative batch stride
    assert q(ctypes.byref(ok), p, 2, 4100, 4, 64, 64, 1, p, p, None) == -1        # contiguous: batch stride % 8
    assert q(ctypes.byref(ok), p, 2, 4096, 4, 48, 48, 1, p, p, None) == -1        # K % 32
    assert q(ctypes.byref(ok), p, 2, 4096, 4, 64, 2, 3, p, p, None) == -1         # unsupported strides
    assert q(ctypes.byref(ok), None, 2, 4096, 4, 64, 64, 1, p, p, None) == -1


def test_gated_gemm_rejects_bad_arguments(lib):
    ok = binding.make_format(binding.FP8_E5M2, True, 32)
    p = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    g = lib.amxfp4_gemm_silu_mul
    big = ctypes.c_size_t(1 << 40)
    assert g(None, 64, 64, 64, p, p, p, p, p, 64, p, big, None) == -1
    assert g(ctypes.byref(ok), 64, 48, 64, p, p, p, p, p, 64, p, big, None) == -1      # width % 32
    assert g(ctypes.byref(ok), 64, 64, 48, p, p, p, p, p, 64, p, big, None) == -1      # K % 32
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 32, p, big, None) == -1      # ld_out < width
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, None, 64, p, big, None) == -1   # no output
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 64, None, 0, None) == -3     # no workspace
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, 64, p, 16, None) == -3       # too small
    q = lib.amxfp4_gemm_silu_mul_workspace_bytes
    assert q(ctypes.byref(ok), 64, 64, 64) == (256 + 256) * 128 * 2                    # both BF16 panels, padded
    pot = binding.make_format(binding.E8M0_FLOOR, False, 32)
    assert q(ctypes.byref(pot), 64, 64, 128) == (256 + 256) // 128 * 1024                # FP4 MFMA: re-laid scale bytes only
    assert q(ctypes.byref(ok), 64, 48, 64) == 0 and q(None, 64, 64, 64) == 0


def test_layer_operators_reject_bad_arguments(lib):
    p = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    assert lib.amxfp4_rmsnorm(None, p, 4, 64, 1e-5, p, None) == -1
    assert lib.amxfp4_rmsnorm(p, p, 4, 60, 1e-5, p, None) == -1           # dim % 8
    assert lib.amxfp4_rmsnorm(p, p, 4, 32768, 1e-5, p, None) == -1        # dim too large
    assert lib.amxfp4_split_heads_rope(p, 8, 100, 0, 2, 64, 1, 0, 10000.0, p, None) == -1   # ld < heads * head_dim
    assert lib.amxfp4_split_heads_rope(p, 8, 128, 0, 2, 64, 1, 0, 0.5, p, None) == -1       # theta <= 1
    assert lib.amxfp4_softmax_causal(p, 1, 8, 20, 1.0, p, None) == -1     # cols % 8
    assert lib.amxfp4_silu_mul(p, 4, 6, p, None) == -1
    assert lib.amxfp4_residual_add(p, p, 6, p, None) == -1
    assert lib.amxfp4_merge_heads(p, 2, 2, 8, 6, p, None) == -1
    assert b"merge_heads" in lib.amxfp4_last_error()


def test_fused_normalisation_and_cast_rejects_bad_arguments(lib):
    p = ctypes.c_void_p(4096)
    q = lib.amxfp4_rmsnorm_quantize
    f = binding.make_format(binding.FP8_E5M2, True)
    fr = ctypes.byref(f)
    assert q(None, p, None, None, p, 4, 4096, 1e-5, p, p, None) == -1
    assert q(fr, None, None, None, p, 4, 4096, 1e-5, p, p, None) == -1
    assert q(fr, p, None, None, p, 0, 4096, 1e-5, p, p, None) == -1           # no rows
    assert q(fr, p, None, None, p, 4, 4080, 1e-5, p, p, None) == -1           # dim % group size
    assert q(fr, p, None, None, p, 4, 32768, 1e-5, p, p, None) == -2          # dim too large
    assert q(fr, p, p, None, p, 4, 4096, 1e-5, p, p, None) == -1              # y without sum_out
    assert q(fr, p, None, p, p, 4, 4096, 1e-5, p, p, None) == -1              # sum_out without y
    assert q(fr, ctypes.c_void_p(4104), None, None, p, 4, 4096, 1e-5, p, p, None) == -1   # misaligned x
    g = binding.make_format(binding.FP8_E5M2, True, 128)
    assert q(ctypes.byref(g), p, None, None, p, 4, 4096, 1e-5, p, p, None) == -2          # groups of 128


def test_double_scaling_and_measurement_calls_reject_bad_arguments(lib):
    ok = binding.make_format(binding.FP8_E4M3, True, 16)
    p = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    assert lib.amxfp4_tensor_scale(None, 4, 64, 64, p, None) == -1
    assert lib.amxfp4_tensor_scale(p, 4, 60, 64, p, None) == -1               # K % 8
    assert lib.amxfp4_tensor_scale(p, 4, 64, 32, p, None) == -1               # row stride shorter than a row
    assert lib.amxfp4_tensor_scale(p, 4, 64, 64, ctypes.c_void_p(0x1004), None) == -1   # misaligned pair
    assert lib.amxfp4_quantize_scaled(ctypes.byref(ok), p, 4, 64, 64, 1, None, p, p, None) == -1
    assert b"scale_pair" in lib.amxfp4_last_error()
    assert lib.amxfp4_quantize_scaled(ctypes.byref(ok), p, 4, 48, 48, 1, p, p, p, None) == -1   # K % 32
    assert lib.amxfp4_dequantize_scaled(ctypes.byref(ok), p, p, 4, 64, None, p, None) == -1
    g = lib.amxfp4_gemm_scaled
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, None, p, p, p, p, 64, 1, p, 1 << 30, None) == -1   # one pair missing
    assert g(ctypes.byref(ok), 64, 64, 64, p, p, p, p, p, p, p, 64, 1, None, 0, None) == -3         # no workspace
    assert lib.amxfp4_gemm_scaled_workspace_bytes(ctypes.byref(ok), 64, 1024, 1024, 1) == (256 + 1024) * 1024 * 2
    # a power-of-two format still gets the BF16 workspace when a tensor-wise scale is applied
    pot = binding.make_format(binding.E8M0_FLOOR, False, 32)
    assert lib.amxfp4_gemm_scaled_workspace_bytes(ctypes.byref(pot), 64, 1024, 1024, 1) == (256 + 1024) * 1024 * 2
    flops = ctypes.c_double()
    assert lib.amxfp4_peak_mfma(5, p, 10, p, ctypes.byref(flops), None) == -1
    assert lib.amxfp4_peak_mfma(0, p, 0, p, ctypes.byref(flops), None) == -1
    assert lib.amxfp4_peak_copy(p, p, 24, None) == -1


def test_attention_rejects_bad_arguments(lib):
    ok = binding.make_format(binding.FP8_E5M2, True, 32)
    p = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    a = lib.amxfp4_attention

    def call(fmt, hq, hkv, sq, sk, d, causal=1, scale=0.1, ws=p, ws_bytes=1 << 40):
        return a(ctypes.byref(fmt), hq, hkv, sq, sk, d, p, p, p, p, p, p, scale, causal, p, ws, ws_bytes, None)

    assert call(ok, 4, 3, 64, 64, 128) == -1            # query heads not a multiple of key/value heads
    assert call(ok, 4, 2, 64, 48, 128) == -1            # Sk % 32
    assert call(ok, 4, 2, 64, 32, 128) == -1            # causal with fewer keys than queries
    assert call(ok, 4, 2, 64, 64, 32) == -2             # head size (128 and 64 are built)
    assert call(binding.make_format(binding.FP8_E5M2, True, 16), 4, 2, 64, 64, 128) == -2   # group size
    assert call(ok, 4, 2, 64, 64, 128, scale=0.0) == -1
    assert call(ok, 4, 2, 64, 64, 128, causal=2) == -1
    assert call(ok, 4, 2, 64, 64, 128, ws=None, ws_bytes=0) == -3
    assert call(ok, 4, 2, 64, 64, 128, ws_bytes=16) == -3
    need = lib.amxfp4_attention_workspace_bytes(ctypes.byref(ok), 4, 2, 50, 96, 128)
    assert need == (4 * 64 + 2 * 96 + 2 * 128) * 128 * 2   # Q rows padded to 32, V keys padded to 64
    assert lib.amxfp4_attention_workspace_bytes(ctypes.byref(ok), 4, 2, 50, 96, 32) == 0
