#!/usr/bin/env python3
"""Benchmark of the AMXFP4 hot path on one MI355X: direct-cast quantization of the activations + fully quantized
GEMM against pre-cast weights, on the 70B-shaped up-projection X[4096 x 8192] . W[28672 x 8192]^T (group 32,
FP8-E5M2 asymmetric scales). One "step" = amxfp4_quantize(X) + amxfp4_gemm(Xq, Wq). Weights are static in inference,
so their cast is done once outside the timed region and reported separately.

Prints ONE JSON line: the whole-job throughput 2*M*N*K / t_step in TFLOP/s, a roofline object for the dominant
kernel (the BF16 MFMA GEMM main loop, timed with HIP events recorded by the library around that kernel) and the CPU
oracle timed on a bounded sample of the same workload on this machine's host cores.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOAD = "c3_70b_up_4096x8192x28672"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense BF16 MFMA
PEAK_FP4_TFLOPS = 10100.0   # MI355X dense block-scaled FP4 MFMA (the metric's reference peak)
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense block-scaled FP8 MFMA
# HBM bytes per GEMM-kernel launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), see
# profiles/gemm_bf16_c3_up_counters.md.
MEASURED_TRAFFIC_BYTES = 3.31e9  # 2.84 GB fetched + 0.47 GB written
# the few-rows kernel on c3_70b_up_32tokens_32x8192x28672 (profiles/gemm_skinny_c3_up_32tokens_kernel_trace.md):
# FETCH_SIZE 139.8 MB + WRITE_SIZE 3.7 MB per launch
MEASURED_TRAFFIC_FEW_ROWS = 143.5e6
# the GEMM kernels of the block-scaled variants on the headline workload, same counters
# (profiles/gemm_fp4_c3_up_counters.md, profiles/gemm_fp6m_c3_up_counters.md)
MEASURED_TRAFFIC_VARIANTS = {"mxfp4_e8m0": 0.749e9 + 0.470e9, "amxfp4_e8m0": 1.138e9 + 0.470e9}


# format name -> (scale kind, asymmetric, MFMA type issued by the GEMM, its dense peak in TFLOP/s)
FORMATS = {
    "amxfp4_e5m2": (2, True, "bf16", PEAK_BF16_TFLOPS),    # the paper's AMXFP4: FP8-E5M2 asymmetric scales
    "mxfp4_e5m2": (2, False, "bf16", PEAK_BF16_TFLOPS),    # the paper's "MXFP4" rows: FP8-E5M2 symmetric scale
    "mxfp4_e8m0": (0, False, "fp4", PEAK_FP4_TFLOPS),      # OCP MXFP4 (power-of-two scale, exponent floored)
    "amxfp4_e8m0": (0, True, "fp6", PEAK_FP4_TFLOPS),      # asymmetric power-of-two scales merged into FP6 (FP4 rate)
    "amxfp4_e4m3": (3, True, "bf16", PEAK_BF16_TFLOPS),    # the 4-exponent-bit FP8 scale of the paper's Sec. 4.2
    # Sec. 5.3 double scaling: groups of 16, E4M3 group scale, tensor-wise FP32 scale (its amax pass is in the step)
    "nvfp4": (3, False, "bf16", PEAK_BF16_TFLOPS),
    "anvfp4": (3, True, "bf16", PEAK_BF16_TFLOPS),
}
DOUBLE_SCALED = ("nvfp4", "anvfp4")


class HipEvents:
    """Raw hipEvent_t pairs (the library records them around its GEMM kernel on the launch stream)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so.7" if sys.platform.startswith("linux") else "amdhip64")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0 and self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.pairs[i][0], self.pairs[i][1])
        assert rc == 0, "hipEventElapsedTime failed: %d" % rc
        return ms.value

    def destroy(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def fp6_patterns(torch, codes):
    """Packed E2M1 codes (two per byte) -> the same values as packed E3M2 patterns (four per three bytes, little
    endian), for the FP6 peak probe only."""
    table = torch.tensor([0, 8, 12, 14, 16, 18, 20, 22], dtype=torch.int32, device=codes.device)
    nib = torch.stack((codes & 15, codes >> 4), dim=-1).flatten().to(torch.int64)
    six = (table[nib & 7] | ((nib >> 3) << 5).to(torch.int32)).view(-1, 4)
    word = six[:, 0] | (six[:, 1] << 6) | (six[:, 2] << 12) | (six[:, 3] << 18)
    return torch.stack((word & 255, (word >> 8) & 255, (word >> 16) & 255), dim=-1).flatten().to(torch.uint8)


def measured_peaks(binding, torch, xd, wd, dev, iterations=30000):
    """What this machine sustains, beside the datasheet peaks: register-resident MFMA loops (no memory traffic) on
    all-zero operands and on operand bits taken from the workload (quantized X and W of the bench: dequantized BF16
    values, the same rounded to FP8-E5M2, and the packed FP4 codes), and a 1 GiB streaming copy."""
    fmt = binding.make_format(binding.FP8_E5M2, True)
    rows = 256 * 16 // (xd.shape[1] // 2) + 1   # enough rows for 256 lanes x 16 bytes of codes
    xc, xs = binding.quantize(fmt, xd[:max(rows, 8)])
    wc, ws = binding.quantize(fmt, wd[:max(rows, 8)])
    xh = binding.dequantize(fmt, xc, xs, torch.bfloat16).flatten()
    wh = binding.dequantize(fmt, wc, ws, torch.bfloat16).flatten()

    def lanes(a_bytes, b_bytes, width):
        buf = torch.zeros((256, 64), dtype=torch.uint8, device=dev)
        buf[:, 0:width] = a_bytes[:256 * width].view(256, width)
        buf[:, 32:32 + width] = b_bytes[:256 * width].view(256, width)
        return buf

    operands = {
        "bf16": lanes(xh.view(torch.uint8), wh.view(torch.uint8), 16),
        # the same values in FP16, each operand biased by 2^-3 as the kernels that use the FP16 MFMA hold them
        "f16": lanes((xh.float() * 0.125).to(torch.float16).view(torch.uint8),
                     (wh.float() * 0.125).to(torch.float16).view(torch.uint8), 16),
        "fp8": lanes(xh.to(torch.float8_e5m2).view(torch.uint8), wh.to(torch.float8_e5m2).view(torch.uint8), 32),
        "fp4": lanes(xc.flatten(), wc.flatten(), 16),
        # the same codes as FP6 (E3M2) patterns, as the merged kernel for asymmetric power-of-two scales holds them
        "fp6": lanes(fp6_patterns(torch, xc.flatten()), fp6_patterns(torch, wc.flatten()), 24),
    }
    zeros = torch.zeros((256, 64), dtype=torch.uint8, device=dev)
    sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    res = {"unit": "TFLOP/s", "mfma_loop": {}}
    for kind, datasheet in (("bf16", PEAK_BF16_TFLOPS), ("f16", PEAK_BF16_TFLOPS), ("fp8", PEAK_FP8_TFLOPS),
                            ("fp6", PEAK_FP4_TFLOPS), ("fp4", PEAK_FP4_TFLOPS)):
        row = {"datasheet": datasheet}
        for label, op in (("zero_operands", zeros), ("workload_operands", operands[kind])):
            binding.peak_mfma(kind, op, 200, sink)  # module load, not timed
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            flops = binding.peak_mfma(kind, op, iterations, sink)
            e1.record()
            torch.cuda.synchronize()
            row[label] = round(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
        res["mfma_loop"][kind] = row
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    binding.peak_copy(src, dst)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        binding.peak_copy(src, dst)
    e1.record()
    torch.cuda.synchronize()
    res["copy_1GiB"] = {"GB_per_s_read_plus_write": round(5 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1),
                        "datasheet": 8000.0}
    return res


def other_workloads():
    """The other benchmark configurations, a few steps each, so that their figures are measured in the same run as the
    headline: the attention workload (32 heads x 4096, fused call and the materialised sequence), one new token
    against 8192 cached keys (decode call), and the LLaMA-3-8B-shaped decoder layer at 8192 tokens in AMXFP4 against
    the MXFP4 baselines (time, TFLOP/s over the flops its seven matmuls execute, MSE against a BF16 layer)."""
    import torch
    from paper_2411_09909_amd import attention_bench, decode_bench, layer_bench
    res = {}
    a = attention_bench.run(steps=5)
    res["attention_32_heads_x_4096"] = {k: a[k] for k in ("format", "cast_qkv_ms", "fused_ms", "fused_TFLOPs_causal",
                                                           "materialised_total_ms", "speedup_fused")}
    torch.cuda.empty_cache()
    d = decode_bench.run(steps=20, splits=(32, 64))
    res["decode_1_token_x_8192_keys"] = {"format": d["format"], "cache_MB": d["cache_MB"], "decode_us": d["decode"],
                                         "many_queries_kernel_us": d["many_queries_kernel_us"]}
    torch.cuda.empty_cache()
    d = decode_bench.run(batch=16, steps=20, splits=(16, 32))
    res["decode_16_sequences_x_8192_keys"] = {"format": d["format"], "cache_MB": d["cache_MB"], "decode_us": d["decode"],
                                              "many_queries_kernel_us": d["many_queries_kernel_us"]}
    torch.cuda.empty_cache()
    lay = layer_bench.run(steps=5, formats=("amxfp4_e5m2", "amxfp4_e5m2[prepared_w]", "mxfp4_e5m2", "amxfp4_e8m0",
                                            "amxfp4_e8m0[prepared_w]", "mxfp4_e8m0"))
    res["decoder_layer_8192_tokens"] = {
        name: {"ms_per_layer": f["ms_per_layer"], "matmul_TFLOPs": f["matmul_TFLOPs"],
               "mse_over_update": round(f["mse_over_update"], 5)} for name, f in lay["formats"].items()}
    res["decoder_layer_8192_tokens"]["note"] = ("fused attention; TFLOP/s over the 4.125 TFLOP the seven matmuls execute; "
                                                "[prepared_w]: the weights' kernel-private form (BF16 / FP6 panels) written once, not per call")
    torch.cuda.empty_cache()
    return res


def cpu_baseline(x_bits, w_bits, K, sample_m=2048, sample_n=14336):
    """The oracle as it stands (oracle/amxfp4_ref.c: scalar C, FP64 accumulate, OpenMP over rows), timed on a slab of
    the same operands: quantize sample_m rows of X and sample_n rows of W, then the sample_m x sample_n x K GEMM."""
    from oracle import ref
    xs, ws = x_bits[:sample_m], w_bits[:sample_n]
    sample_m, sample_n = xs.shape[0], ws.shape[0]  # (workloads with fewer rows than the sample use all of them)
    ref.lib()  # compile / load outside the timed region
    t0 = time.perf_counter()
    xc, xsc = ref.quantize(xs)
    wc, wsc = ref.quantize(ws)
    ref.gemm(xc, xsc, wc, wsc)
    dt = time.perf_counter() - t0
    flops = 2.0 * sample_m * sample_n * K
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": ref.num_threads(), "kind": "oracle",
            "sample": "cast of X[:%d] and W[:%d] + their %dx%dx%d GEMM, %.1f s" % (sample_m, sample_n, sample_m,
                                                                                   sample_n, K, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps; the chip needs about 0.1 s of this load to settle at its sustained rate")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", default=WORKLOAD)
    ap.add_argument("--format", default="amxfp4_e5m2", choices=sorted(FORMATS),
                    help="operand format of the timed step (default: the paper's AMXFP4)")
    ap.add_argument("--group-size", type=int, default=32, choices=[16, 32, 64, 128],
                    help="elements per scale group (the headline metric is group 32; the others run on the BF16 MFMA)")
    ap.add_argument("--e5m2-kernel", default="panel", choices=["panel", "hybrid", "fused"],
                    help="which of the library's kernels for FP8-E5M2 scales runs the timed GEMM (default: panel)")
    ap.add_argument("--pot-kernel", default="merged_fp6", choices=["merged_fp6", "merged_fp8", "split"],
                    help="which of the library's kernels for asymmetric power-of-two scales runs the timed GEMM")
    ap.add_argument("--variants", action="store_true",
                    help="time every other format and kernel as well (the block-scaled formats are always listed)")
    ap.add_argument("--no-variants", action="store_true", help="only the headline format")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the attention, decoding and decoder-layer workloads reported beside the headline")
    ap.add_argument("--no-cast-bandwidth", action="store_true",
                    help="skip the cast's bandwidth measurement over rotating buffers")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the register-resident MFMA loops and the streaming copy reported as measured_peaks")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (the known-size reference that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2411_09909_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py needs an MI355X", file=sys.stderr)
        sys.exit(1)
    binding.load()
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.workload]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    x_bits, w_bits = synth.linear_operands(args.workload, seed=0)
    xd = torch.from_numpy(x_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    wd = torch.from_numpy(w_bits.view(np.int16)).to(dev).view(torch.bfloat16)

    C = torch.empty((M, N), dtype=torch.float32, device=dev)
    flops = 2.0 * M * N * K

    def run_format(name, steps, warmup, e5m2_kernel="panel", pot_kernel="merged_fp6", prepared=False):
        """Times `steps` steps (cast X + GEMM against pre-cast W) in the given format; returns a dict of timings.
        e5m2_kernel: which of the library's three kernels for FP8-E5M2 scales multiplies; pot_kernel: which of the
        kernels for asymmetric power-of-two scales (both ignored by the other formats). prepared: the GEMM is
        amxfp4_gemm_prepared on weights whose kernel-private form was written once, outside the timed step."""
        kind, asym, mfma, peak = FORMATS[name]
        if name == "amxfp4_e8m0" and pot_kernel == "split":
            mfma, peak = "fp4", PEAK_FP4_TFLOPS
        if name == "amxfp4_e8m0" and pot_kernel == "merged_fp8":
            mfma, peak = "fp8", PEAK_FP8_TFLOPS
        scaled = name in DOUBLE_SCALED
        gs = 16 if scaled else args.group_size
        if gs != 32:
            mfma, peak, e5m2_kernel = "bf16", PEAK_BF16_TFLOPS, "panel"
        if kind == 2 and e5m2_kernel != "panel":
            mfma = "f16"
        opts = None if scaled else binding.gemm_options(e5m2_kernel=e5m2_kernel, pot_kernel=pot_kernel)
        fmt = binding.make_format(kind, asym, gs)
        nsc = (M, K // gs, 2) if asym else (M, K // gs)
        xc = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        xs = torch.empty(nsc, dtype=torch.uint8, device=dev)
        need = (binding.load().amxfp4_gemm_scaled_workspace_bytes(ctypes.byref(fmt), M, N, K, 1) if scaled
                else binding.gemm_workspace_bytes(fmt, M, N, K, options=opts))
        if prepared:
            need = int(binding.load().amxfp4_gemm_prepared_workspace_bytes(ctypes.byref(fmt), M, N, K))
        ws = torch.empty(need, dtype=torch.uint8, device=dev) if need else None
        xp = torch.empty(2, dtype=torch.float32, device=dev) if scaled else None

        def cast_x():
            if scaled:
                binding.tensor_scale(xd, out=xp)
            binding.quantize(fmt, xd, codes=xc, scales=xs, tensor_pair=xp)

        cast_x()  # first launch of these kernels: module load, not timed
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        wp = binding.tensor_scale(wd) if scaled else None
        wc, wsc = binding.quantize(fmt, wd, tensor_pair=wp)  # weights: cast once, outside the timed step
        torch.cuda.synchronize()
        t_cast_w = time.perf_counter() - t0
        w_prepared = binding.prepare_weights(fmt, wc, wsc) if prepared else None
        torch.cuda.synchronize()

        def step(pair=None):
            cast_x()
            if pair is not None:
                binding.profile_next_gemm(pair[0], pair[1])
            if prepared:
                binding.gemm_prepared(fmt, xc, xs, wc, wsc, w_prepared, out=C, workspace=ws)
            else:
                binding.gemm(fmt, xc, xs, wc, wsc, out=C, workspace=ws, a_pair=xp, b_pair=wp, options=opts)

        for _ in range(warmup):
            step()
        ev = HipEvents(steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(ev.pairs[i])
        torch.cuda.synchronize()
        t_total = time.perf_counter() - t0
        kern_ms = sum(ev.elapsed_ms(i) for i in range(steps)) / steps
        ev.destroy()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            cast_x()
        torch.cuda.synchronize()
        t_cast_x = (time.perf_counter() - t0) / steps
        return {"t_step": t_total / steps, "kern_ms": kern_ms, "t_cast_x": t_cast_x, "t_cast_w": t_cast_w,
                "mfma": mfma, "peak": peak, "asym": asym, "workspace_bytes": need,
                "prepared_bytes": w_prepared.numel() if prepared else 0}

    def cast_bandwidth(name, reps=20):
        """The cast of X timed three ways, as GB/s of algorithmic bytes (2 B read + 0.5 B codes + scale bytes per
        element): on ONE buffer re-cast back to back, whose 67 MB stay in the 256 MB last-level cache between launches
        ("cached"); rotating over enough distinct copies of X that more than 512 MB pass between two casts of the
        same buffer, so every read comes from HBM ("hbm"); and the cast of the weights, 470 MB read per launch
        ("weights")."""
        kind, asym, _, _ = FORMATS[name]
        gs = 16 if name in DOUBLE_SCALED else args.group_size
        fmt = binding.make_format(kind, asym, gs)
        x_bytes = M * K * 2
        copies = max(2, -(-(640 << 20) // x_bytes))   # ceil(640 MiB / |X|): 10 copies of the 64 MiB headline X
        xs_rot = [xd.clone() for _ in range(copies)]
        codes = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        scales = torch.empty((M, K // gs, 2) if asym else (M, K // gs), dtype=torch.uint8, device=dev)

        def timed(fn, n):
            fn(0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(n):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / n

        def per_elem(rows):
            return rows * K * 2 + rows * K // 2 + rows * (K // gs) * (2 if asym else 1)

        t_cached = timed(lambda i: binding.quantize(fmt, xd, codes=codes, scales=scales), reps)
        t_hbm = timed(lambda i: binding.quantize(fmt, xs_rot[i % copies], codes=codes, scales=scales), reps * 2)
        wcodes = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
        wscales = torch.empty((N, K // gs, 2) if asym else (N, K // gs), dtype=torch.uint8, device=dev)
        t_w = timed(lambda i: binding.quantize(fmt, wd, codes=wcodes, scales=wscales), 5)
        return {"unit": "GB/s of algorithmic bytes (2.5625 B per element for the asymmetric format)",
                "x_cached": round(per_elem(M) / t_cached / 1e9, 1), "x_cached_us": round(t_cached * 1e6, 2),
                "x_hbm": round(per_elem(M) / t_hbm / 1e9, 1), "x_hbm_us": round(t_hbm * 1e6, 2),
                "x_hbm_rotation": "%d buffers, %.0f MB" % (copies, copies * x_bytes / 1e6),
                "weights": round(per_elem(N) / t_w / 1e9, 1), "weights_us": round(t_w * 1e6, 1),
                "frac_of_hbm_peak": round(per_elem(M) / t_hbm / 1e9 / 8000.0, 4)}

    # The reference measurements come first: the register-resident MFMA loops and the streaming copy, the cast's
    # bandwidth, then the other formats' steps. They also leave the chip in the state it holds under sustained load
    # (its power management takes about 0.1 s of such work to settle, and the settled state is the faster one: in a
    # run with --steps 20 --warmup 5 the same GEMM kernel took 1.335 ms when the headline came before the other
    # formats and 1.302 ms right after), so a short run times what a long one does. The warm-up and timed steps of
    # the headline follow, unchanged.
    peaks = None if args.no_measured_peaks else measured_peaks(binding, torch, xd, wd, dev)
    cast_bw = None if args.no_cast_bandwidth else cast_bandwidth(args.format)
    # The formats that run on the block-scaled matrix instructions are part of every run (about ten steps each): OCP
    # MXFP4 and the asymmetric power-of-two format, each with its GEMM kernel's time and fraction of the peak of the
    # MFMA type it issues. --variants adds the rest.
    cases = [("mxfp4_e8m0", "panel", "merged_fp6", False), ("amxfp4_e8m0", "panel", "merged_fp6", False),
             ("amxfp4_e8m0", "panel", "merged_fp6", True),   # B's merged FP6 panel written once
             ("amxfp4_e8m0", "panel", "merged_fp8", False), ("amxfp4_e8m0", "panel", "split", False)]
    if args.format not in DOUBLE_SCALED and FORMATS[args.format][2] == "bf16":
        # the headline format against weights whose BF16 expansion was written once (amxfp4_gemm_prepared): the step
        # then expands only X; costs 2 bytes per weight element of extra memory
        cases.append((args.format, "panel", "merged_fp6", True))
    if args.variants:
        cases += [(name, "panel", "merged_fp6", False) for name in sorted(FORMATS) if name not in ("mxfp4_e8m0", "amxfp4_e8m0")]
        cases += [(name, k, "merged_fp6", False) for name in ("amxfp4_e5m2", "mxfp4_e5m2") for k in ("hybrid", "fused")]
    if args.no_variants or args.group_size != 32:
        cases = []
    v_steps = max(3, min(args.steps, 10)) if not args.variants else max(3, args.steps // 2)
    v_warm = max(2, min(args.warmup, 5)) if not args.variants else max(2, args.warmup // 2)
    variants = {}
    for name, kern, pot, prep in cases:
        if name == args.format and kern == args.e5m2_kernel and pot == args.pot_kernel and not prep:
            continue
        # (the first of them is where the chip goes from register loops and casts to sustained GEMM load: it gets
        # the warm-up steps that takes)
        v = run_format(name, v_steps, v_warm if variants else max(v_warm, 40), kern, pot, prep)
        label = (name + ("[%s]" % kern if kern != "panel" else "") + ("[%s]" % pot if pot != "merged_fp6" else "")
                 + ("[prepared_w]" if prep else ""))
        variants[label] = {
            "value": round(flops / v["t_step"] / 1e12, 2), "unit": "TFLOP/s",
            "frac_of_fp4_mfma_peak": round(flops / v["t_step"] / 1e12 / PEAK_FP4_TFLOPS, 4),
            "ms_per_step": round(v["t_step"] * 1e3, 4), "steps": v_steps, "mfma": v["mfma"],
            "workspace_MB": round(v["workspace_bytes"] / 1e6, 1), "prepared_weights_MB": round(v["prepared_bytes"] / 1e6, 1),
            "gemm_kernel_ms": round(v["kern_ms"], 4),
            "kernel_frac_of_mfma_peak": round(flops / (v["kern_ms"] * 1e-3) / 1e12 / v["peak"], 4),
            "kernel_traffic_bytes": MEASURED_TRAFFIC_VARIANTS.get(label) if args.workload == WORKLOAD else None}
    r = run_format(args.format, args.steps, args.warmup, args.e5m2_kernel, args.pot_kernel)
    ms_per_step = r["t_step"] * 1e3
    value = flops / r["t_step"] / 1e12
    achieved = flops / (r["kern_ms"] * 1e-3) / 1e12
    scaled = args.format in DOUBLE_SCALED   # the tensor-wise maximum reads X once more
    cast_bytes = (M * K * 2 * (2 if scaled else 1) + M * K // 2 +
                  M * (K // (16 if scaled else args.group_size)) * (2 if r["asym"] else 1))
    kernel_name = "gemm_fp4_kernel" if r["mfma"] == "fp4" else "gemm_fp8m_kernel" if r["mfma"] == "fp8" else "gemm_fp6m_kernel" if r["mfma"] == "fp6" else {"panel": "gemm_bf16_kernel", "hybrid":
                  "gemm_e5m2_hybrid_kernel", "fused": "gemm_e5m2_kernel"}[args.e5m2_kernel if args.group_size == 32 else "panel"]
    if M <= 256 and K % 256 == 0 and args.group_size == 32 and args.format not in DOUBLE_SCALED:
        kernel_name = "gemm_skinny_kernel"  # few rows: B dequantized in registers straight from its codes
    dtype = r["mfma"]
    if kernel_name == "gemm_skinny_kernel":
        dtype = "f16" if FORMATS[args.format][0] == 2 else "bf16"  # the few-rows kernel's MFMA operand type
    if kernel_name == "gemm_skinny_kernel":
        # a few rows against a weight matrix: bound by reading B's codes and scales (plus A's panel and C) from HBM
        kbytes = N * K // 2 + N * (K // 32) * (2 if r["asym"] else 1) + ((M + 31) // 32 * 32) * K * 2 + M * N * 4
        gbps = kbytes / (r["kern_ms"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": round(gbps, 1), "peak": 8000.0, "unit": "GB/s",
                    "frac": round(gbps / 8000.0, 4),
                    "traffic": MEASURED_TRAFFIC_FEW_ROWS if args.format == "amxfp4_e5m2" and args.group_size == 32
                    and args.workload == "c3_70b_up_32tokens_32x8192x28672" else None,
                    "kernel_ms": round(r["kern_ms"], 4),
                    "algorithmic_bytes": kbytes}
    else:
        roofline = {"bound": "mfma", "kernel": kernel_name, "achieved": round(achieved, 2), "peak": r["peak"],
                    "unit": "TFLOP/s", "frac": round(achieved / r["peak"], 4),
                    "traffic": MEASURED_TRAFFIC_BYTES if args.format == "amxfp4_e5m2" and args.workload == WORKLOAD
                    and args.e5m2_kernel == "panel" and args.group_size == 32 else None,
                    "kernel_ms": round(r["kern_ms"], 4)}
    out = {
        "metric": "AMXFP4 cast+GEMM TFLOPS at %dx%dx%d" % (M, K, N), "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": args.workload, "M": M, "N": N, "K": K, "format": args.format, "group_size": 16 if args.format in DOUBLE_SCALED else args.group_size,
                   "tensor_scale": args.format in DOUBLE_SCALED,
                   "e5m2_kernel": ("packed_codes" if kernel_name == "gemm_skinny_kernel" else args.e5m2_kernel)
                   if FORMATS[args.format][0] == 2 and args.group_size == 32 else None,
                   "step": "amxfp4_quantize(X) + amxfp4_gemm(Xq, Wq), W pre-cast"},
        "roofline": roofline,
        "frac_of_fp4_mfma_peak": round(value / PEAK_FP4_TFLOPS, 4),
        "breakdown_ms": {"cast_x": round(r["t_cast_x"] * 1e3, 4),
                         "gemm_call": round(ms_per_step - r["t_cast_x"] * 1e3, 4),
                         "gemm_mfma_kernel": round(r["kern_ms"], 4), "cast_w_once": round(r["t_cast_w"] * 1e3, 3)},
        # the cast inside the timed step re-reads one buffer that the last-level cache holds: a cached figure
        "cast_x_gbps_cached_in_step": round(cast_bytes / r["t_cast_x"] / 1e9, 1),
    }
    if cast_bw is not None:
        out["cast_bandwidth"] = cast_bw
    if variants:
        out["variants"] = variants
    if not (args.no_workloads or args.no_variants or args.workload != WORKLOAD):
        out["workloads"] = other_workloads()
    if peaks is not None:
        out["measured_peaks"] = peaks
    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["calib_copy_bytes"] = 1 << 30
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x_bits, w_bits, K)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
