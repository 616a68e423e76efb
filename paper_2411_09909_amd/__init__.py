"""AMXFP4 / MXFP4 direct-cast quantization and fully quantized GEMM for AMD MI355X (gfx950).

The compute lives in the HIP library built from csrc/ (C ABI declared in include/amxfp4.h); `binding` marshals
arguments to it. `synth` draws the seeded synthetic operands used by tests and the benchmark.
"""
