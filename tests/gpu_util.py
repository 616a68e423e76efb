"""Shared plumbing of the GPU parity tests: move seeded host arrays to the device, call the library through its
ctypes binding, bring results back."""
import numpy as np
import torch

from paper_2411_09909_amd import binding


def to_dev_bf16(bits):
    """uint16 BF16 patterns (numpy) -> torch.bfloat16 CUDA tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.uint8)).cuda()


def gpu_quantize(bits, scale, asym, k_axis=-1, baseline=False, group_size=32):
    fmt = binding.make_format(scale, asym, group_size)
    c, s = binding.quantize(fmt, to_dev_bf16(bits), k_axis=k_axis, baseline=baseline)
    torch.cuda.synchronize()
    return c.cpu().numpy(), s.cpu().numpy()


def gpu_gemm(ac, as_, bc, bs, scale, asym, baseline=False, group_size=32, options=None):
    """options: binding.gemm_options(...) for a per-call kernel choice (amxfp4_gemm_ex), None for amxfp4_gemm."""
    fmt = binding.make_format(scale, asym, group_size)
    C = binding.gemm(fmt, to_dev_u8(ac), to_dev_u8(as_), to_dev_u8(bc), to_dev_u8(bs), baseline=baseline,
                     options=options)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def rel_fro(C, Cref):
    C = np.asarray(C, np.float64)
    Cref = np.asarray(Cref, np.float64)
    d = np.linalg.norm(Cref)
    return float(np.linalg.norm(C - Cref) / d) if d else float(np.linalg.norm(C))
