"""Helpers shared by the GPU parity tests: host<->device marshalling and the error metric."""

import numpy as np
import torch

from paper_1605_04711_amd import workloads as wl

BF16_TOL = 2e-2      # max relative error of bf16-MFMA paths
FP32_TOL = 1e-5      # max relative error of float32 paths


def to_dev_bf16(a_f32):
    """numpy float32 (bf16-valued) -> CUDA bfloat16 tensor, bit-exact."""
    bits = wl.f32_to_bf16_bits(a_f32).view(np.int16)
    return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(a_f32.shape)


def to_dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host_f64(t):
    """CUDA tensor (bf16 or fp32) -> numpy float64, exact."""
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return wl.bf16_bits_to_f32(bits).astype(np.float64).reshape(t.shape)
    return t.float().cpu().numpy().astype(np.float64)


def packed_to_host(t):
    return t.cpu().numpy().view(np.uint32)


def rel_err(y, ref):
    """max_i |y_i - ref_i| / max(|ref_i|, 1e-2 * rms(ref))."""
    y = np.asarray(y, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    floor = max(1e-2 * rms, 1e-30)
    return float(np.max(np.abs(y - ref) / np.maximum(np.abs(ref), floor))) if ref.size else 0.0
