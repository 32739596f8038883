"""Rounding of fp32 master inputs to the storage types, done once by the harness with
PyTorch's CPU casts so that the GPU library and the CPU oracle receive the same bits."""
import numpy as np
import torch

E4M3_MAX = 448.0


def bf16_bits(a):
    """fp32 array -> uint16 bit patterns of the nearest bfloat16 (ties to even)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def e4m3_scale(a):
    """Per-tensor scale s = amax / 448 (1.0 for an all-zero tensor)."""
    amax = float(np.max(np.abs(a))) if a.size else 0.0
    return amax / E4M3_MAX if amax > 0.0 else 1.0


def e4m3_codes(a, scale):
    """fp32 array -> uint8 codes of sat(RNE(a / scale)) in OCP E4M3 (finite, no inf)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)) / float(scale)
    t = t.clamp_(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn)
    return t.view(torch.uint8).numpy()
