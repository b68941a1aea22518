"""Helpers for the GPU parity tests: torch is used for device memory only."""
import numpy as np
import torch

import synth


def dev_bf16(x_f32: np.ndarray) -> torch.Tensor:
    """Upload fp32 values as bf16 (values are expected to be bf16-representable or are rounded RNE)."""
    bits = synth.f32_to_bf16_bits(x_f32).reshape(x_f32.shape)
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def close(got, ref, atol, rtol):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    err = np.abs(got - ref) - (atol + rtol * np.abs(ref))
    return float(err.max()) <= 0, float(np.abs(got - ref).max())
