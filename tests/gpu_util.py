"""Helpers for the GPU parity tests (host <-> device plumbing only)."""
import numpy as np
import torch


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 CUDA tensor of the same shape."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def rnd_bits(shape, seed, scale=1.0):
    from paper_2508_16201_amd.synth import f32_to_bf16_bits
    x = np.random.default_rng(seed).standard_normal(shape).astype(np.float32) * np.float32(scale)
    return f32_to_bf16_bits(x)


# spec tolerances for bf16-in / fp32-accumulate attention against the fp64 oracle
ATTN_MAX_ABS = 2e-2
ATTN_MEAN_ABS = 2e-3


def assert_attn_close(got: torch.Tensor, want: np.ndarray, what=""):
    err = np.abs(host_f64(got) - want)
    assert np.isfinite(err).all(), what
    assert err.max() <= ATTN_MAX_ABS, (what, err.max())
    assert err.mean() <= ATTN_MEAN_ABS, (what, err.mean())
