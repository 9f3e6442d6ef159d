"""Shared plumbing for the GPU parity tests: bf16 bit patterns <-> torch tensors, error metrics."""
import numpy as np
import torch

from oracle import flux_oracle as O
from paper_2604_07394_amd import synth


def bits_to_torch(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the device (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def torch_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def torch_to_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return O.bf16_to_f64(torch_to_bits(t))
    return t.detach().cpu().numpy().astype(np.float64)


def normal_bits(seed, kind, shape, layer=0, step=0, scale=None, scale_axis=None):
    return synth.normal_bf16(seed, synth.stream_id(kind, layer, step), shape, scale, scale_axis)


def errors(got: np.ndarray, ref: np.ndarray):
    """(max abs error, relative L2 error)."""
    diff = got.astype(np.float64) - ref
    return float(np.abs(diff).max()), float(np.sqrt((diff ** 2).sum() / max((ref ** 2).sum(), 1e-300)))


MAX_ABS = 1e-2      # tolerance of the attention outputs against the fp64 oracle (fp32 output)
REL_L2 = 5e-3


def assert_close(got, ref, what=""):
    ma, rl = errors(got, ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert ma <= MAX_ABS and rl <= REL_L2, f"{what}: max-abs {ma:.3e} rel-L2 {rl:.3e}"
    return ma, rl
