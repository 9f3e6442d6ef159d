"""Device side of the seeded input generator: fills torch bf16 tensors in place through
libflux_synth.so (test and bench infrastructure; holds none of the method's arithmetic).

The values are bit-identical to `synth.normal_bf16` for the same (seed, stream, counter)."""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import synth

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libflux_synth.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_07394_amd.build`")
_lib = C.CDLL(LIB_PATH)
_lib.synth_fill_normal_bf16.argtypes = [C.c_void_p] + [C.c_longlong] * 7 + [C.c_ulonglong, C.c_ulonglong,
                                                                              C.c_void_p, C.c_int, C.c_void_p]
_lib.synth_fill_normal_bf16.restype = C.c_int


def fill_normal_bf16(t: torch.Tensor, seed: int, stream: int, scale: torch.Tensor | None = None,
                     scale_axis: int = 0, counter0: int = 0) -> None:
    """Fill a 4-D bf16 CUDA tensor (last axis contiguous, a multiple of 8 long) with scale * N(0,1).

    Element (i0,i1,i2,i3) takes counter ``counter0`` + its row-major index in ``t.shape``.
    ``scale``: optional fp32 CUDA vector indexed along ``scale_axis``.
    """
    assert t.dtype == torch.bfloat16 and t.is_cuda and t.dim() == 4 and t.stride(3) == 1
    if scale is not None:
        assert scale.dtype == torch.float32 and scale.is_cuda and scale.numel() == t.shape[scale_axis]
    n0, n1, n2, n3 = t.shape
    rc = _lib.synth_fill_normal_bf16(t.data_ptr(), n0, n1, n2, n3, t.stride(0), t.stride(1), t.stride(2),
                                     synth.stream_key(seed, stream), counter0,
                                     scale.data_ptr() if scale is not None else None, scale_axis,
                                     torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill_normal_bf16 failed with hipError {rc}")
