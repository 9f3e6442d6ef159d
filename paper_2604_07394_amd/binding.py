"""ctypes binding of libflux.so: the same entry points as include/flux.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs inside the HIP library.
Importing this module loads the in-tree library and fails loudly if it has not been built
(`python -m paper_2604_07394_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libflux.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_07394_amd.build` "
                      "(there is no fallback path)")
_lib = C.CDLL(LIB_PATH)

FLUX_OK, FLUX_EINVAL, FLUX_ECAPACITY, FLUX_EWORKSPACE, FLUX_EHIP, FLUX_ENOMEM = 0, -1, -2, -3, -4, -5
FLUX_DEV_KV_OVERFLOW, FLUX_DEV_BAD_LENGTH = 1, 2
FA, SA = 1, 0

EXPORTS = ["flux_create", "flux_destroy", "flux_strerror", "flux_workspace_needed", "flux_last_device_status",
           "flux_router", "flux_kv_append", "flux_attn_prefill", "flux_attn_decode",
           "flux_kv_append_ring", "flux_kv_compact_ring", "flux_attn_decode_ring", "flux_attn_decode_static",
           "flux_attn_prefill_blocksparse", "flux_xa_select", "flux_attn_decode_append"]
STATIC_SCRATCH_BYTES = 16 * 1024 * 1024 + 256


class FluxAttnCfg(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("n_sink", C.c_int32), ("window", C.c_int32), ("softmax_scale", C.c_float),
                ("out_dtype", C.c_int32), ("sa_block", C.c_int32)]


class FluxKVCache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_t", C.c_int64),
                ("kv_len", C.c_void_p), ("batch", C.c_int32), ("capacity", C.c_int32)]


_lib.flux_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_size_t]
_lib.flux_create.restype = C.c_int
_lib.flux_destroy.argtypes = [C.c_void_p]
_lib.flux_destroy.restype = C.c_int
_lib.flux_strerror.argtypes = [C.c_int]
_lib.flux_strerror.restype = C.c_char_p
_lib.flux_workspace_needed.argtypes = [C.POINTER(FluxAttnCfg), C.c_int, C.c_int]
_lib.flux_workspace_needed.restype = C.c_size_t
_lib.flux_last_device_status.argtypes = [C.c_void_p, C.c_void_p]
_lib.flux_last_device_status.restype = C.c_int
_lib.flux_router.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.flux_router.restype = C.c_int
_lib.flux_kv_append.argtypes = [C.c_void_p, C.POINTER(FluxKVCache), C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_int, C.c_int, C.c_void_p]
_lib.flux_kv_append.restype = C.c_int
_lib.flux_attn_prefill.argtypes = [C.c_void_p, C.POINTER(FluxAttnCfg), C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                   C.POINTER(FluxKVCache), C.c_void_p, C.c_void_p, C.c_void_p]
_lib.flux_attn_prefill.restype = C.c_int
_lib.flux_attn_prefill_blocksparse.argtypes = [C.c_void_p, C.POINTER(FluxAttnCfg), C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                               C.POINTER(FluxKVCache), C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                               C.c_void_p, C.c_void_p]
_lib.flux_attn_prefill_blocksparse.restype = C.c_int
_lib.flux_xa_select.argtypes = [C.c_void_p, C.POINTER(FluxAttnCfg), C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                C.POINTER(FluxKVCache), C.c_int, C.c_float, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
_lib.flux_xa_select.restype = C.c_int
_lib.flux_attn_decode.argtypes = [C.c_void_p, C.POINTER(FluxAttnCfg), C.c_void_p, C.c_int, C.POINTER(FluxKVCache),
                                  C.c_void_p, C.c_void_p, C.c_void_p]
_lib.flux_attn_decode.restype = C.c_int
_lib.flux_attn_decode_append.argtypes = [C.c_void_p, C.POINTER(FluxAttnCfg), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                         C.POINTER(FluxKVCache), C.c_void_p, C.c_void_p, C.c_void_p]
_lib.flux_attn_decode_append.restype = C.c_int
_lib.flux_attn_decode_static.argtypes = [C.POINTER(FluxAttnCfg), C.c_void_p, C.c_int, C.POINTER(FluxKVCache), C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
_lib.flux_attn_decode_static.restype = C.c_int
_lib.flux_kv_append_ring.argtypes = [C.c_void_p, C.POINTER(FluxKVCache), C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
_lib.flux_kv_append_ring.restype = C.c_int
_lib.flux_kv_compact_ring.argtypes = [C.c_void_p, C.POINTER(FluxKVCache), C.POINTER(FluxKVCache), C.c_int, C.c_int,
                                      C.c_int, C.c_int, C.c_void_p]
_lib.flux_kv_compact_ring.restype = C.c_int
_lib.flux_attn_decode_ring.argtypes = [C.c_void_p, C.POINTER(FluxAttnCfg), C.c_void_p, C.POINTER(FluxKVCache),
                                       C.c_void_p, C.c_void_p]
_lib.flux_attn_decode_ring.restype = C.c_int


class FluxError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"flux error {code}: {flux_strerror(code)}")


def _check(rc: int) -> None:
    if rc != FLUX_OK:
        raise FluxError(rc)


def _ptr(t) -> int | None:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def flux_strerror(code: int) -> str:
    return _lib.flux_strerror(code).decode()


def flux_create(device: int = 0, workspace_bytes: int = 0) -> int:
    """Returns the opaque context handle.  device < 0: a device-less context for argument checks."""
    h = C.c_void_p()
    _check(_lib.flux_create(C.byref(h), device, workspace_bytes))
    return h.value


def flux_destroy(ctx: int) -> None:
    _check(_lib.flux_destroy(ctx))


def attn_cfg(n_q_heads, n_kv_heads, head_dim, n_sink, window, softmax_scale=0.0, out_dtype=0, sa_block=0) -> FluxAttnCfg:
    return FluxAttnCfg(n_q_heads, n_kv_heads, head_dim, n_sink, window, softmax_scale, out_dtype, sa_block)


def flux_workspace_needed(cfg: FluxAttnCfg, batch: int, max_kv_len: int) -> int:
    return _lib.flux_workspace_needed(C.byref(cfg), batch, max_kv_len)


def flux_last_device_status(ctx: int, stream=None) -> int:
    rc = _lib.flux_last_device_status(ctx, _stream(stream))
    if rc < 0:
        raise FluxError(rc)
    return rc


@dataclass
class KVCache:
    """One layer's cache: torch tensors k, v [B, Hkv, capacity, D] bf16 (any strides with D contiguous)
    and kv_len int32 [B].  Plain device memory; all reads and writes happen in the library."""
    k: torch.Tensor
    v: torch.Tensor
    kv_len: torch.Tensor

    @classmethod
    def empty(cls, batch, n_kv_heads, capacity, head_dim, device="cuda"):
        k = torch.empty(batch, n_kv_heads, capacity, head_dim, dtype=torch.bfloat16, device=device)
        v = torch.empty_like(k)
        return cls(k, v, torch.zeros(batch, dtype=torch.int32, device=device))

    def c_struct(self) -> FluxKVCache:
        assert self.k.stride() == self.v.stride() and self.k.stride(3) == 1
        b, _, cap, _ = self.k.shape
        return FluxKVCache(self.k.data_ptr(), self.v.data_ptr(), self.k.stride(0), self.k.stride(1),
                           self.k.stride(2), self.kv_len.data_ptr(), b, cap)


def _cache_struct(cache) -> FluxKVCache:
    return cache if isinstance(cache, FluxKVCache) else cache.c_struct()


def flux_router(ctx, x, cu_seqlens, batch, hidden, pool, w1, b1, w2, b2, inner, mode_out, logits_out=None,
                stream=None) -> None:
    _check(_lib.flux_router(ctx, _ptr(x), _ptr(cu_seqlens), batch, hidden, pool, _ptr(w1), _ptr(b1), _ptr(w2),
                            _ptr(b2), inner, _ptr(mode_out), _ptr(logits_out), _stream(stream)))


def flux_kv_append(ctx, cache, n_kv_heads, head_dim, k_new, v_new, cu_new, total_new, max_new, stream=None) -> None:
    cs = _cache_struct(cache)
    _check(_lib.flux_kv_append(ctx, C.byref(cs), n_kv_heads, head_dim, _ptr(k_new), _ptr(v_new), _ptr(cu_new),
                               total_new, max_new, _stream(stream)))


def flux_attn_prefill(ctx, cfg, q, cu_q, max_q_len, max_kv_len, cache, mode, out, stream=None) -> None:
    cs = _cache_struct(cache)
    _check(_lib.flux_attn_prefill(ctx, C.byref(cfg), _ptr(q), _ptr(cu_q), max_q_len, max_kv_len, C.byref(cs),
                                  _ptr(mode), _ptr(out), _stream(stream)))


def flux_attn_prefill_blocksparse(ctx, cfg, q, cu_q, max_q_len, max_kv_len, cache, mode, block_mask, mask_heads,
                                  n_qblocks, n_kblocks, out, stream=None) -> None:
    cs = _cache_struct(cache)
    _check(_lib.flux_attn_prefill_blocksparse(ctx, C.byref(cfg), _ptr(q), _ptr(cu_q), max_q_len, max_kv_len, C.byref(cs),
                                              _ptr(mode), _ptr(block_mask), mask_heads, n_qblocks, n_kblocks, _ptr(out),
                                              _stream(stream)))


def flux_xa_select(ctx, cfg, q, cu_q, max_q_len, max_kv_len, cache, stride, threshold, block_mask, n_qblocks, n_kblocks,
                   stream=None) -> None:
    cs = _cache_struct(cache)
    _check(_lib.flux_xa_select(ctx, C.byref(cfg), _ptr(q), _ptr(cu_q), max_q_len, max_kv_len, C.byref(cs), stride,
                               threshold, _ptr(block_mask), n_qblocks, n_kblocks, _stream(stream)))


def flux_attn_decode(ctx, cfg, q, max_kv_len, cache, mode, out, stream=None) -> None:
    cs = _cache_struct(cache)
    _check(_lib.flux_attn_decode(ctx, C.byref(cfg), _ptr(q), max_kv_len, C.byref(cs), _ptr(mode), _ptr(out),
                                 _stream(stream)))


def flux_attn_decode_append(ctx, cfg, q, k_new, v_new, max_kv_len, cache, mode, out, stream=None) -> None:
    cs = _cache_struct(cache)
    _check(_lib.flux_attn_decode_append(ctx, C.byref(cfg), _ptr(q), _ptr(k_new), _ptr(v_new), max_kv_len, C.byref(cs),
                                        _ptr(mode), _ptr(out), _stream(stream)))


def flux_attn_decode_static(cfg, q, max_kv_len, cache, mode, out, status=None, stream=None) -> None:
    cs = _cache_struct(cache)
    _check(_lib.flux_attn_decode_static(C.byref(cfg), _ptr(q), max_kv_len, C.byref(cs), _ptr(mode), _ptr(out),
                                        _ptr(status), _stream(stream)))


def flux_kv_append_ring(ctx, ring, n_kv_heads, head_dim, n_sink, window, k_new, v_new, cu_new, total_new, max_new,
                        stream=None) -> None:
    cs = _cache_struct(ring)
    _check(_lib.flux_kv_append_ring(ctx, C.byref(cs), n_kv_heads, head_dim, n_sink, window, _ptr(k_new), _ptr(v_new),
                                    _ptr(cu_new), total_new, max_new, _stream(stream)))


def flux_kv_compact_ring(ctx, src, dst, n_kv_heads, head_dim, n_sink, window, stream=None) -> None:
    ss, ds = _cache_struct(src), _cache_struct(dst)
    _check(_lib.flux_kv_compact_ring(ctx, C.byref(ss), C.byref(ds), n_kv_heads, head_dim, n_sink, window,
                                     _stream(stream)))


def flux_attn_decode_ring(ctx, cfg, q, ring, out, stream=None) -> None:
    cs = _cache_struct(ring)
    _check(_lib.flux_attn_decode_ring(ctx, C.byref(cfg), _ptr(q), C.byref(cs), _ptr(out), _stream(stream)))
