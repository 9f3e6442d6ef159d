"""flux_attn_decode_static, the decode entry point that allocates nothing (its split-K partials live in a
static device array): same results as flux_attn_decode bit for bit, and within the attention tolerance of
the fp64 oracle, on two calls in a row, the second with a smaller input (the array keeps the first call's
contents)."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as O
from paper_2604_07394_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

FA, SA = 1, 0


def _case(F, ctx, seed, lens, modes, hq, hkv, d, n_sink, window):
    B = len(lens)
    cap = max(lens) + 8
    cache = F.KVCache.empty(B, hkv, cap, d)
    t = sum(lens)
    kb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_K), (t, hkv, d))
    vb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_V), (t, hkv, d))
    qb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_QDEC), (B, hq, d))
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device="cuda")
    F.flux_kv_append(ctx, cache, hkv, d, H.bits_to_torch(kb), H.bits_to_torch(vb), cu, t, max(lens))
    md = torch.tensor(modes, dtype=torch.uint8, device="cuda")
    q = H.bits_to_torch(qb)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    res = {}
    for dt, tdt in ((1, torch.float32), (0, torch.bfloat16)):
        cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, dt)
        ref_out = torch.full((B, hq, d), float("nan"), dtype=tdt, device="cuda")
        new_out = torch.full((B, hq, d), float("nan"), dtype=tdt, device="cuda")
        F.flux_attn_decode(ctx, cfg, q, max(lens), cache, md, ref_out)
        F.flux_attn_decode_static(cfg, q, max(lens), cache, md, new_out, status)
        torch.cuda.synchronize()
        assert torch.equal(ref_out, new_out), f"static scratch result differs (out_dtype {dt})"
        res[dt] = new_out
    assert int(status[0]) == 0
    # the oracle, at the attention tolerance
    qf, kf, vf = O.bf16_to_f64(qb), O.bf16_to_f64(kb), O.bf16_to_f64(vb)
    off = 0
    for b, n in enumerate(lens):
        ref = O.attention(qf[b][None], kf[off:off + n], vf[off:off + n], modes[b], n_sink, window)[0]
        H.assert_close(res[1][b].cpu().numpy(), ref, f"static decode seq {b} (len {n})")
        off += n
    return status


def test_static_scratch_decode_two_calls_second_smaller():
    from paper_2604_07394_amd import binding as F
    ctx = F.flux_create(0, 0)
    try:
        # several chunks per pair, mixed modes, then a smaller batch of shorter sequences on the same array
        _case(F, ctx, 91, [5000, 2300, 700, 64], [FA, SA, FA, SA], 8, 2, 128, 16, 512)
        _case(F, ctx, 92, [900, 130], [SA, FA], 7, 1, 64, 4, 100)
        # the device-side clamp reports through the caller's status word: a bound below the visible keys
        cache = F.KVCache.empty(1, 2, 600, 128)
        kb = synth.normal_bf16(93, synth.stream_id(synth.STREAM_K), (600, 2, 128))
        F.flux_kv_append(ctx, cache, 2, 128, H.bits_to_torch(kb), H.bits_to_torch(kb),
                         torch.tensor([0, 600], dtype=torch.int32, device="cuda"), 600, 600)
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        out = torch.empty(1, 8, 128, dtype=torch.float32, device="cuda")
        q = H.bits_to_torch(synth.normal_bf16(93, synth.stream_id(synth.STREAM_QDEC), (1, 8, 128)))
        F.flux_attn_decode_static(F.attn_cfg(8, 2, 128, 4, 64, 0.0, 1), q, 300, cache,
                                  torch.ones(1, dtype=torch.uint8, device="cuda"), out, status)
        torch.cuda.synchronize()
        assert int(status[0]) == F.FLUX_DEV_BAD_LENGTH
        assert F.flux_last_device_status(ctx) == 0                  # the context's own word is untouched
    finally:
        F.flux_destroy(ctx)


def test_static_scratch_rejects_shapes_beyond_the_array():
    from paper_2604_07394_amd import binding as F
    # 16 query heads per KV head: 16 partial rows per unit; 4096 pairs -> far beyond 16 MiB
    cfg = F.attn_cfg(256, 16, 128, 4, 64, 0.0, 1)
    cache = F.FluxKVCache(4096, 8192, 1 << 30, 1 << 26, 128, 256, 256, 1 << 20)
    with pytest.raises(F.FluxError) as e:
        F.flux_attn_decode_static(cfg, 4096, 1 << 20, cache, 512, 1024, None)
    assert e.value.code == F.FLUX_EWORKSPACE
