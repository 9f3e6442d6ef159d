"""flux_attn_decode_append, a whole decode step of a layer in one launch (append one row per sequence, attend,
merge): bit-identical outputs, cache rows and lengths to flux_kv_append followed by flux_attn_decode, over several
steps in a row (the arrival counters clear themselves), and within the attention tolerance of the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as O
from paper_2604_07394_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

FA, SA = 1, 0


def _filled(F, ctx, seed, lens, cap, hkv, d):
    """Two caches with the same seeded rows and lengths."""
    B, t = len(lens), sum(lens)
    kb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_K), (max(t, 1), hkv, d))
    vb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_V), (max(t, 1), hkv, d))
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device="cuda")
    caches = []
    for _ in range(2):
        c = F.KVCache.empty(B, hkv, cap, d)
        c.k.zero_()
        c.v.zero_()
        if t > 0:
            F.flux_kv_append(ctx, c, hkv, d, H.bits_to_torch(kb), H.bits_to_torch(vb), cu, t, max(lens))
        caches.append(c)
    return caches, kb, vb


def _steps(F, ctx, seed, lens, modes, hq, hkv, d, n_sink, window, steps, out_dtype=1, cap=None, oracle_step=None):
    B = len(lens)
    cap = cap if cap is not None else max(lens) + steps + 3
    (ca, cb), kb, vb = _filled(F, ctx, seed, lens, cap, hkv, d)
    md = torch.tensor(modes, dtype=torch.uint8, device="cuda")
    cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, out_dtype)
    tdt = torch.float32 if out_dtype == 1 else torch.bfloat16
    cu1 = torch.arange(B + 1, dtype=torch.int32, device="cuda")
    cur = list(lens)
    new_rows = []
    for s in range(steps):
        qb = synth.normal_bf16(seed + 100 + s, synth.stream_id(synth.STREAM_QDEC), (B, hq, d))
        knb = synth.normal_bf16(seed + 200 + s, synth.stream_id(synth.STREAM_K), (B, hkv, d))
        vnb = synth.normal_bf16(seed + 300 + s, synth.stream_id(synth.STREAM_V), (B, hkv, d))
        new_rows.append((knb, vnb))
        q, kn, vn = H.bits_to_torch(qb), H.bits_to_torch(knb), H.bits_to_torch(vnb)
        bound = min(max(cur) + 1, cap)
        ref = torch.full((B, hq, d), float("nan"), dtype=tdt, device="cuda")
        got = torch.full((B, hq, d), float("nan"), dtype=tdt, device="cuda")
        F.flux_kv_append(ctx, ca, hkv, d, kn, vn, cu1, B, 1)
        F.flux_attn_decode(ctx, cfg, q, bound, ca, md, ref)
        F.flux_attn_decode_append(ctx, cfg, q, kn, vn, bound, cb, md, got)
        torch.cuda.synchronize()
        cur = [min(n + 1, cap) for n in cur]
        assert torch.equal(ref, got), f"step {s}: fused output differs from append + decode"
        assert torch.equal(ca.kv_len, cb.kv_len) and ca.kv_len.tolist() == cur, f"step {s}: lengths"
        assert torch.equal(ca.k, cb.k) and torch.equal(ca.v, cb.v), f"step {s}: cache rows differ"
        if oracle_step == s:
            kf, vf = O.bf16_to_f64(kb), O.bf16_to_f64(vb)
            qf = O.bf16_to_f64(qb)
            off = 0
            for b, n in enumerate(lens):
                ks = [kf[off:off + n]] + [O.bf16_to_f64(r[0])[b][None] for r in new_rows]
                vs = [vf[off:off + n]] + [O.bf16_to_f64(r[1])[b][None] for r in new_rows]
                want = O.attention(qf[b][None], np.concatenate(ks), np.concatenate(vs), modes[b], n_sink, window)[0]
                H.assert_close(got[b].float().cpu().numpy(), want, f"fused decode seq {b} (len {n} + {s + 1})")
                off += n
    return ca, cb


@pytest.fixture(scope="module")
def lib():
    from paper_2604_07394_amd import binding as F
    ctx = F.flux_create(0, 0)
    yield F, ctx
    F.flux_destroy(ctx)


def test_fused_step_equals_append_then_decode_mixed_batch(lib):
    F, ctx = lib
    # several chunks per pair, ragged lengths, both modes, a sequence that starts empty
    _steps(F, ctx, 11, [5000, 2300, 0, 700, 63, 64], [FA, SA, FA, SA, FA, SA], 8, 2, 128, 16, 512, steps=4,
           oracle_step=2)


def test_fused_step_head_dim_64_single_head_and_bf16_out(lib):
    F, ctx = lib
    _steps(F, ctx, 12, [900, 130, 31], [SA, FA, SA], 7, 1, 64, 4, 100, steps=3, out_dtype=0, oracle_step=1)


def test_fused_step_more_than_16_heads_per_kv_head(lib):
    F, ctx = lib
    # 20 query heads per KV head: two query blocks per pair, both attend to the appended row
    _steps(F, ctx, 13, [300, 1500], [FA, SA], 40, 2, 128, 8, 256, steps=2, oracle_step=1)


def test_fused_step_lengths_on_block_edges(lib):
    F, ctx = lib
    # the appended row is the first key of a 32-key block, the last one, and the only key
    _steps(F, ctx, 14, [32, 31, 0, 255, 256, 4224, 4223], [FA, FA, SA, SA, FA, SA, SA], 8, 2, 128, 128, 4096, steps=3,
           oracle_step=0)


def test_fused_step_full_cache_drops_the_row_and_reports(lib):
    F, ctx = lib
    assert F.flux_last_device_status(ctx) == 0
    ca, cb = _steps(F, ctx, 15, [100, 40], [FA, SA], 8, 2, 128, 4, 16, steps=2, cap=101)
    # sequence 0 was full after the first step: the second row was dropped by both paths
    assert ca.kv_len.tolist() == [101, 42]
    assert F.flux_last_device_status(ctx) == F.FLUX_DEV_KV_OVERFLOW


def test_fused_step_long_lists_nontemporal_path(lib):
    F, ctx = lib
    # enough K/V bytes for the streaming (nontemporal) instantiation: batch 4 x 8 KV heads x 70000 keys x 512 B
    B, hq, hkv, d, n = 4, 32, 8, 128, 70000
    cap = n + 8
    cfg = F.attn_cfg(hq, hkv, d, 128, 4096, 0.0, 1)
    from paper_2604_07394_amd import synth_gpu
    outs = []
    lens0 = [n, n - 1, n - 777, 5]
    kn = torch.empty(1, B, hkv, d, dtype=torch.bfloat16, device="cuda")
    vn = torch.empty(1, B, hkv, d, dtype=torch.bfloat16, device="cuda")
    q = torch.empty(1, B, hq, d, dtype=torch.bfloat16, device="cuda")
    synth_gpu.fill_normal_bf16(kn, 21, 1)
    synth_gpu.fill_normal_bf16(vn, 21, 2)
    synth_gpu.fill_normal_bf16(q, 21, 3)
    kn, vn, q = kn[0], vn[0], q[0]
    md = torch.tensor([FA, SA, FA, FA], dtype=torch.uint8, device="cuda")
    cu1 = torch.arange(B + 1, dtype=torch.int32, device="cuda")
    for fused in (False, True):
        c = F.KVCache.empty(B, hkv, cap, d)
        synth_gpu.fill_normal_bf16(c.k, 22, 1)
        synth_gpu.fill_normal_bf16(c.v, 22, 2)
        c.kv_len.copy_(torch.tensor(lens0, dtype=torch.int32))
        out = torch.empty(B, hq, d, dtype=torch.float32, device="cuda")
        for _ in range(2):
            if fused:
                F.flux_attn_decode_append(ctx, cfg, q, kn, vn, n + 2, c, md, out)
            else:
                F.flux_kv_append(ctx, c, hkv, d, kn, vn, cu1, B, 1)
                F.flux_attn_decode(ctx, cfg, q, n + 2, c, md, out)
        torch.cuda.synchronize()
        outs.append((out, c.kv_len.clone(), c.k[:, :, n - 2:n + 3].clone()))
    assert torch.equal(outs[0][0], outs[1][0])
    assert torch.equal(outs[0][1], outs[1][1]) and outs[1][1].tolist() == [m + 2 for m in lens0]
    assert torch.equal(outs[0][2], outs[1][2])
    assert F.flux_last_device_status(ctx) == 0
