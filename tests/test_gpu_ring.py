"""GPU parity of the sparse-decode residency (Sec. 3.3): ring append, compaction after prefill and
ring decode, through the C ABI, against the oracle's RingKVCache / decode_step_ring.

Cache contents are compared bit for bit (copies), attention outputs to the attention tolerance
(max-abs 1e-2, relative L2 5e-3, fp32 output)."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as O
from paper_2604_07394_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

FA, SA = 1, 0


@pytest.fixture(scope="module")
def F():
    from paper_2604_07394_amd import binding
    return binding


@pytest.fixture(scope="module")
def ctx(F):
    c = F.flux_create(0, 0)
    yield c
    F.flux_destroy(c)


def i32(x):
    return torch.tensor(np.asarray(x), dtype=torch.int32, device="cuda")


def cu(lens):
    return i32(np.concatenate([[0], np.cumsum(lens)]))


class Draw:
    """Seeded bf16 rows, the same bits for the device and for the oracle."""

    def __init__(self, seed, d):
        self.seed, self.d, self.counter = seed, d, 0

    def rows(self, kind, n, heads):
        bits = synth.normal_bf16(self.seed, synth.stream_id(kind), (n, heads, self.d), counter0=self.counter)
        self.counter += n * heads * self.d
        return bits


def ring_rows_equal(F, ring, oring, b):
    """Every row the oracle has written holds the same bits on the device."""
    rows = np.nonzero(oring.pos[b] >= 0)[0]
    kd = H.torch_to_f64(ring.k[b][:, rows]).transpose(1, 0, 2)     # [rows, Hkv, D]
    vd = H.torch_to_f64(ring.v[b][:, rows]).transpose(1, 0, 2)
    return np.array_equal(kd, oring.k[b][rows]) and np.array_equal(vd, oring.v[b][rows])


@pytest.mark.parametrize("d,hq,hkv,n_sink,window", [(128, 8, 2, 16, 200), (64, 4, 4, 0, 96), (128, 7, 1, 5, 33)])
def test_ring_append_and_decode_across_wraparounds(F, ctx, d, hq, hkv, n_sink, window):
    """Ragged batch: a sequence shorter than the sinks, one shorter than the ring, one several rings long.
    A bulk append (more rows than the ring holds for the long one), then single-row decode steps that wrap
    the ring more than once; ring contents bit-exact, outputs against the oracle."""
    B = 3
    lens0 = [max(n_sink // 2, 1), n_sink + window // 2, 3 * (n_sink + window) + 7]
    cap = n_sink + window
    ring = F.KVCache.empty(B, hkv, cap, d)
    ring.k.fill_(float("nan"))
    ring.v.fill_(float("nan"))
    oring = O.RingKVCache(B, hkv, d, n_sink, window)
    cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, 1)
    dr = Draw(71, d)
    kb, vb = dr.rows(synth.STREAM_K, sum(lens0), hkv), dr.rows(synth.STREAM_V, sum(lens0), hkv)
    F.flux_kv_append_ring(ctx, ring, hkv, d, n_sink, window, H.bits_to_torch(kb), H.bits_to_torch(vb), cu(lens0),
                          sum(lens0), max(lens0))
    off = 0
    for b, n in enumerate(lens0):
        oring.append(b, O.bf16_to_f64(kb[off:off + n]), O.bf16_to_f64(vb[off:off + n]))
        off += n
    torch.cuda.synchronize()
    assert ring.kv_len.cpu().tolist() == lens0
    for b in range(B):
        assert ring_rows_equal(F, ring, oring, b), b
    steps = 2 * window + 5 if window < 64 else window // 2 + 40
    one = [1] * B
    for step in range(steps):
        qb = dr.rows(synth.STREAM_Q, B, hq)
        kb, vb = dr.rows(synth.STREAM_K, B, hkv), dr.rows(synth.STREAM_V, B, hkv)
        F.flux_kv_append_ring(ctx, ring, hkv, d, n_sink, window, H.bits_to_torch(kb), H.bits_to_torch(vb), cu(one), B, 1)
        out = torch.full((B, hq, d), float("nan"), dtype=torch.float32, device="cuda")
        F.flux_attn_decode_ring(ctx, cfg, H.bits_to_torch(qb), ring, out)
        ref = O.decode_step_ring(oring, O.bf16_to_f64(qb), O.bf16_to_f64(kb), O.bf16_to_f64(vb))
        torch.cuda.synchronize()
        if step % 7 == 0 or step == steps - 1:
            H.assert_close(out.cpu().numpy(), ref, f"ring decode step {step}")
    assert ring.kv_len.cpu().tolist() == [n + steps for n in lens0]
    for b in range(B):
        assert ring_rows_equal(F, ring, oring, b), b
    assert F.flux_last_device_status(ctx) == 0


def test_prefill_then_compact_then_ring_decode_equals_full_cache_sa_decode(F, ctx):
    """The deployment order: prefill the prompt on a full cache (SA mode), compact to the ring, decode on
    the ring.  Each decode output is compared with the oracle AND with the library's own SA decode on the
    full cache, which reads the same keys from the other layout: those two must agree bit for bit."""
    B, hq, hkv, d, n_sink, window = 2, 8, 2, 128, 32, 256
    lens = [1500, 140]
    full = F.KVCache.empty(B, hkv, 1500 + 300 + 4, d)
    ring = F.KVCache.empty(B, hkv, n_sink + window + 8, d)          # a little spare capacity is allowed
    ofull = O.KVCache(B, hkv, d)
    oring = O.RingKVCache(B, hkv, d, n_sink, window)
    cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, 1)
    dr = Draw(72, d)
    qb = dr.rows(synth.STREAM_Q, sum(lens), hq)
    kb, vb = dr.rows(synth.STREAM_K, sum(lens), hkv), dr.rows(synth.STREAM_V, sum(lens), hkv)
    F.flux_kv_append(ctx, full, hkv, d, H.bits_to_torch(kb), H.bits_to_torch(vb), cu(lens), sum(lens), max(lens))
    out = torch.empty(sum(lens), hq, d, dtype=torch.float32, device="cuda")
    F.flux_attn_prefill(ctx, cfg, H.bits_to_torch(qb), cu(lens), max(lens), max(lens), full,
                        torch.zeros(B, dtype=torch.uint8, device="cuda"), out)
    F.flux_kv_compact_ring(ctx, full, ring, hkv, d, n_sink, window)
    off = 0
    for b, n in enumerate(lens):
        ofull.append(b, O.bf16_to_f64(kb[off:off + n]), O.bf16_to_f64(vb[off:off + n]))
        off += n
    O.compact_to_ring(ofull, oring)
    torch.cuda.synchronize()
    assert ring.kv_len.cpu().tolist() == lens
    for b in range(B):
        assert ring_rows_equal(F, ring, oring, b), b
    sa = torch.zeros(B, dtype=torch.uint8, device="cuda")
    for step in range(300):                                           # wraps the 256-row ring
        qd = dr.rows(synth.STREAM_Q, B, hq)
        kd, vd = dr.rows(synth.STREAM_K, B, hkv), dr.rows(synth.STREAM_V, B, hkv)
        kt, vt, one = H.bits_to_torch(kd), H.bits_to_torch(vd), cu([1] * B)
        F.flux_kv_append(ctx, full, hkv, d, kt, vt, one, B, 1)
        F.flux_kv_append_ring(ctx, ring, hkv, d, n_sink, window, kt, vt, one, B, 1)
        o_ring = torch.empty(B, hq, d, dtype=torch.float32, device="cuda")
        o_full = torch.empty(B, hq, d, dtype=torch.float32, device="cuda")
        F.flux_attn_decode_ring(ctx, cfg, H.bits_to_torch(qd), ring, o_ring)
        F.flux_attn_decode(ctx, cfg, H.bits_to_torch(qd), n_sink + window, full, sa, o_full)
        ref = O.decode_step_ring(oring, O.bf16_to_f64(qd), O.bf16_to_f64(kd), O.bf16_to_f64(vd))
        torch.cuda.synchronize()
        assert torch.equal(o_ring, o_full), step                      # same keys, same order, same arithmetic
        if step % 29 == 0 or step == 299:
            H.assert_close(o_ring.cpu().numpy(), ref, f"ring decode after compaction, step {step}")
    assert F.flux_last_device_status(ctx) == 0


def test_ring_never_reads_rows_it_does_not_own(F, ctx):
    """Spare rows past n_sink + window stay untouched (NaN) and are never read."""
    B, hq, hkv, d, n_sink, window = 1, 8, 2, 128, 8, 64
    ring = F.KVCache.empty(B, hkv, n_sink + window + 16, d)
    ring.k.fill_(float("nan"))
    ring.v.fill_(float("nan"))
    cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, 1)
    dr = Draw(73, d)
    kb, vb = dr.rows(synth.STREAM_K, 500, hkv), dr.rows(synth.STREAM_V, 500, hkv)
    F.flux_kv_append_ring(ctx, ring, hkv, d, n_sink, window, H.bits_to_torch(kb), H.bits_to_torch(vb), cu([500]), 500, 500)
    out = torch.empty(B, hq, d, dtype=torch.float32, device="cuda")
    F.flux_attn_decode_ring(ctx, cfg, H.bits_to_torch(dr.rows(synth.STREAM_Q, B, hq)), ring, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    assert torch.isnan(ring.k[:, :, n_sink + window:].float()).all() and torch.isnan(ring.v[:, :, n_sink + window:].float()).all()
    assert torch.isfinite(ring.k[:, :, :n_sink + window].float()).all()


def test_ring_with_block_granular_mask(F, ctx):
    """Block 64 with 100 sinks and a 200-token window: the ring is filled with the geometry rounded to
    whole blocks (128 + 256 rows); the ring decode must equal the library's block-granular SA decode on the
    full cache bit for bit, and the oracle's block-granular decode within tolerance."""
    B, hq, hkv, d, n_sink, window, block = 2, 8, 2, 128, 100, 200, 64
    rs, rw = 128, 256
    lens = [900, 130]
    full = F.KVCache.empty(B, hkv, 1300, d)
    ring = F.KVCache.empty(B, hkv, rs + rw, d)
    ofull = O.KVCache(B, hkv, d)
    cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, 1, block)
    dr = Draw(74, d)
    kb, vb = dr.rows(synth.STREAM_K, sum(lens), hkv), dr.rows(synth.STREAM_V, sum(lens), hkv)
    F.flux_kv_append(ctx, full, hkv, d, H.bits_to_torch(kb), H.bits_to_torch(vb), cu(lens), sum(lens), max(lens))
    F.flux_kv_compact_ring(ctx, full, ring, hkv, d, rs, rw)
    off = 0
    for b, n in enumerate(lens):
        ofull.append(b, O.bf16_to_f64(kb[off:off + n]), O.bf16_to_f64(vb[off:off + n]))
        off += n
    sa = torch.zeros(B, dtype=torch.uint8, device="cuda")
    for step in range(330):
        qd = dr.rows(synth.STREAM_Q, B, hq)
        kd, vd = dr.rows(synth.STREAM_K, B, hkv), dr.rows(synth.STREAM_V, B, hkv)
        kt, vt, one = H.bits_to_torch(kd), H.bits_to_torch(vd), cu([1] * B)
        F.flux_kv_append(ctx, full, hkv, d, kt, vt, one, B, 1)
        F.flux_kv_append_ring(ctx, ring, hkv, d, rs, rw, kt, vt, one, B, 1)
        o_ring = torch.empty(B, hq, d, dtype=torch.float32, device="cuda")
        o_full = torch.empty(B, hq, d, dtype=torch.float32, device="cuda")
        F.flux_attn_decode_ring(ctx, cfg, H.bits_to_torch(qd), ring, o_ring)
        F.flux_attn_decode(ctx, cfg, H.bits_to_torch(qd), rs + rw, full, sa, o_full)
        torch.cuda.synchronize()
        assert torch.equal(o_ring, o_full), step
        if step % 41 == 0 or step == 329:
            ref = O.decode_step(ofull, O.bf16_to_f64(qd), O.bf16_to_f64(kd), O.bf16_to_f64(vd), [SA] * B, n_sink, window,
                                block=block)
            H.assert_close(o_ring.cpu().numpy(), ref, f"block-granular ring decode step {step}")
        else:
            for b in range(B):
                ofull.append(b, O.bf16_to_f64(kd[b])[None], O.bf16_to_f64(vd[b])[None])
    assert F.flux_last_device_status(ctx) == 0
