"""The hot calls are plain kernel launches on the caller's stream: a decode step (append + attention for a
few layers: one through the fused call, one through the two calls, one on a ring cache) can be captured into a HIP
graph once and replayed, with the program's own eager work between replays.  Every replay is checked against the
oracle."""
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


def test_decode_step_replays_from_a_graph(F):
    B, hq, hkv, d, n_sink, window = 2, 8, 2, 128, 16, 128
    lens = [700, 300]
    n_layers = 3
    modes = [[FA, FA], [SA, FA], None]                       # the last layer lives on a ring cache
    ctx = F.flux_create(0, 0)
    cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, 1)
    cu_b = torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda")
    caches, ocaches = [], []
    seed = 81
    for l in range(n_layers):
        kb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_K, l), (sum(lens), hkv, d))
        vb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_V, l), (sum(lens), hkv, d))
        full = F.KVCache.empty(B, hkv, 800, d)
        F.flux_kv_append(ctx, full, hkv, d, H.bits_to_torch(kb), H.bits_to_torch(vb),
                         torch.tensor([0, lens[0], sum(lens)], dtype=torch.int32, device="cuda"), sum(lens), max(lens))
        of = O.KVCache(B, hkv, d)
        off = 0
        for b, n in enumerate(lens):
            of.append(b, O.bf16_to_f64(kb[off:off + n]), O.bf16_to_f64(vb[off:off + n]))
            off += n
        if modes[l] is None:
            ring = F.KVCache.empty(B, hkv, n_sink + window, d)
            F.flux_kv_compact_ring(ctx, full, ring, hkv, d, n_sink, window)
            caches.append(ring)
        else:
            caches.append(full)
        ocaches.append(of)
    mode_dev = [None if m is None else torch.tensor(m, dtype=torch.uint8, device="cuda") for m in modes]
    # static buffers the graph reads and writes
    q_in = torch.zeros(n_layers, B, hq, d, dtype=torch.bfloat16, device="cuda")
    k_in = torch.zeros(n_layers, B, hkv, d, dtype=torch.bfloat16, device="cuda")
    v_in = torch.zeros(n_layers, B, hkv, d, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(n_layers, B, hq, d, dtype=torch.float32, device="cuda")

    def step():
        for l in range(n_layers):
            if modes[l] is None:
                F.flux_kv_append_ring(ctx, caches[l], hkv, d, n_sink, window, k_in[l], v_in[l], cu_b, B, 1)
                F.flux_attn_decode_ring(ctx, cfg, q_in[l], caches[l], out[l])
            elif l == 0:                                         # the decode step of a layer as one call
                F.flux_attn_decode_append(ctx, cfg, q_in[l], k_in[l], v_in[l], 800, caches[l], mode_dev[l], out[l])
            else:
                F.flux_kv_append(ctx, caches[l], hkv, d, k_in[l], v_in[l], cu_b, B, 1)
                F.flux_attn_decode(ctx, cfg, q_in[l], 800, caches[l], mode_dev[l], out[l])

    def new_inputs(it):
        bits = []
        for l in range(n_layers):
            qb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_QDEC, l, it), (B, hq, d))
            kb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_KDEC, l, it), (B, hkv, d))
            vb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_VDEC, l, it), (B, hkv, d))
            q_in[l].copy_(H.bits_to_torch(qb)); k_in[l].copy_(H.bits_to_torch(kb)); v_in[l].copy_(H.bits_to_torch(vb))
            bits.append((qb, kb, vb))
        return bits

    def check(it, bits):
        for l in range(n_layers):
            qb, kb, vb = bits[l]
            m = [SA, SA] if modes[l] is None else modes[l]
            ref = O.decode_step(ocaches[l], O.bf16_to_f64(qb), O.bf16_to_f64(kb), O.bf16_to_f64(vb), m, n_sink, window)
            H.assert_close(out[l].cpu().numpy(), ref, f"step {it} layer {l}")

    # one eager step first (also warms everything up before capture)
    bits = new_inputs(0)
    step()
    torch.cuda.synchronize()
    check(0, bits)

    g = torch.cuda.CUDAGraph()
    bits = new_inputs(1)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        step()
    # capture does not execute: run the captured step for the inputs that are in place
    g.replay()
    torch.cuda.synchronize()
    check(1, bits)
    for it in range(2, 6):
        bits = new_inputs(it)                                  # eager copies between replays
        scratch = (q_in.float() * 2).sum()                     # unrelated eager work on the same device
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check(it, bits)
        assert torch.isfinite(scratch)
    want = [n + 6 for n in lens]
    for l in range(n_layers):
        assert caches[l].kv_len.cpu().tolist() == want
    assert F.flux_last_device_status(ctx) == 0
    F.flux_destroy(ctx)
