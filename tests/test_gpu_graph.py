"""The hot calls are plain kernel launches on the caller's stream: a decode step (append + attention for a
few layers: one through the fused call, one through the two calls, one on a ring cache) and the prefill of a layer
(router, append, routed prefill, XA selection, block-sparse prefill) can be captured into a HIP graph once and
replayed, with the program's own eager work between replays.  Every replay is checked against the oracle."""
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


def test_prefill_of_a_layer_replays_from_a_graph(F):
    """Router, append, routed prefill, XA block selection and block-sparse prefill of one layer, captured once and
    replayed for new prompts of the same lengths (the lengths are reset by eager work between the replays): every
    replay against the oracle, and the keep matrix against the matrix of an eager call on the same inputs."""
    B, hq, hkv, d, n_sink, window = 2, 4, 2, 128, 16, 100
    lens = [333, 130]
    T, hidden, inner, pool = sum(lens), hq * d, 16, 10
    nb = (max(lens) + 63) // 64
    ctx = F.flux_create(0, 0)
    cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0, 1)
    cu_dev = torch.tensor([0, lens[0], T], dtype=torch.int32, device="cuda")
    cache = F.KVCache.empty(B, hkv, 400, d)
    seed = 83
    w1b = synth.f32_to_bf16_bits(synth.normal_f32(seed, synth.stream_id(synth.STREAM_W1), np.arange(inner * hidden, dtype=np.uint64))
                                 * np.float32(0.02)).reshape(inner, hidden)
    w2b = synth.f32_to_bf16_bits(synth.normal_f32(seed, synth.stream_id(synth.STREAM_W2), np.arange(2 * inner, dtype=np.uint64))
                                 * np.float32(0.02)).reshape(2, inner)
    w1, w2 = H.bits_to_torch(w1b), H.bits_to_torch(w2b)
    q_in = torch.zeros(T, hq, d, dtype=torch.bfloat16, device="cuda")
    k_in = torch.zeros(T, hkv, d, dtype=torch.bfloat16, device="cuda")
    v_in = torch.zeros(T, hkv, d, dtype=torch.bfloat16, device="cuda")
    mode = torch.zeros(B, dtype=torch.uint8, device="cuda")
    all_sa = torch.zeros(B, dtype=torch.uint8, device="cuda")
    out = torch.zeros(T, hq, d, dtype=torch.float32, device="cuda")
    out_bs = torch.zeros(T, hq, d, dtype=torch.float32, device="cuda")
    keep = torch.zeros(B, hq, nb, nb, dtype=torch.uint8, device="cuda")

    def layer():
        F.flux_router(ctx, q_in.view(T, hidden), cu_dev, B, hidden, pool, w1, None, w2, None, inner, mode)
        F.flux_kv_append(ctx, cache, hkv, d, k_in, v_in, cu_dev, T, max(lens))
        F.flux_attn_prefill(ctx, cfg, q_in, cu_dev, max(lens), max(lens), cache, mode, out)
        F.flux_xa_select(ctx, cfg, q_in, cu_dev, max(lens), max(lens), cache, 16, 0.9, keep, nb, nb)
        F.flux_attn_prefill_blocksparse(ctx, cfg, q_in, cu_dev, max(lens), max(lens), cache, all_sa, keep, hq, nb, nb, out_bs)

    def new_inputs(it):
        qb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_Q, 0, it), (T, hq, d))
        kb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_K, 0, it), (T, hkv, d))
        vb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_V, 0, it), (T, hkv, d))
        q_in.copy_(H.bits_to_torch(qb)); k_in.copy_(H.bits_to_torch(kb)); v_in.copy_(H.bits_to_torch(vb))
        cache.kv_len.zero_()                                     # a new prompt starts from an empty cache
        return qb, kb, vb

    def check(it, bits, keep_eager=None):
        qb, kb, vb = bits
        qf, kf, vf = O.bf16_to_f64(qb), O.bf16_to_f64(kb), O.bf16_to_f64(vb)
        got_keep = keep.cpu().numpy()
        if keep_eager is not None:
            assert np.array_equal(got_keep, keep_eager), f"replay {it}: keep matrix differs from the eager call's"
        off = 0
        for b, n in enumerate(lens):
            lg, m = O.router(qf[off:off + n].reshape(n, hidden), pool, O.bf16_to_f64(w1b), None, O.bf16_to_f64(w2b), None)
            assert abs(lg[0] - lg[1]) >= 1e-6, f"seed {seed}: router margin below 1e-6, pick another seed"
            assert int(mode[b]) == m, f"replay {it}: router decision of sequence {b}"
            ref = O.attention(qf[off:off + n], kf[off:off + n], vf[off:off + n], m, n_sink, window)
            H.assert_close(out[off:off + n].cpu().numpy(), ref, f"replay {it} prefill seq {b}")
            nbb = (n + 63) // 64
            ref = O.attention(qf[off:off + n], kf[off:off + n], vf[off:off + n], FA, 0, 1,
                              block_mask=got_keep[b, :, :nbb, :nbb].astype(bool))
            H.assert_close(out_bs[off:off + n].cpu().numpy(), ref, f"replay {it} block-sparse seq {b}")
            off += n
        assert cache.kv_len.cpu().tolist() == lens

    bits = new_inputs(0)
    layer()                                                      # eager first (also warms everything up before capture)
    torch.cuda.synchronize()
    check(0, bits)
    g = torch.cuda.CUDAGraph()
    bits = new_inputs(1)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        layer()
    for it in range(1, 5):
        if it > 1:
            bits = new_inputs(it)
        layer()                                                  # the eager call on these inputs: its keep matrix is the reference
        torch.cuda.synchronize()
        keep_eager = keep.cpu().numpy().copy()
        keep.zero_(); out.zero_(); out_bs.zero_(); cache.kv_len.zero_()
        scratch = (q_in.float() * 2).sum()                       # unrelated eager work on the same device
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check(it, bits, keep_eager)
        assert torch.isfinite(scratch)
    assert F.flux_last_device_status(ctx) == 0
    F.flux_destroy(ctx)
