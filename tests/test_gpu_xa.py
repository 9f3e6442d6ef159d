"""GPU parity of flux_xa_select (the XA block selection: antidiagonal scoring with stride 16, threshold 0.9,
block 64; this build's reading of Sec. 4.1 / Table 3) against the fp64 oracle.

A floating-point sum decides which blocks are kept, so what is compared is what is unique: a block the oracle
keeps at a threshold lowered by 1e-5 (and with the cut mass raised by 1e-5 relative) must be kept, a block the
oracle drops at a threshold raised by 1e-5 (cut mass lowered) must be dropped, and the blocks in between may go
either way; the number of rows that differ at all from the oracle's exact selection is printed and bounded.  The
selection is then used: flux_attn_prefill_blocksparse with the GPU's matrix against the oracle's attention under
the same matrix."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as O
from paper_2604_07394_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

FA, SA = 1, 0
BLK, STRIDE = 64, 16


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
    return torch.tensor(x, dtype=torch.int32, device="cuda")


def cu(lens):
    return i32(np.concatenate([[0], np.cumsum(lens)]))


def envelope(mass_row, bi, threshold, eps=1e-5):
    """(must keep, may keep) for one query block from the oracle's masses."""
    m = mass_row[: bi + 1]
    order = np.argsort(-m, kind="stable")
    csum = np.cumsum(m[order])

    def cut_mass(t):
        c = min(int(np.searchsorted(csum, t * csum[-1], side="left")), bi)
        return m[order[c]]
    must = m >= cut_mass(threshold - eps) * (1 + eps)
    may = m >= cut_mass(min(threshold + eps, 1.0)) * (1 - eps)
    must[bi] = may[bi] = True
    return must, may


def check_selection(got, q, k, hq, group, threshold, rows=None, scale=None):
    """got: bool [hq, n_qb, n_kb] from the GPU for one sequence; q [n, hq, D], k [n, hkv, D] fp64."""
    n = q.shape[0]
    nb = -(-n // BLK)
    differ = total = 0
    for h in range(hq):
        keep, mass = O.xa_select(q[:, h], k[:, h // group], STRIDE, threshold, BLK, scale, return_mass=True, blocks=rows)
        for bi in (range(nb) if rows is None else rows):
            must, may = envelope(mass[bi], bi, threshold)
            g = got[h, bi, : bi + 1]
            assert (g | ~must).all(), f"head {h} query block {bi}: a block that must be kept is missing"
            assert (may | ~g).all(), f"head {h} query block {bi}: a block that must be dropped is kept"
            assert not got[h, bi, bi + 1:].any(), f"head {h} query block {bi}: a block above the diagonal"
            differ += int(not np.array_equal(g, keep[bi, : bi + 1]))
            total += 1
    return differ, total


@pytest.mark.parametrize("d,hq,hkv,threshold", [(128, 8, 2, 0.9), (64, 4, 4, 0.9), (128, 7, 1, 0.5), (128, 4, 2, 0.99)])
def test_xa_selection_ragged_prompts(F, ctx, d, hq, hkv, threshold):
    lens = [1000, 517, 64, 300, 15]
    B, t = len(lens), sum(lens)
    qb = synth.normal_bf16(91, synth.stream_id(synth.STREAM_Q), (t, hq, d))
    kb = synth.normal_bf16(91, synth.stream_id(synth.STREAM_K), (t, hkv, d))
    vb = synth.normal_bf16(91, synth.stream_id(synth.STREAM_V), (t, hkv, d))
    cache = F.KVCache.empty(B, hkv, max(lens) + 3, d)
    F.flux_kv_append(ctx, cache, hkv, d, H.bits_to_torch(kb), H.bits_to_torch(vb), cu(lens), t, max(lens))
    nb = -(-max(lens) // BLK)
    mask = torch.full((B, hq, nb + 1, nb + 2), 7, dtype=torch.uint8, device="cuda")    # a matrix larger than needed
    cfg = F.attn_cfg(hq, hkv, d, 0, 1, 0.0, 1)
    F.flux_xa_select(ctx, cfg, H.bits_to_torch(qb), cu(lens), max(lens), max(lens), cache, STRIDE, threshold, mask,
                     nb + 1, nb + 2)
    torch.cuda.synchronize()
    got = mask.cpu().numpy()
    assert set(np.unique(got)) <= {0, 1}                                  # every byte written
    qf, kf, vf = O.bf16_to_f64(qb), O.bf16_to_f64(kb), O.bf16_to_f64(vb)
    off, differ, total = 0, 0, 0
    for b, n in enumerate(lens):
        nbb = -(-n // BLK)
        assert not got[b, :, nbb:].any() and not got[b, :, :, nbb:].any()  # nothing beyond the prompt's blocks
        dd, tt = check_selection(got[b].astype(bool)[:, :nbb, :nbb], qf[off:off + n], kf[off:off + n], hq, hq // hkv, threshold)
        differ += dd
        total += tt
        off += n
    print("XA selection: %d of %d rows differ from the oracle's exact selection (all inside the 1e-5 envelope)" % (differ, total))
    assert differ <= max(1, total // 50)
    assert F.flux_last_device_status(ctx) == 0
    # ---- use it: block-sparse prefill under the GPU's matrix against the oracle's attention under the same matrix
    out = torch.full((t, hq, d), float("nan"), dtype=torch.float32, device="cuda")
    F.flux_attn_prefill_blocksparse(ctx, cfg, H.bits_to_torch(qb), cu(lens), max(lens), max(lens), cache,
                                    torch.zeros(B, dtype=torch.uint8, device="cuda"), mask, hq, nb + 1, nb + 2, out)
    torch.cuda.synchronize()
    off = 0
    for b, n in enumerate(lens):
        nbb = -(-n // BLK)
        ref = O.attention(qf[off:off + n], kf[off:off + n], vf[off:off + n], FA, 0, 1, block_mask=got[b].astype(bool)[:, :nbb, :nbb])
        H.assert_close(out[off:off + n].cpu().numpy(), ref, f"XA prefill, sequence of {n}")
        off += n
    kept = sum(int(got[b, :, :(-(-n // BLK)), :(-(-n // BLK))].sum()) for b, n in enumerate(lens))
    causal = sum(hq * (-(-n // BLK)) * (-(-n // BLK) + 1) // 2 for n in lens)
    print("kept %d of %d causal block pairs (%.0f %%)" % (kept, causal, 100.0 * kept / causal))


def test_xa_dominant_key_block_and_threshold_one(F, ctx):
    """One block of keys that every query points at takes the mass: the selection is that block plus the diagonal.
    Threshold 1 keeps every causal block (all of them carry mass)."""
    n, hq, hkv, d = 1024, 4, 1, 128
    r = np.random.default_rng(92)
    q = np.zeros((n, hq, d), np.float32)
    q[:, :, 0] = 3.0
    k = (0.01 * r.standard_normal((n, hkv, d))).astype(np.float32)
    k[128:192, :, :] = 0.0
    k[128:192, :, 0] = 32.0                                           # key block 2: scaled score 8.5 against about 0
    qb, kb = synth.f32_to_bf16_bits(q), synth.f32_to_bf16_bits(k)
    cache = F.KVCache.empty(1, hkv, n, d)
    F.flux_kv_append(ctx, cache, hkv, d, H.bits_to_torch(kb), H.bits_to_torch(kb), cu([n]), n, n)
    nb = n // BLK
    cfg = F.attn_cfg(hq, hkv, d, 0, 1, 0.0, 1)
    mask = torch.zeros(1, hq, nb, nb, dtype=torch.uint8, device="cuda")
    F.flux_xa_select(ctx, cfg, H.bits_to_torch(qb), cu([n]), n, n, cache, STRIDE, 0.9, mask, nb, nb)
    torch.cuda.synchronize()
    got = mask.cpu().numpy()[0].astype(bool)
    for h in range(hq):
        for bi in range(3, nb):
            assert set(np.nonzero(got[h, bi])[0]) == {2, bi}
    kr = synth.normal_bf16(93, synth.stream_id(synth.STREAM_K), (n, hkv, d))
    qr = synth.normal_bf16(93, synth.stream_id(synth.STREAM_Q), (n, hq, d))
    F.flux_kv_append(ctx, cache, hkv, d, H.bits_to_torch(kr), H.bits_to_torch(kr), cu([0]), 0, 0)
    cache.kv_len.zero_()
    F.flux_kv_append(ctx, cache, hkv, d, H.bits_to_torch(kr), H.bits_to_torch(kr), cu([n]), n, n)
    F.flux_xa_select(ctx, cfg, H.bits_to_torch(qr), cu([n]), n, n, cache, STRIDE, 1.0, mask, nb, nb)
    torch.cuda.synchronize()
    assert np.array_equal(mask.cpu().numpy()[0].astype(bool), np.broadcast_to(np.tril(np.ones((nb, nb), bool)), (hq, nb, nb)))


def test_xa_selection_long_prompt_sampled_rows(F, ctx):
    """32768 tokens, 32/8 heads of 128: sampled (head, query block) rows of the matrix against the oracle."""
    S, HQ, HKV, D = 32768, 32, 8, 128
    from paper_2604_07394_amd import synth_gpu as G
    q = torch.empty(1, S, HQ, D, dtype=torch.bfloat16, device="cuda")
    kn = torch.empty(1, S, HKV, D, dtype=torch.bfloat16, device="cuda")
    G.fill_normal_bf16(q, 94, synth.stream_id(synth.STREAM_Q))
    G.fill_normal_bf16(kn, 94, synth.stream_id(synth.STREAM_K))
    cache = F.KVCache.empty(1, HKV, S, D)
    F.flux_kv_append(ctx, cache, HKV, D, kn[0], kn[0], i32([0, S]), S, S)
    nb = S // BLK
    mask = torch.empty(1, HQ, nb, nb, dtype=torch.uint8, device="cuda")
    cfg = F.attn_cfg(HQ, HKV, D, 0, 1, 0.0, 1)
    F.flux_xa_select(ctx, cfg, q[0], i32([0, S]), S, S, cache, STRIDE, 0.9, mask, nb, nb)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    F.flux_xa_select(ctx, cfg, q[0], i32([0, S]), S, S, cache, STRIDE, 0.9, mask, nb, nb)
    e1.record()
    torch.cuda.synchronize()
    got = mask.cpu().numpy()[0].astype(bool)
    rows = [0, 1, 63, 200, nb - 1]
    differ = total = 0
    for h in (0, 17, 31):
        qf = H.torch_to_f64(q[0, :, h])
        kf = H.torch_to_f64(kn[0, :, h // 4])
        dd, tt = check_selection(got[h:h + 1], qf[:, None, :], kf[:, None, :], 1, 1, 0.9, rows=rows)
        differ += dd
        total += tt
    dens = got.sum() / (HQ * nb * (nb + 1) / 2)
    print("XA selection at 32768 tokens: %.3f ms, %.1f %% of the causal block pairs kept, %d of %d sampled rows differ"
          % (e0.elapsed_time(e1), 100 * dens, differ, total))
    assert F.flux_last_device_status(ctx) == 0


def test_xa_selection_beyond_65536_positions_two_walks(F, ctx):
    """A prompt of 66100 positions: the (square row, key block) table of a workgroup no longer fits LDS, so the kernel
    walks the keys twice (maximum and sum first, probabilities second).  Sampled rows against the oracle."""
    S, HQ, HKV, D = 66100, 2, 1, 64
    from paper_2604_07394_amd import synth_gpu as G
    q = torch.empty(1, S, HQ, D, dtype=torch.bfloat16, device="cuda")
    kn = torch.empty(1, S, HKV, D, dtype=torch.bfloat16, device="cuda")
    G.fill_normal_bf16(q, 95, synth.stream_id(synth.STREAM_Q))
    G.fill_normal_bf16(kn, 95, synth.stream_id(synth.STREAM_K))
    cache = F.KVCache.empty(1, HKV, S, D)
    F.flux_kv_append(ctx, cache, HKV, D, kn[0], kn[0], i32([0, S]), S, S)
    nb = -(-S // BLK)
    assert nb > 1024
    mask = torch.full((1, HQ, nb, nb), 9, dtype=torch.uint8, device="cuda")
    cfg = F.attn_cfg(HQ, HKV, D, 0, 1, 0.0, 1)
    F.flux_xa_select(ctx, cfg, q[0], i32([0, S]), S, S, cache, STRIDE, 0.9, mask, nb, nb)
    torch.cuda.synchronize()
    got = mask.cpu().numpy()[0].astype(bool)
    assert mask.max().item() <= 1                                      # every byte written
    rows = [0, 7, 640, nb - 2, nb - 1]
    differ = total = 0
    for h in range(HQ):
        qf = H.torch_to_f64(q[0, :, h])
        kf = H.torch_to_f64(kn[0, :, 0])
        dd, tt = check_selection(got[h:h + 1], qf[:, None, :], kf[:, None, :], 1, 1, 0.9, rows=rows)
        differ += dd
        total += tt
    print("XA selection at %d tokens (two walks): %d of %d sampled rows differ" % (S, differ, total))
    assert F.flux_last_device_status(ctx) == 0

