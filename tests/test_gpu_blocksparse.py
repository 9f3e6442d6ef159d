"""GPU parity of flux_attn_prefill_blocksparse (Eq. 2 over an arbitrary set of 64-position key blocks) against
the fp64 oracle's explicit block mask, element by element; plus what is unique about the form: an all-kept
matrix is FA bit for bit, the sink + window pattern written as blocks is the block-granular SA bit for bit, and
key blocks that no query block of a tile keeps are never read."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as O
from paper_2604_07394_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

FA, SA = 1, 0
BLK = 64


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


def u8(x):
    return torch.tensor(np.asarray(x, dtype=np.uint8), device="cuda")


def cu(lens):
    return i32(np.concatenate([[0], np.cumsum(lens)]))


class Case:
    """A ragged batch with `prior` positions already cached per sequence and `n_q` new queries each."""

    def __init__(self, F, ctx, seed, prior, n_q, hq, hkv, d):
        self.F, self.ctx = F, ctx
        self.prior, self.n_q, self.hq, self.hkv, self.d = prior, n_q, hq, hkv, d
        self.B = len(n_q)
        self.lens = [p + n for p, n in zip(prior, n_q)]
        t_all = sum(self.lens)
        self.kb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_K), (t_all, hkv, d))
        self.vb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_V), (t_all, hkv, d))
        self.qb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_Q), (sum(n_q), hq, d))
        self.cache = F.KVCache.empty(self.B, hkv, max(self.lens) + 5, d)
        F.flux_kv_append(ctx, self.cache, hkv, d, H.bits_to_torch(self.kb), H.bits_to_torch(self.vb), cu(self.lens),
                         t_all, max(self.lens))
        self.n_kb = -(-max(self.lens) // BLK)
        self.n_qb = max((l - 1) // BLK - p // BLK + 1 for l, p in zip(self.lens, prior))

    def run(self, masks, modes, heads):
        """masks: bool [B, heads, n_qb, n_kb]."""
        F = self.F
        cfg = F.attn_cfg(self.hq, self.hkv, self.d, 0, 1, 0.0, 1)
        out = torch.full((sum(self.n_q), self.hq, self.d), float("nan"), dtype=torch.float32, device="cuda")
        F.flux_attn_prefill_blocksparse(self.ctx, cfg, H.bits_to_torch(self.qb), cu(self.n_q), max(self.n_q),
                                        max(self.lens), self.cache, u8(modes), u8(masks), heads, self.n_qb, self.n_kb, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def reference(self, masks, modes):
        ref, qo, ko = [], 0, 0
        for b in range(self.B):
            n, l = self.n_q[b], self.lens[b]
            q = O.bf16_to_f64(self.qb[qo:qo + n])
            k = O.bf16_to_f64(self.kb[ko:ko + l])
            v = O.bf16_to_f64(self.vb[ko:ko + l])
            if n:
                if modes[b] == FA:
                    ref.append(O.attention(q, k, v, FA, 0, 1))
                else:
                    m = masks[b] if masks.shape[1] > 1 else masks[b, 0]
                    ref.append(O.attention(q, k, v, FA, 0, 1, block_mask=m))
            qo += n
            ko += l
        return np.concatenate(ref, axis=0)


@pytest.mark.parametrize("d,hq,hkv,heads", [(128, 8, 2, 8), (128, 7, 1, 1), (64, 4, 4, 4), (128, 6, 3, 1)])
def test_random_block_masks_ragged_batch(F, ctx, d, hq, hkv, heads):
    """Whole prompts of ragged lengths, random 35 % dense keep matrices per head or shared, one FA sequence."""
    n_q = [700, 300, 64, 1, 129]
    case = Case(F, ctx, 81, [0] * 5, n_q, hq, hkv, d)
    masks = np.random.default_rng(82).random((5, heads, case.n_qb, case.n_kb)) < 0.35
    modes = [SA, SA, SA, SA, FA]
    got = case.run(masks, modes, heads)
    ref = case.reference(masks, modes)
    off = 0
    for n in n_q:
        H.assert_close(got[off:off + n], ref[off:off + n], f"block-sparse sequence of {n}")
        off += n
    assert F.flux_last_device_status(ctx) == 0


@pytest.mark.parametrize("prior,n_q", [([500, 64, 1000], [333, 200, 1]), ([128, 0, 37], [256, 65, 130])])
def test_chunks_that_start_inside_a_block(F, ctx, prior, n_q):
    """Queries are the last positions of the cache; the first one may sit anywhere inside a 64-position block, so a
    128-row tile spans three query blocks of the matrix."""
    case = Case(F, ctx, 83, prior, n_q, 8, 2, 128)
    masks = np.random.default_rng(84).random((3, 8, case.n_qb, case.n_kb)) < 0.3
    got = case.run(masks, [SA] * 3, 8)
    H.assert_close(got, case.reference(masks, [SA] * 3), "block-sparse chunk")
    assert F.flux_last_device_status(ctx) == 0
    # a matrix with one query-block row too few: the uncovered pairs count as not kept, and the call says so
    if (case.n_qb - 1) * BLK >= max(n_q):                       # (a shorter one is refused on the host)
        short = np.ascontiguousarray(masks[:, :, :case.n_qb - 1])
        full_nqb, case.n_qb = case.n_qb, case.n_qb - 1
        got_short = case.run(short, [SA] * 3, 8)
        case.n_qb = full_nqb
        assert F.flux_last_device_status(ctx) == F.FLUX_DEV_BAD_LENGTH
        hidden = masks.copy()
        hidden[:, :, full_nqb - 1] = False
        H.assert_close(got_short, case.reference(hidden, [SA] * 3), "matrix one row short")


def test_all_kept_is_fa_and_sink_window_blocks_are_block_granular_sa_bit_for_bit(F, ctx):
    n = 1000
    case = Case(F, ctx, 85, [0], [n], 8, 2, 128)
    nb = case.n_kb
    everything = np.ones((1, 1, nb, nb), bool)
    got = case.run(everything, [SA], 1)
    cfg = F.attn_cfg(8, 2, 128, 128, 192, 0.0, 1, 64)
    fa = torch.empty(n, 8, 128, dtype=torch.float32, device="cuda")
    F.flux_attn_prefill(ctx, cfg, H.bits_to_torch(case.qb), cu([n]), n, n, case.cache, u8([FA]), fa)
    sa = torch.empty(n, 8, 128, dtype=torch.float32, device="cuda")
    F.flux_attn_prefill(ctx, cfg, H.bits_to_torch(case.qb), cu([n]), n, n, case.cache, u8([SA]), sa)
    torch.cuda.synchronize()
    assert np.array_equal(got, fa.cpu().numpy())
    bi, bj = np.arange(nb)[:, None], np.arange(nb)[None, :]
    streaming = ((bj < 2) | (bi - bj < 3))[None, None]               # 128 sinks = 2 blocks, window 192 = 3 blocks
    assert np.array_equal(case.run(streaming, [SA], 1), sa.cpu().numpy())
    # nothing kept: every query still sees its own block, causally
    nothing = case.run(np.zeros((1, 1, nb, nb), bool), [SA], 1)
    H.assert_close(nothing, case.reference(np.zeros((1, 1, nb, nb), bool), [SA]), "diagonal blocks only")
    assert np.array_equal(nothing[:64], fa.cpu().numpy()[:64])


def test_blocks_nobody_keeps_are_never_read(F, ctx):
    """Key blocks that no query block of a 128-row tile keeps are skipped, not masked: poisoning their K and V
    rows with NaN leaves the output bit-identical."""
    n = 1024
    case = Case(F, ctx, 86, [0], [n], 4, 1, 128)
    nb = case.n_kb
    masks = np.zeros((1, 1, nb, nb), bool)
    masks[0, 0, :, 0] = True                                        # block 0 for everyone
    masks[0, 0, 9:, 5] = True                                       # block 5 for the late queries
    clean = case.run(masks, [SA], 1)
    for kbk in range(nb):
        tiles = [t for t in range(nb // 2) if 2 * t + 1 >= kbk]     # 128-row tiles that could reach this block
        kept = any(masks[0, 0, r, kbk] or r == kbk for t in tiles for r in (2 * t, 2 * t + 1) if kbk <= r)
        if not kept:
            case.cache.k[0, :, kbk * 64:(kbk + 1) * 64] = float("nan")
            case.cache.v[0, :, kbk * 64:(kbk + 1) * 64] = float("nan")
    # blocks 1..4 and 6.. are kept only by their own diagonal tiles; poison what lies strictly between
    poisoned = case.run(masks, [SA], 1)
    assert np.isfinite(poisoned).all()
    assert np.array_equal(clean, poisoned)
    H.assert_close(clean, case.reference(masks, [SA]), "two-column mask")


def test_long_prompt_ten_percent_dense(F, ctx):
    """32768 tokens, 32/8 heads of 128, a random 10 % dense keep matrix per head: sampled rows against the oracle."""
    S, HQ, HKV, D = 32768, 32, 8, 128
    from paper_2604_07394_amd import synth_gpu as G
    q = torch.empty(1, S, HQ, D, dtype=torch.bfloat16, device="cuda")
    kn = torch.empty(1, S, HKV, D, dtype=torch.bfloat16, device="cuda")
    vn = torch.empty(1, S, HKV, D, dtype=torch.bfloat16, device="cuda")
    G.fill_normal_bf16(q, 87, synth.stream_id(synth.STREAM_Q))
    G.fill_normal_bf16(kn, 87, synth.stream_id(synth.STREAM_K))
    G.fill_normal_bf16(vn, 87, synth.stream_id(synth.STREAM_V))
    cache = F.KVCache.empty(1, HKV, S, D)
    F.flux_kv_append(ctx, cache, HKV, D, kn[0], vn[0], i32([0, S]), S, S)
    nb = S // BLK
    masks = np.random.default_rng(88).random((1, HQ, nb, nb)) < 0.10
    out = torch.full((S, HQ, D), float("nan"), dtype=torch.float32, device="cuda")
    F.flux_attn_prefill_blocksparse(ctx, F.attn_cfg(HQ, HKV, D, 0, 1, 0.0, 1), q[0], i32([0, S]), S, S, cache, u8([SA]),
                                    u8(masks), HQ, nb, nb, out)
    torch.cuda.synchronize()
    rows = sorted(set([0, 63, 64, 127, 128, 4095, 4096, S - 129, S - 128, S - 1] +
                      np.random.default_rng(89).integers(0, S, 14).tolist()))
    worst = 0.0
    for h in (0, 13, 31):
        kf = H.torch_to_f64(kn[0, :, h // 4])
        vf = H.torch_to_f64(vn[0, :, h // 4])
        for i in rows:
            ref = O.attention_row(H.torch_to_f64(q[0, i, h:h + 1]), kf, vf, i, FA, 0, 1, block_row=masks[0, h, i // BLK])
            got = H.torch_to_f64(out[i, h:h + 1])
            e = H.assert_close(got, ref, f"10 % dense, head {h}, position {i}")
            worst = max(worst, e[0])
    print("ten percent dense block mask at 32768 tokens: worst max-abs %.2e" % worst)
    assert F.flux_last_device_status(ctx) == 0
