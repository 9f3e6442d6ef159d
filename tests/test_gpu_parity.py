"""GPU parity: every entry point of libflux against the fp64 CPU oracle, element by element, on the
same seeded inputs.  Tolerance for attention (bf16 inputs, fp32 accumulation, fp32 output):
max-abs 1e-2 and relative L2 5e-3; router decisions are bit-exact outside a 1e-6 logit margin;
copies and lengths are bit-exact."""
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
    return torch.tensor(x, dtype=torch.int32, device="cuda")


def u8(x):
    return torch.tensor(x, dtype=torch.uint8, device="cuda")


def cu(lens):
    return i32(np.concatenate([[0], np.cumsum(lens)]))


class Layer:
    """Drives one layer through the C ABI and mirrors it in the oracle."""

    def __init__(self, F, ctx, seed, batch, hq, hkv, d, capacity, n_sink, window, layer=0, scales=False, block=1,
                 scale=None):
        self.F, self.ctx, self.seed, self.layer = F, ctx, seed, layer
        self.B, self.hq, self.hkv, self.d = batch, hq, hkv, d
        self.block = block
        self.scale = scale                                  # None: the default 1/sqrt(d) (cfg value 0)
        self.cfg = F.attn_cfg(hq, hkv, d, n_sink, window, 0.0 if scale is None else scale, 1, block if block > 1 else 0)
        self.n_sink, self.window = n_sink, window
        self.cache = F.KVCache.empty(batch, hkv, capacity, d)
        self.ocache = O.KVCache(batch, hkv, d)
        self.lens = [0] * batch
        self.counter = 0
        self.qs = self.ks = self.vs = None
        if scales:
            self.qs = synth.head_scales(seed, synth.stream_id(synth.STREAM_QSCALE, layer), hq)
            self.ks = synth.head_scales(seed, synth.stream_id(synth.STREAM_KSCALE, layer), hkv)
            self.vs = synth.head_scales(seed, synth.stream_id(synth.STREAM_VSCALE, layer), hkv)

    def _draw(self, kind, rows, heads, scale):
        bits = synth.normal_bf16(self.seed, synth.stream_id(kind, self.layer), (rows, heads, self.d),
                                 scale, 1 if scale is not None else None, counter0=self.counter)
        self.counter += rows * heads * self.d
        return bits

    def new_tokens(self, n_new):
        """Draw q/k/v for n_new[b] new tokens per sequence (packed), as bit patterns."""
        t = int(sum(n_new))
        return (self._draw(synth.STREAM_Q, t, self.hq, self.qs), self._draw(synth.STREAM_K, t, self.hkv, self.ks),
                self._draw(synth.STREAM_V, t, self.hkv, self.vs))

    def append(self, kb, vb, n_new):
        F = self.F
        F.flux_kv_append(self.ctx, self.cache, self.hkv, self.d, H.bits_to_torch(kb), H.bits_to_torch(vb),
                         cu(n_new), int(sum(n_new)), int(max(n_new)))
        off = 0
        for b, n in enumerate(n_new):
            self.ocache.append(b, O.bf16_to_f64(kb[off:off + n]), O.bf16_to_f64(vb[off:off + n]))
            self.lens[b] += n
            off += n

    def prefill(self, qb, n_q, modes, max_q_len=None, want_ref=True):
        """max_q_len: the host's bound on the longest prompt of the call (default: the longest); a larger bound is
        valid and chooses the launch shape (from 32768 rows on: 256-row workgroups at head dimension 128)."""
        F = self.F
        t = int(sum(n_q))
        out = torch.full((t, self.hq, self.d), float("nan"), dtype=torch.float32, device="cuda")
        F.flux_attn_prefill(self.ctx, self.cfg, H.bits_to_torch(qb), cu(n_q), int(max_q_len or max(n_q)),
                            int(max(max_q_len or 0, max(self.lens))), self.cache, u8(modes), out)
        torch.cuda.synchronize()
        if not want_ref:
            return out.cpu().numpy(), None
        ref = []
        off = 0
        for b, n in enumerate(n_q):
            if n:
                ref.append(O.attention(O.bf16_to_f64(qb[off:off + n]), self.ocache.k[b], self.ocache.v[b],
                                       int(modes[b]), self.n_sink, self.window, scale=self.scale, block=self.block))
            off += n
        return out.cpu().numpy(), np.concatenate(ref, axis=0)

    def decode(self, qb, modes, max_kv_len=None):
        F = self.F
        out = torch.full((self.B, self.hq, self.d), float("nan"), dtype=torch.float32, device="cuda")
        F.flux_attn_decode(self.ctx, self.cfg, H.bits_to_torch(qb), int(max_kv_len or max(self.lens)), self.cache,
                           u8(modes), out)
        torch.cuda.synchronize()
        qf = O.bf16_to_f64(qb)
        ref = np.stack([O.attention(qf[b][None], self.ocache.k[b], self.ocache.v[b], int(modes[b]), self.n_sink,
                                    self.window, scale=self.scale, block=self.block)[0] if self.lens[b] else np.zeros((self.hq, self.d))
                        for b in range(self.B)])
        return out.cpu().numpy(), ref


# ----------------------------------------------------------------------------- generator

def test_device_generator_matches_host_bits():
    from paper_2604_07394_amd import synth_gpu
    big = torch.zeros(3, 4, 40, 72, dtype=torch.bfloat16, device="cuda")
    view = big[:, :, 3:36, :64]                        # strided view: capacity padding and wider rows
    scale = synth.head_scales(5, synth.stream_id(synth.STREAM_KSCALE), 4)
    synth_gpu.fill_normal_bf16(view, 5, synth.stream_id(synth.STREAM_K, 2), torch.from_numpy(scale).cuda(), 1,
                               counter0=12345)
    torch.cuda.synchronize()
    host = synth.normal_bf16(5, synth.stream_id(synth.STREAM_K, 2), (3, 4, 33, 64), scale, 1, counter0=12345)
    assert np.array_equal(H.torch_to_bits(view), host)
    assert float(big[:, :, :3].abs().max()) == 0 and float(big[..., 64:].abs().max()) == 0
    # a larger unscaled draw: 2M samples must agree bit for bit
    t = torch.empty(1, 1, 8192, 256, dtype=torch.bfloat16, device="cuda")
    synth_gpu.fill_normal_bf16(t, 9, 77)
    assert np.array_equal(H.torch_to_bits(t), synth.normal_bf16(9, 77, (1, 1, 8192, 256)))


# ----------------------------------------------------------------------------- kv append

def test_kv_append_ragged_bit_exact(F, ctx):
    lay = Layer(F, ctx, 11, 3, 4, 2, 64, 300, 4, 16)
    for n_new in ([5, 0, 130], [1, 1, 1], [64, 7, 100]):
        _, kb, vb = lay.new_tokens(n_new)
        lay.append(kb, vb, n_new)
    torch.cuda.synchronize()
    assert lay.cache.kv_len.cpu().tolist() == lay.lens == [70, 8, 231]
    for b in range(3):
        k_dev = H.torch_to_f64(lay.cache.k[b, :, :lay.lens[b]]).transpose(1, 0, 2)
        v_dev = H.torch_to_f64(lay.cache.v[b, :, :lay.lens[b]]).transpose(1, 0, 2)
        assert np.array_equal(k_dev, lay.ocache.k[b]) and np.array_equal(v_dev, lay.ocache.v[b])
    assert F.flux_last_device_status(ctx) == 0


def test_kv_append_overflow_is_clamped_and_flagged(F, ctx):
    lay = Layer(F, ctx, 12, 2, 2, 2, 64, 16, 0, 4)
    _, kb, vb = lay.new_tokens([10, 3])
    lay.append(kb, vb, [10, 3])
    # 8 more rows for sequence 0 (only 6 fit), 0 for sequence 1
    _, kb2, vb2 = lay.new_tokens([8, 0])
    F.flux_kv_append(ctx, lay.cache, 2, 64, H.bits_to_torch(kb2), H.bits_to_torch(vb2), cu([8, 0]), 8, 8)
    torch.cuda.synchronize()
    assert lay.cache.kv_len.cpu().tolist() == [16, 3]
    assert F.flux_last_device_status(ctx) & F.FLUX_DEV_KV_OVERFLOW
    assert F.flux_last_device_status(ctx) == 0                      # sticky bit cleared by the read
    got = H.torch_to_bits(lay.cache.k[0, :, 10:16]).transpose(1, 0, 2)
    assert np.array_equal(got, kb2[:6])


# ----------------------------------------------------------------------------- prefill

def test_prefill_tiny_config_full_compare(F, ctx):
    """The Tiny configuration: 4 layers [FA, SA, FA, SA], S 512, 8/2 heads, D 64, 16 sinks, window 128,
    every output element compared; then 16 decode steps appending new rows."""
    worst = (0.0, 0.0)
    for layer, mode in enumerate([FA, SA, FA, SA]):
        lay = Layer(F, ctx, 0, 1, 8, 2, 64, 512 + 16, 16, 128, layer=layer)
        qb, kb, vb = lay.new_tokens([512])
        lay.append(kb, vb, [512])
        got, ref = lay.prefill(qb, [512], [mode])
        e = H.assert_close(got, ref, f"tiny prefill layer {layer}")
        worst = max(worst, e)
        for step in range(16):
            qb, kb, vb = lay.new_tokens([1])
            lay.append(kb, vb, [1])
            got, ref = lay.decode(qb.reshape(1, 8, 64), [mode])
            H.assert_close(got, ref, f"tiny decode layer {layer} step {step}")
    print("tiny worst (max-abs, rel-L2):", worst)


@pytest.mark.parametrize("d,hq,hkv", [(128, 8, 2), (128, 7, 1), (64, 4, 4), (128, 6, 3)])
def test_prefill_ragged_multi_tile(F, ctx, d, hq, hkv):
    """Ragged batch over several 128-row tiles with ragged tails, per-sequence modes, sinks and a
    window that are not multiples of the 64-key block, per-head scales up to 2.  The four shapes give
    8, 4, 16 and 12 (sequence, KV head) pairs: every workgroup-to-XCD mapping of the kernel is used."""
    lens = [700, 129, 64, 1]
    modes = [SA, FA, SA, SA]
    lay = Layer(F, ctx, 21, 4, hq, hkv, d, 704, 37, 150, scales=True)
    qb, kb, vb = lay.new_tokens(lens)
    lay.append(kb, vb, lens)
    got, ref = lay.prefill(qb, lens, modes)
    H.assert_close(got, ref, "ragged prefill")
    # per-sequence check so that a short sequence cannot hide behind a long one
    off = 0
    for n in lens:
        H.assert_close(got[off:off + n], ref[off:off + n], f"sequence of {n}")
        off += n


def test_prefill_chunked_equals_whole(F, ctx):
    """Queries are the last n_q positions of the cache: a second chunk attends the first."""
    lay = Layer(F, ctx, 22, 2, 4, 2, 128, 512, 8, 100)
    q1, k1, v1 = lay.new_tokens([300, 200])
    lay.append(k1, v1, [300, 200])
    got1, ref1 = lay.prefill(q1, [300, 200], [SA, FA])
    H.assert_close(got1, ref1, "first chunk")
    q2, k2, v2 = lay.new_tokens([150, 0])
    lay.append(k2, v2, [150, 0])
    got2, ref2 = lay.prefill(q2, [150, 0], [SA, FA])
    H.assert_close(got2, ref2, "second chunk")


def test_prefill_sa_window_covering_everything_equals_fa(F, ctx):
    lay = Layer(F, ctx, 23, 1, 4, 1, 128, 400, 0, 4096)
    qb, kb, vb = lay.new_tokens([400])
    lay.append(kb, vb, [400])
    got_sa, ref = lay.prefill(qb, [400], [SA])
    got_fa, _ = lay.prefill(qb, [400], [FA])
    assert np.array_equal(got_sa, got_fa)
    H.assert_close(got_sa, ref, "wide window")


def test_prefill_bf16_output(F, ctx):
    lay = Layer(F, ctx, 24, 1, 4, 2, 128, 256, 4, 64)
    qb, kb, vb = lay.new_tokens([256])
    lay.append(kb, vb, [256])
    got32, ref = lay.prefill(qb, [256], [SA])
    cfg16 = F.attn_cfg(4, 2, 128, 4, 64, 0.0, 0)
    out16 = torch.empty(256, 4, 128, dtype=torch.bfloat16, device="cuda")
    F.flux_attn_prefill(ctx, cfg16, H.bits_to_torch(qb), cu([256]), 256, 256, lay.cache, u8([SA]), out16)
    torch.cuda.synchronize()
    # the bf16 output is the fp32 output rounded once
    assert torch.equal(out16.cpu(), torch.from_numpy(got32).to(torch.bfloat16))
    got16 = H.torch_to_f64(out16)
    assert (np.abs(got16 - ref) <= np.maximum(1e-2, 2.0 ** -8 * np.abs(ref))).all()


def test_prefill_is_deterministic(F, ctx):
    lay = Layer(F, ctx, 25, 2, 8, 2, 128, 384, 16, 128)
    qb, kb, vb = lay.new_tokens([384, 200])
    lay.append(kb, vb, [384, 200])
    a, _ = lay.prefill(qb, [384, 200], [FA, SA])
    b, _ = lay.prefill(qb, [384, 200], [FA, SA])
    assert np.array_equal(a, b)


def _scaled_bits(bits, factor):
    """bf16 bit patterns times a per-row factor, rounded to bf16 again (input preparation only)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).float()
    t = (t * torch.from_numpy(np.asarray(factor, dtype=np.float32)).reshape(-1, 1, 1)).to(torch.bfloat16)
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("shape", ["rising", "falling", "spikes"])
def test_prefill_and_decode_softmax_range(F, ctx, shape):
    """Scores that move by hundreds of powers of two along the keys: key norms that rise or fall 40-fold over
    the prompt, and isolated keys 60 times larger than their neighbours.  The running reference of the online
    softmax has to follow (rescale) without overflow, and rows whose early keys end up negligible must not
    lose the late ones."""
    S, hq, hkv, d = 1100, 4, 1, 128
    lay = Layer(F, ctx, 71, 1, hq, hkv, d, S + 8, 16, 300)
    qb, kb, vb = lay.new_tokens([S])
    j = np.arange(S, dtype=np.float64)
    if shape == "rising":
        f = 0.25 + 10.0 * j / S
    elif shape == "falling":
        f = 10.0 - 9.75 * j / S
    else:
        f = np.where((j % 97) == 41, 15.0, 0.25)
    kb = _scaled_bits(kb, f)
    qb = _scaled_bits(qb, np.full(S, 2.0))
    lay.append(kb, vb, [S])
    for mode in (FA, SA):
        got, ref = lay.prefill(qb, [S], [mode])
        H.assert_close(got, ref, f"{shape} keys, mode {mode}")
    dec, dref = lay.decode(qb[S - 1][None], [FA])
    H.assert_close(dec, dref, f"{shape} keys, decode")


# ----------------------------------------------------------------------------- decode

@pytest.mark.parametrize("d,hq,hkv", [(128, 8, 2), (128, 7, 1), (64, 8, 2), (128, 40, 2)])
def test_decode_ragged_multi_chunk(F, ctx, d, hq, hkv):
    """Caches long enough for several split-K chunks, ragged lengths (one shorter than sinks+window,
    one a single token), mixed modes, and group sizes 4, 7 and 20 (more than one MFMA column block)."""
    lens = [3000, 1537, 100, 1]
    modes = [FA, SA, SA, FA]
    lay = Layer(F, ctx, 31, 4, hq, hkv, d, 3100, 24, 333, scales=True)
    _, kb, vb = lay.new_tokens(lens)
    lay.append(kb, vb, lens)
    for step in range(3):
        qb, kb, vb = lay.new_tokens([1, 1, 1, 1])
        lay.append(kb, vb, [1, 1, 1, 1])
        got, ref = lay.decode(qb.reshape(4, hq, d), modes)
        for b in range(4):
            H.assert_close(got[b], ref[b], f"decode step {step} seq {b} (len {lay.lens[b]})")


@pytest.mark.parametrize("B,top", [(70, 2600), (300, 600)])
def test_decode_wide_ragged_batch_more_sequences_than_lanes(F, ctx, B, top):
    """70 and 300 sequences (the device-side split walks the batch 64 at a time) with lengths from 0 to `top`
    and alternating modes: every sequence is found by the prefix sum and merged with its own chunks."""
    hq, hkv, d = 4, 1, 128
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(0, top, size=B)]
    lens[3], lens[64], lens[B - 1] = 0, top - 1, 1
    modes = [FA if (b * 7) % 3 else SA for b in range(B)]
    lay = Layer(F, ctx, 35, B, hq, hkv, d, 2700, 16, 200)
    _, kb, vb = lay.new_tokens(lens)
    lay.append(kb, vb, lens)
    qb = lay._draw(synth.STREAM_Q, B, hq, None)
    got, ref = lay.decode(qb.reshape(B, hq, d), modes, max_kv_len=2700)
    for b in range(B):
        if lens[b]:
            H.assert_close(got[b], ref[b], f"wide batch seq {b} (len {lens[b]}, mode {modes[b]})")
        else:
            assert not got[b].any()
    assert F.flux_last_device_status(ctx) == 0


def test_decode_long_ragged_batch_chunk_above_minimum(F, ctx):
    """Enough visible keys in the batch that the device picks a chunk above its minimum, with one long,
    one medium and one short sequence sharing the call."""
    lens = [100000, 40000, 5000]
    modes = [FA, FA, SA]
    lay = Layer(F, ctx, 36, 3, 8, 2, 128, 100010, 64, 1000)
    _, kb, vb = lay.new_tokens(lens)
    lay.append(kb, vb, lens)
    qb, kb, vb = lay.new_tokens([1, 1, 1])
    lay.append(kb, vb, [1, 1, 1])
    got, ref = lay.decode(qb.reshape(3, 8, 128), modes)
    for b in range(3):
        H.assert_close(got[b], ref[b], f"long ragged seq {b}")
    again, _ = lay.decode(qb.reshape(3, 8, 128), modes, max_kv_len=100010)     # a looser host bound changes nothing
    assert np.array_equal(got, again)


def test_decode_equals_last_prefill_row_on_gpu(F, ctx):
    lay = Layer(F, ctx, 32, 2, 8, 2, 128, 600, 16, 128)
    qb, kb, vb = lay.new_tokens([600, 333])
    lay.append(kb, vb, [600, 333])
    pre, _ = lay.prefill(qb, [600, 333], [SA, FA])
    q_last = np.stack([qb[599], qb[600 + 332]])
    dec, ref = lay.decode(q_last, [SA, FA])
    H.assert_close(dec, ref, "decode")
    assert np.abs(dec[0] - pre[599]).max() < 2e-3 and np.abs(dec[1] - pre[600 + 332]).max() < 2e-3


def test_decode_sparse_launch_sizing_and_never_reads_the_middle(F, ctx):
    """An SA layer sized for n_sink + window keys gives the same result, and poisoning the hidden
    middle of the cache with NaN does not change it: those rows are never read."""
    lay = Layer(F, ctx, 33, 2, 8, 2, 128, 2100, 32, 256)
    _, kb, vb = lay.new_tokens([2048, 1500])
    lay.append(kb, vb, [2048, 1500])
    qb, kb, vb = lay.new_tokens([1, 1])
    lay.append(kb, vb, [1, 1])
    q = qb.reshape(2, 8, 128)
    full, ref = lay.decode(q, [SA, SA])
    H.assert_close(full, ref, "sa decode")
    small, _ = lay.decode(q, [SA, SA], max_kv_len=32 + 256)
    assert np.array_equal(full, small)
    lay.cache.k[0, :, 32:2049 - 256] = float("nan")
    lay.cache.v[0, :, 32:2049 - 256] = float("nan")
    lay.cache.k[1, :, 32:1501 - 256] = float("nan")
    lay.cache.v[1, :, 32:1501 - 256] = float("nan")
    poisoned, _ = lay.decode(q, [SA, SA])
    assert np.array_equal(full, poisoned)


def test_decode_is_deterministic(F, ctx):
    lay = Layer(F, ctx, 34, 3, 8, 2, 128, 5000, 16, 512)
    _, kb, vb = lay.new_tokens([5000, 2500, 700])
    lay.append(kb, vb, [5000, 2500, 700])
    qb, _, _ = lay.new_tokens([1, 1, 1])
    a, _ = lay.decode(qb.reshape(3, 8, 128), [FA, SA, FA])
    b, _ = lay.decode(qb.reshape(3, 8, 128), [FA, SA, FA])
    assert np.array_equal(a, b)


@pytest.mark.parametrize("d,hq,hkv", [(128, 8, 2), (64, 7, 1)])
def test_decode_bf16_output(F, ctx, d, hq, hkv):
    """The output type the latency runs use (BF16 throughout, App. B.3): the bf16 output of a decode call is
    its fp32 output rounded once, and it stays within max(1e-2, 2^-8 |o|) of the oracle.  Several chunks,
    mixed modes, a short and an empty sequence."""
    lens = [2900, 1300, 40, 0]
    modes = [FA, SA, SA, FA]
    lay = Layer(F, ctx, 36, 4, hq, hkv, d, 3000, 24, 333, scales=True)
    _, kb, vb = lay.new_tokens(lens)
    lay.append(kb, vb, lens)
    qb, _, _ = lay.new_tokens([1, 1, 1, 1])
    q = qb.reshape(4, hq, d)
    got32, ref = lay.decode(q, modes)
    cfg16 = F.attn_cfg(hq, hkv, d, 24, 333, 0.0, 0)
    out16 = torch.full((4, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    F.flux_attn_decode(ctx, cfg16, H.bits_to_torch(q), max(lens), lay.cache, u8(modes), out16)
    torch.cuda.synchronize()
    assert torch.equal(out16.cpu(), torch.from_numpy(got32).to(torch.bfloat16))
    got16 = H.torch_to_f64(out16)
    assert (np.abs(got16 - ref) <= np.maximum(1e-2, 2.0 ** -8 * np.abs(ref))).all()


@pytest.mark.parametrize("d,scale", [(128, 0.25), (64, 1.7 / 8.0), (128, 0.011)])
def test_explicit_softmax_scale_prefill_and_decode(F, ctx, d, scale):
    """Eq. (1) leaves the scale out; the call takes any positive one.  A scale well above 1/sqrt(d) (sharp
    rows), 1.7 times the default, and a nearly flat one, against the oracle given the same scale."""
    lens = [600, 130]
    modes = [SA, FA]
    lay = Layer(F, ctx, 37, 2, 8, 2, d, 640, 9, 100, scale=scale)
    qb, kb, vb = lay.new_tokens(lens)
    lay.append(kb, vb, lens)
    got, ref = lay.prefill(qb, lens, modes)
    H.assert_close(got, ref, f"prefill, scale {scale}")
    # the default-scale result must differ: the argument is really used
    lay0 = Layer(F, ctx, 37, 2, 8, 2, d, 640, 9, 100)
    lay0.cache, lay0.ocache, lay0.lens = lay.cache, lay.ocache, lay.lens
    got0, _ = lay0.prefill(qb, lens, modes)
    assert np.abs(got0 - got).max() > 1e-2
    q1, k1, v1 = lay.new_tokens([1, 1])
    lay.append(k1, v1, [1, 1])
    dec, dref = lay.decode(q1.reshape(2, 8, d), modes)
    H.assert_close(dec, dref, f"decode, scale {scale}")


# ----------------------------------------------------------------------------- router

def router_case(F, ctx, seed, lens, hidden, inner, pool, bias):
    t = int(sum(lens))
    xb = synth.normal_bf16(seed, synth.stream_id(synth.STREAM_X), (t, hidden))
    w1f = synth.normal_f32(seed, synth.stream_id(synth.STREAM_W1), np.arange(inner * hidden, dtype=np.uint64)) * np.float32(0.02)
    w2f = synth.normal_f32(seed, synth.stream_id(synth.STREAM_W2), np.arange(2 * inner, dtype=np.uint64)) * np.float32(0.02)
    w1b = synth.f32_to_bf16_bits(w1f).reshape(inner, hidden)
    w2b = synth.f32_to_bf16_bits(w2f).reshape(2, inner)
    b1b = b2b = None
    if bias:
        b1b = synth.f32_to_bf16_bits(synth.normal_f32(seed, synth.stream_id(synth.STREAM_B1), np.arange(inner, dtype=np.uint64)) * np.float32(0.1))
        b2b = synth.f32_to_bf16_bits(synth.normal_f32(seed, synth.stream_id(synth.STREAM_B2), np.arange(2, dtype=np.uint64)) * np.float32(0.01))
    mode = torch.full((len(lens),), 7, dtype=torch.uint8, device="cuda")
    logits = torch.full((len(lens), 2), float("nan"), dtype=torch.float32, device="cuda")
    F.flux_router(ctx, H.bits_to_torch(xb), cu(lens), len(lens), hidden, pool, H.bits_to_torch(w1b),
                  H.bits_to_torch(b1b) if bias else None, H.bits_to_torch(w2b), H.bits_to_torch(b2b) if bias else None,
                  inner, mode, logits)
    torch.cuda.synchronize()
    x = O.bf16_to_f64(xb)
    w1, w2 = O.bf16_to_f64(w1b), O.bf16_to_f64(w2b)
    b1 = O.bf16_to_f64(b1b) if bias else None
    b2 = O.bf16_to_f64(b2b) if bias else None
    off = 0
    margins = []
    for b, n in enumerate(lens):
        ref_logits, ref_mode = O.router(x[off:off + n], pool, w1, b1, w2, b2)
        off += n
        got = logits[b].cpu().numpy().astype(np.float64)
        assert np.abs(got - ref_logits).max() < 1e-6, (b, got, ref_logits)
        margin = abs(ref_logits[0] - ref_logits[1])
        margins.append(margin)
        # the stated tie margin: every decision of the seed must be a real one (a smaller margin anywhere
        # is a bad seed to be replaced, not a kernel failure), and then every decision is bit-exact
        assert margin >= 1e-6, f"seed {seed}: margin {margin:.3e} of sequence {b} is below 1e-6, pick another seed"
        assert int(mode[b]) == ref_mode, (b, got, ref_logits)
    print("router seed", seed, "pool", pool, "bias", bias, "min margin %.3e" % min(margins))
    return margins


@pytest.mark.parametrize("pool", [100, 0, 3])
@pytest.mark.parametrize("bias", [False, True])
def test_router_matches_oracle(F, ctx, pool, bias):
    margins = router_case(F, ctx, 4, [1000, 150, 200, 201, 1, 7], 4096, 256, pool, bias)
    assert min(margins) >= 1e-6                              # every (sequence) decision of the seed is a real one


def test_router_small_shapes(F, ctx):
    router_case(F, ctx, 41, [5, 300], 64, 8, 2, True)
    router_case(F, ctx, 42, [9], 1000, 24, 4, False)


def test_router_zero_head_is_a_tie_and_goes_to_fa(F, ctx):
    x = torch.randn(50, 256, device="cuda").to(torch.bfloat16)
    w1 = (torch.randn(16, 256, device="cuda") * 0.02).to(torch.bfloat16)
    w2 = torch.zeros(2, 16, dtype=torch.bfloat16, device="cuda")
    mode = torch.full((1,), 7, dtype=torch.uint8, device="cuda")
    F.flux_router(ctx, x, cu([50]), 1, 256, 10, w1, None, w2, None, 16, mode)
    torch.cuda.synchronize()
    assert int(mode[0]) == FA


# ----------------------------------------------------------------------------- block-granular SA mask (App. C.3)

@pytest.mark.parametrize("block,n_sink,window", [(64, 128, 256), (16, 20, 100), (64, 1, 1), (128, 100, 300)])
def test_block_granular_prefill_and_decode(F, ctx, block, n_sink, window):
    """Sinks and window rounded to whole blocks (the block is the minimum unit of sparsity): ragged
    multi-tile prefill in two chunks whose boundary is not block-aligned, then decode steps that cross a
    block boundary; mixed with one FA sequence."""
    lens = [700, 333, 64]
    modes = [SA, SA, FA] if block != 16 else [SA, FA, SA]
    lay = Layer(F, ctx, 51, 3, 8, 2, 128, 800, n_sink, window, scales=True, block=block)
    first = [401, 100, 64]
    qb, kb, vb = lay.new_tokens(first)
    lay.append(kb, vb, first)
    got, ref = lay.prefill(qb, first, modes)
    H.assert_close(got, ref, f"block {block} prefill chunk 1")
    rest = [lens[b] - first[b] for b in range(3)]
    qb, kb, vb = lay.new_tokens(rest)
    lay.append(kb, vb, rest)
    got, ref = lay.prefill(qb, rest, modes)
    H.assert_close(got, ref, f"block {block} prefill chunk 2")
    for step in range(block // 8 + 3 if block <= 64 else 6):
        qb, kb, vb = lay.new_tokens([1, 1, 1])
        lay.append(kb, vb, [1, 1, 1])
        got, ref = lay.decode(qb.reshape(3, 8, 128), modes)
        H.assert_close(got, ref, f"block {block} decode step {step}")


def test_block_granular_differs_from_token_exact_and_block_one_does_not(F, ctx):
    """sa_block = 1 and 0 are the token-exact kernel (bit-identical); 64 changes the visible set."""
    outs = {}
    for block in (0, 1, 64):
        lay = Layer(F, ctx, 52, 1, 8, 2, 128, 600, 10, 100)
        lay.cfg = F.attn_cfg(8, 2, 128, 10, 100, 0.0, 1, block)
        qb, kb, vb = lay.new_tokens([600])
        lay.append(kb, vb, [600])
        outs[block], _ = lay.prefill(qb, [600], [SA])
    assert np.array_equal(outs[0], outs[1])
    assert not np.array_equal(outs[0][300:], outs[64][300:])
    assert np.array_equal(outs[0][:64], outs[64][:64])          # the first block row sees everything either way


@pytest.mark.parametrize("block", [1, 64, 4096])
def test_window_of_the_largest_int_equals_fa(F, ctx, block):
    """Eq. (2) with the whole history as its subset is Eq. (1): window = INT32_MAX (rounded up to whole blocks
    without wrapping) gives the FA result bit for bit, in prefill and in decode."""
    big = (1 << 31) - 1
    lay = Layer(F, ctx, 53, 2, 8, 2, 128, 800, 3, big, block=block)
    lens = [700, 333]
    qb, kb, vb = lay.new_tokens(lens)
    lay.append(kb, vb, lens)
    got_sa, ref = lay.prefill(qb, lens, [SA, SA])
    got_fa, _ = lay.prefill(qb, lens, [FA, FA])
    assert np.array_equal(got_sa, got_fa)
    H.assert_close(got_sa, ref, "largest window")
    q1, k1, v1 = lay.new_tokens([1, 1])
    lay.append(k1, v1, [1, 1])
    dec_sa, dref = lay.decode(q1.reshape(2, 8, 128), [SA, SA])
    dec_fa, _ = lay.decode(q1.reshape(2, 8, 128), [FA, FA])
    assert np.array_equal(dec_sa, dec_fa)
    H.assert_close(dec_sa, dref, "largest window, decode")


# ----------------------------------------------------------------------------- cache layouts and degenerate batches

def test_token_major_cache_layout_and_empty_sequences(F, ctx):
    """The cache strides are free: a [B, capacity, Hkv, D] allocation (token-major, stride_t = Hkv * D,
    stride_h = D) passed as its [B, Hkv, capacity, D] view must behave like the head-major one, in append,
    prefill and decode.  The batch has a sequence with no new tokens in the first call and a one-token one."""
    B, hq, hkv, d, cap = 3, 8, 2, 128, 700
    lay = Layer(F, ctx, 61, B, hq, hkv, d, cap, 16, 96, scales=True)
    km = torch.empty(B, cap, hkv, d, dtype=torch.bfloat16, device="cuda")
    vm = torch.empty(B, cap, hkv, d, dtype=torch.bfloat16, device="cuda")
    lay.cache = F.KVCache(km.permute(0, 2, 1, 3), vm.permute(0, 2, 1, 3), torch.zeros(B, dtype=torch.int32, device="cuda"))
    assert lay.cache.k.stride() == (cap * hkv * d, d, hkv * d, 1)
    first = [300, 0, 1]
    qb, kb, vb = lay.new_tokens(first)
    lay.append(kb, vb, first)
    got, ref = lay.prefill(qb, first, [SA, FA, SA])
    H.assert_close(got, ref, "token-major prefill, empty middle sequence")
    assert lay.cache.kv_len.cpu().tolist() == first
    second = [257, 130, 0]
    qb, kb, vb = lay.new_tokens(second)
    lay.append(kb, vb, second)
    got, ref = lay.prefill(qb, second, [SA, FA, SA])
    H.assert_close(got, ref, "token-major prefill, second chunk")
    for step in range(3):
        qb, kb, vb = lay.new_tokens([1, 1, 1])
        lay.append(kb, vb, [1, 1, 1])
        got, ref = lay.decode(qb.reshape(B, hq, d), [SA, FA, SA])
        H.assert_close(got, ref, f"token-major decode step {step}")
    # the rows sit where the token-major layout says
    kd = H.torch_to_f64(km[0, :lay.lens[0]])
    assert np.array_equal(kd, lay.ocache.k[0])
    assert F.flux_last_device_status(ctx) == 0


def test_decode_with_an_empty_cache_row_returns_zeros(F, ctx):
    """kv_len = 0 for one sequence: nothing to attend, the output row is zeros (not NaN), others are unaffected."""
    lay = Layer(F, ctx, 62, 2, 8, 2, 128, 300, 8, 64)
    _, kb, vb = lay.new_tokens([200, 0])
    lay.append(kb, vb, [200, 0])
    qb = lay._draw(synth.STREAM_Q, 2, 8, None)
    out = torch.full((2, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    F.flux_attn_decode(ctx, lay.cfg, H.bits_to_torch(qb), 200, lay.cache, u8([SA, FA]), out)
    torch.cuda.synchronize()
    ref = O.attention(O.bf16_to_f64(qb[0])[None], lay.ocache.k[0], lay.ocache.v[0], SA, 8, 64)[0]
    H.assert_close(out[0].cpu().numpy(), ref, "non-empty sequence next to an empty one")
    assert torch.equal(out[1], torch.zeros_like(out[1]))


def test_inconsistent_lengths_are_clamped_and_flagged(F, ctx):
    """kv_len values the host cannot see: past the capacity in decode, fewer cached positions than queries
    in prefill.  Nothing leaves the buffers, the sticky status word reports FLUX_DEV_BAD_LENGTH once read."""
    lay = Layer(F, ctx, 63, 1, 8, 2, 128, 256, 8, 64)
    qb, kb, vb = lay.new_tokens([256])
    lay.append(kb, vb, [256])
    assert F.flux_last_device_status(ctx) == 0
    q1 = qb[255].reshape(1, 8, 128)
    good, ref = lay.decode(q1, [FA])
    H.assert_close(good, ref, "decode at capacity")
    lay.cache.kv_len.fill_(256 + 5)                                   # corrupt: beyond the buffers
    out = torch.full((1, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    F.flux_attn_decode(ctx, lay.cfg, H.bits_to_torch(q1), 256, lay.cache, u8([FA]), out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), good)                    # clamped to the capacity
    assert F.flux_last_device_status(ctx) & F.FLUX_DEV_BAD_LENGTH
    assert F.flux_last_device_status(ctx) == 0                        # reading clears it
    # a host bound below what a sequence attends to: the visible list is cut at the bound and the cut reported
    lay.cache.kv_len.fill_(256)
    F.flux_attn_decode(ctx, lay.cfg, H.bits_to_torch(q1), 100, lay.cache, u8([FA]), out)
    torch.cuda.synchronize()
    cut = O.attention(O.bf16_to_f64(q1), lay.ocache.k[0][:100], lay.ocache.v[0][:100], FA, 8, 64)[0]
    H.assert_close(out[0].cpu().numpy(), cut, "decode cut at the host bound")
    assert F.flux_last_device_status(ctx) & F.FLUX_DEV_BAD_LENGTH
    lay.cache.kv_len.fill_(50)                                        # fewer cached positions than queries
    outp = torch.full((100, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    F.flux_attn_prefill(ctx, lay.cfg, H.bits_to_torch(qb[:100]), cu([100]), 100, 256, lay.cache, u8([SA]), outp)
    torch.cuda.synchronize()
    # only as many query rows as there are cached positions are computed (as the last 50 positions of a
    # 50-token cache); the surplus rows are left alone
    ref = O.attention(O.bf16_to_f64(qb[:50]), lay.ocache.k[0][:50], lay.ocache.v[0][:50], SA, 8, 64)
    H.assert_close(outp[:50].cpu().numpy(), ref, "prefill with more queries than cached positions")
    assert torch.isnan(outp[50:]).all()
    assert F.flux_last_device_status(ctx) & F.FLUX_DEV_BAD_LENGTH


def test_workspace_sizing_for_decode(F):
    """A context made with the size flux_workspace_needed reports runs the decode it was sized for; one made
    with a smaller workspace refuses it with FLUX_EWORKSPACE before anything is launched."""
    hq, hkv, d, batch, n = 16, 8, 128, 12, 900
    cfg = F.attn_cfg(hq, hkv, d, 8, 64, 0.0, 1)
    need = F.flux_workspace_needed(cfg, batch, n)
    assert need > 0
    cache = F.KVCache.empty(batch, hkv, n, d)
    cache.kv_len.fill_(n)
    cache.k.normal_()
    cache.v.normal_()
    q = torch.randn(batch, hq, d, device="cuda").to(torch.bfloat16)
    mode = torch.ones(batch, dtype=torch.uint8, device="cuda")
    outs = []
    for size in (need, 0):
        c = F.flux_create(0, size)
        out = torch.full((batch, hq, d), float("nan"), dtype=torch.float32, device="cuda")
        F.flux_attn_decode(c, cfg, q, n, cache, mode, out)
        torch.cuda.synchronize()
        assert torch.isfinite(out).all()
        outs.append(out)
        F.flux_destroy(c)
    assert torch.equal(outs[0], outs[1])
    small = F.flux_create(0, 1)                                       # rounded up to the smallest context
    out = torch.full((batch, hq, d), float("nan"), dtype=torch.float32, device="cuda")
    with pytest.raises(F.FluxError) as e:
        F.flux_attn_decode(small, cfg, q, n, cache, mode, out)
    assert e.value.code == F.FLUX_EWORKSPACE
    torch.cuda.synchronize()
    assert torch.isnan(out).all()                                     # nothing was launched
    F.flux_destroy(small)
