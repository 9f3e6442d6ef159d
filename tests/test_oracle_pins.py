"""Pins for the CPU oracle: closed forms, invariants, special cases and brute force.

Each test is chosen so that a plausible mistake in oracle/flux_oracle.py (a
dropped term, an off-by-one in the window, a transposed operand, a wrong GQA
group, a missing scale) fails it.  Nothing here touches the GPU.
"""
import math

import numpy as np
import pytest

from oracle import flux_oracle as O

FA, SA = O.FA, O.SA


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------- mask

def closed_form_visible(i, n_sink, window):
    """Keys seen by SA row i: the window part plus the sinks that lie before the window."""
    return min(i + 1, window) + max(0, min(n_sink, i + 1 - window))


@pytest.mark.parametrize("n,n_sink,window", [(40, 0, 1), (40, 3, 5), (64, 16, 16), (50, 7, 64), (33, 40, 4)])
def test_visible_count_closed_form(n, n_sink, window):
    m = O.mask_matrix(n, n, SA, n_sink, window)
    for i in range(n):
        assert m[i].sum() == closed_form_visible(i, n_sink, window), i
    # never anything from the future, always the query's own position
    assert not np.triu(m, 1).any()
    assert m.diagonal().all()


def test_visible_pair_totals_config_shapes():
    # Tiny config: S 512, 16 sinks, window 128 (values derived by hand from the closed form)
    m = O.mask_matrix(512, 512, SA, 16, 128)
    assert int(m.sum()) == 63432
    assert int(O.mask_matrix(512, 512, FA, 16, 128).sum()) == 131328
    # Stack-prefill config: S 32768, 128 sinks, window 4096, counted row block by row block
    total_sa = total_fa = 0
    n = 32768
    j = np.arange(n)[None, :]
    for r0 in range(0, n, 2048):
        i = np.arange(r0, r0 + 2048)[:, None]
        total_sa += int(O.visible(i, j, SA, 128, 4096).sum())
        total_fa += int(O.visible(i, j, FA, 128, 4096).sum())
    assert total_sa == 129_493_056
    assert total_fa == 536_887_296
    # High-sparsity config: S 65536, 64 sinks, window 2048.  The predicate is evaluated on two disjoint key
    # slices per block of 1024 rows: the sinks below the slice, and everything from `window` keys before the
    # block's first row to its last row (no other key can be visible to a row of the block); sampled whole
    # rows below check that nothing outside the slices is.
    n, n_sink, window = 65536, 64, 2048
    total_sa = 0
    for r0 in range(0, n, 1024):
        i = np.arange(r0, r0 + 1024)[:, None]
        lo = max(0, r0 - window)
        total_sa += int(O.visible(i, np.arange(lo, r0 + 1024)[None, :], SA, n_sink, window).sum())
        total_sa += int(O.visible(i, np.arange(0, min(n_sink, lo))[None, :], SA, n_sink, window).sum())
    for i in (0, 63, 64, 2047, 2048, 2111, 2112, 40000, 65535):   # whole rows against the closed form
        assert int(O.visible(i, np.arange(n), SA, n_sink, window).sum()) == closed_form_visible(i, n_sink, window)
    assert total_sa == 136_182_816
    assert n * (n + 1) // 2 == 2_147_516_416
    assert int(O.visible(np.arange(n - 64, n)[:, None], np.arange(n)[None, :], FA, n_sink, window).sum()) == sum(range(n - 63, n + 1))


def test_query_rows_are_the_last_positions():
    # 3 queries over 10 cached positions: rows are positions 7, 8, 9
    m = O.mask_matrix(3, 10, SA, 2, 3)
    expect = np.zeros((3, 10), bool)
    for r, i in enumerate((7, 8, 9)):
        for j in range(10):
            expect[r, j] = j <= i and (j < 2 or i - j < 3)
    assert (m == expect).all()


# ----------------------------------------------------------------------------- attention

def make_qkv(seed, n_q, n_kv, hq, hkv, d):
    r = rng(seed)
    return (r.standard_normal((n_q, hq, d)), r.standard_normal((n_kv, hkv, d)),
            r.standard_normal((n_kv, hkv, d)))


def test_sa_with_window_covering_sequence_is_fa_bit_for_bit():
    q, k, v = make_qkv(1, 48, 48, 4, 2, 8)
    fa = O.attention(q, k, v, FA, 0, 0)
    assert np.array_equal(O.attention(q, k, v, SA, 0, 48), fa)
    assert np.array_equal(O.attention(q, k, v, SA, 5, 4096), fa)
    assert np.array_equal(O.attention(q, k, v, SA, 48, 1), fa)      # sinks alone cover it


def test_window_one_no_sinks_returns_own_value():
    q, k, v = make_qkv(2, 20, 20, 4, 2, 8)
    out = O.attention(q, k, v, SA, 0, 1)
    for h in range(4):
        assert np.allclose(out[:, h], v[:, h // 2], atol=0, rtol=0)


def test_probability_rows_sum_to_one_and_respect_mask():
    q, k, v = make_qkv(3, 30, 30, 2, 1, 4)
    for mode in (FA, SA):
        _, p = O.attention(q, k, v, mode, 3, 6, return_probs=True)
        assert np.abs(p.sum(-1) - 1).max() < 1e-15
        m = O.mask_matrix(30, 30, mode, 3, 6)
        assert (p[:, ~m] == 0).all() and (p[:, m] > 0).all()


def test_constant_values_and_first_row():
    q, k, v = make_qkv(4, 16, 16, 4, 4, 8)
    ones = np.ones_like(v)
    for mode in (FA, SA):
        assert np.abs(O.attention(q, k, ones, mode, 2, 4) - 1).max() < 1e-15
        out = O.attention(q, k, v, mode, 2, 4)
        assert np.array_equal(out[0], v[0])                   # row 0 sees only key 0


def test_identical_keys_give_plain_mean_of_visible_values():
    q, k, v = make_qkv(5, 24, 24, 2, 1, 4)
    k[:] = k[0]
    out = O.attention(q, k, v, SA, 2, 5)
    m = O.mask_matrix(24, 24, SA, 2, 5)
    for i in range(24):
        assert np.allclose(out[i, 0], v[m[i], 0].mean(0), atol=1e-14)
        assert np.allclose(out[i, 1], v[m[i], 0].mean(0), atol=1e-14)


def test_shift_invariance_of_scores():
    # add the same vector u to every key: each score of row i moves by scale * q_i.u, the same
    # for all keys of the row, so O is unchanged
    q, k, v = make_qkv(6, 12, 12, 2, 2, 8)
    u = rng(60).standard_normal(8)
    a = O.attention(q, k, v, FA, 0, 0)
    b = O.attention(q, k + u, v, FA, 0, 0)
    assert np.abs(a - b).max() < 1e-12


def brute_force(q, k, v, mode, n_sink, window):
    """Independent enumeration in pure-Python loops, no max-subtraction, own mask predicate."""
    n_q, hq, d = q.shape
    n_kv, hkv, _ = k.shape
    group = hq // hkv
    out = [[[0.0] * d for _ in range(hq)] for _ in range(n_q)]
    for r in range(n_q):
        i = n_kv - n_q + r
        for h in range(hq):
            kvh = h // group
            weights = {}
            for j in range(n_kv):
                if j > i:
                    continue
                if mode == SA and not (j < n_sink or (i - j) <= window - 1):
                    continue
                dot = 0.0
                for t in range(d):
                    dot += q[r, h, t] * k[j, kvh, t]
                weights[j] = math.exp(dot / math.sqrt(d))
            z = sum(weights.values())
            for j, w in weights.items():
                for t in range(d):
                    out[r][h][t] += w / z * v[j, kvh, t]
    return np.array(out)


@pytest.mark.parametrize("mode,n_sink,window", [(FA, 0, 0), (SA, 2, 3), (SA, 0, 2), (SA, 1, 1), (SA, 3, 8)])
def test_brute_force_eight_tokens(mode, n_sink, window):
    q, k, v = make_qkv(7, 8, 8, 2, 1, 4)
    assert np.abs(O.attention(q, k, v, mode, n_sink, window) - brute_force(q, k, v, mode, n_sink, window)).max() < 1e-12
    # chunked: 3 new queries over 8 cached positions
    assert np.abs(O.attention(q[5:], k, v, mode, n_sink, window)
                  - brute_force(q[5:], k, v, mode, n_sink, window)).max() < 1e-12


def test_row_form_matches_matrix_form_and_brute_force():
    q, k, v = make_qkv(8, 8, 8, 4, 2, 4)
    ref = brute_force(q, k, v, SA, 2, 3)
    for i in range(8):
        for kvh in range(2):
            row = O.attention_row(q[i, 2 * kvh:2 * kvh + 2], k[:, kvh], v[:, kvh], i, SA, 2, 3)
            assert np.abs(row - ref[i, 2 * kvh:2 * kvh + 2]).max() < 1e-12


def test_textbook_dense_formula_no_gqa():
    # FA with one KV head per query head is softmax(Q K^T / sqrt(d) + causal) V
    q, k, v = make_qkv(9, 32, 32, 3, 3, 16)
    out = O.attention(q, k, v, FA, 0, 0)
    for h in range(3):
        s = q[:, h] @ k[:, h].T / np.sqrt(16.0)
        s = s + np.triu(np.full((32, 32), -np.inf), 1)
        e = np.exp(s - s.max(1, keepdims=True))
        ref = (e / e.sum(1, keepdims=True)) @ v[:, h]
        assert np.abs(out[:, h] - ref).max() < 1e-13


def test_explicit_scale_is_used():
    q, k, v = make_qkv(10, 8, 8, 2, 2, 4)
    a = O.attention(q, k, v, FA, 0, 0, scale=0.5)          # 1/sqrt(4): the default
    assert np.array_equal(a, O.attention(q, k, v, FA, 0, 0))
    assert np.abs(a - O.attention(q, k, v, FA, 0, 0, scale=1.0)).max() > 1e-3
    assert np.abs(O.attention(2 * q, k, v, FA, 0, 0, scale=0.25) - a).max() < 1e-13


def test_gqa_equals_repeated_kv_heads():
    q, k, v = make_qkv(11, 16, 16, 6, 2, 8)
    a = O.attention(q, k, v, SA, 2, 5)
    b = O.attention(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), SA, 2, 5)
    assert np.array_equal(a, b)
    # and the group order is h // G, not h % G
    c = O.attention(q, np.tile(k, (1, 3, 1)), np.tile(v, (1, 3, 1)), SA, 2, 5)
    assert np.abs(a - c).max() > 1e-3


def test_decode_equals_last_prefill_row():
    n, hq, hkv, d = 20, 4, 2, 8
    q, k, v = make_qkv(12, n, n, hq, hkv, d)
    for mode in (FA, SA):
        full = O.attention(q, k, v, mode, 2, 4)
        cache = O.KVCache(1, hkv, d)
        cache.append(0, k[:10], v[:10])
        for t in range(10, n):
            out = O.decode_step(cache, q[t][None], k[t][None], v[t][None], [mode], 2, 4)
            assert np.abs(out[0] - full[t]).max() < 1e-14
        assert cache.length(0) == n


def test_prefill_ragged_batch_and_chunks():
    hq, hkv, d = 2, 1, 4
    lens = [5, 9]
    data = [make_qkv(20 + b, n, n, hq, hkv, d) for b, n in enumerate(lens)]
    cache = O.KVCache(2, hkv, d)
    # two chunks per sequence must equal one shot
    outs1 = O.prefill(cache, [x[0][:3] for x in data], [x[1][:3] for x in data], [x[2][:3] for x in data], [FA, SA], 1, 2)
    outs2 = O.prefill(cache, [x[0][3:] for x in data], [x[1][3:] for x in data], [x[2][3:] for x in data], [FA, SA], 1, 2)
    for b, mode in enumerate([FA, SA]):
        qq, kk, vv = data[b]
        whole = O.attention(qq, kk, vv, mode, 1, 2)
        assert np.abs(np.concatenate([outs1[b], outs2[b]]) - whole).max() < 1e-14


# ----------------------------------------------------------------------------- router

def test_pooled_rows():
    assert list(O.pooled_rows(10, 2)) == [0, 1, 8, 9]
    assert list(O.pooled_rows(4, 2)) == [0, 1, 2, 3]         # stretches meet: every row once
    assert list(O.pooled_rows(3, 2)) == [0, 1, 2]            # stretches overlap: every row once
    assert list(O.pooled_rows(5, 0)) == [0, 1, 2, 3, 4]      # pool 0 = whole sequence
    assert list(O.pooled_rows(5, 2)) == [0, 1, 3, 4]


def test_router_hand_computation():
    # S 6, pool 2 -> rows 0, 1, 4, 5; the middle rows must not matter
    x = np.array([[1, 2, 3, 4], [3, 2, 1, 0], [100, -50, 7, 9], [-3, 8, 1e3, 2], [1, 0, 1, 0], [3, 4, -1, 8]], float)
    # pooled mean by hand: [8/4, 8/4, 4/4, 12/4] = [2, 2, 1, 3]
    w1 = np.array([[1, -1, 2, 0], [0.5, 0, -1, 0.5]])        # W1 p = [2, 1.5]
    b1 = np.array([-1, 0.5])                                 # pre-activation [1, 2]
    w2 = np.array([[1, 2], [3, -1]])
    b2 = np.array([0.25, -0.5])
    silu1 = 0.7310585786300049                               # 1 * sigmoid(1)
    silu2 = 2 * 0.8807970779778823                           # 2 * sigmoid(2)
    pi_fa = 1 * silu1 + 2 * silu2 + 0.25
    pi_sa = 3 * silu1 - 1 * silu2 - 0.5
    logits, mode = O.router(x, 2, w1, b1, w2, b2)
    assert abs(logits[0] - pi_fa) < 1e-12 and abs(logits[1] - pi_sa) < 1e-12
    assert abs(logits[0] - 4.504246890541535) < 1e-12 and abs(logits[1] - (-0.06841842006575)) < 1e-12
    assert mode == FA
    # swapping the two head rows flips the decision: r_hard = 0 <=> SA
    logits2, mode2 = O.router(x, 2, w1, b1, w2[::-1], b2[::-1])
    assert np.allclose(logits2, logits[::-1], atol=0) and mode2 == SA
    # no biases
    l3, _ = O.router(x, 2, w1, None, w2, None)
    h = np.array([2 / (1 + math.exp(-2)), 1.5 / (1 + math.exp(-1.5))])
    assert np.abs(l3 - w2 @ h).max() < 1e-12
    # whole-sequence pooling sees the middle rows
    l4, _ = O.router(x, 0, w1, b1, w2, b2)
    assert abs(l4[0] - logits[0]) > 1e-3


def test_router_tie_goes_to_fa():
    x = rng(30).standard_normal((7, 4))
    w1 = rng(31).standard_normal((3, 4))
    logits, mode = O.router(x, 2, w1, None, np.zeros((2, 3)), None)
    assert logits[0] == logits[1] == 0 and mode == FA


def test_model_sparsity_ratio():
    assert O.model_sparsity_ratio([FA, SA, FA, SA]) == 0.5
    assert O.model_sparsity_ratio([[FA, FA], [SA, FA]]) == 0.25
    assert O.model_sparsity_ratio([FA] * 4) == 0.0


def test_bf16_widening_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3DCD, 0x0000, 0x7F7F], dtype=np.uint16)
    vals = O.bf16_to_f64(bits)
    assert vals[0] == 1.0 and vals[1] == -1.0 and vals[2] == 2.0 and vals[4] == 0.0
    assert vals[3] == 0.10009765625                      # 0x3DCD = 1.6015625 * 2**-4
    assert vals[5] == (2 - 2 ** -7) * 2.0 ** 127


# ----------------------------------------------------------------------------- sparse-decode residency (Sec. 3.3)

@pytest.mark.parametrize("n_sink,window", [(3, 5), (0, 4), (4, 1), (2, 7)])
def test_ring_stores_exactly_the_visible_set(n_sink, window):
    """After n appended rows the ring holds positions {0..n_sink-1} and {n-window..n-1}, each once,
    never more than n_sink + window rows: the set Eq. (2) lets the newest position see."""
    g = rng(30)
    ring = O.RingKVCache(1, 1, 2, n_sink, window)
    for n in range(1, 4 * (n_sink + window) + 3):
        row = g.standard_normal((1, 1, 2))
        ring.append(0, row, -row)
        pos, kk, vv = ring.stored(0)
        want = sorted(set(range(min(n_sink, n))) | set(range(max(n - window, 0), n)))
        assert pos.tolist() == want
        assert len(pos) == closed_form_visible(n - 1, n_sink, window) <= n_sink + window
        assert np.array_equal(vv, -kk)                      # K and V of a position travel together
        assert np.array_equal(kk[-1], row[0])               # the newest row is the last stored position


def test_ring_decode_equals_full_cache_sa_decode_bit_for_bit():
    """The minimal cache changes where rows live, not what is computed: step by step, across several
    wrap-arounds of the ring, the output equals the SA decode step on the full history exactly."""
    g = rng(31)
    B, Hq, Hkv, D, n_sink, window = 2, 4, 2, 8, 3, 5
    full = O.KVCache(B, Hkv, D)
    ring = O.RingKVCache(B, Hkv, D, n_sink, window)
    prompt = [g.standard_normal((4, Hkv, D)), g.standard_normal((11, Hkv, D))]   # one shorter, one longer than the ring
    pv = [g.standard_normal(p.shape) for p in prompt]
    for b in range(B):
        full.append(b, prompt[b], pv[b])
    O.compact_to_ring(full, ring)
    assert [ring.length(b) for b in range(B)] == [4, 11]
    for step in range(23):
        q = g.standard_normal((B, Hq, D))
        kn, vn = g.standard_normal((B, Hkv, D)), g.standard_normal((B, Hkv, D))
        ref = O.decode_step(full, q, kn, vn, [SA, SA], n_sink, window)
        got = O.decode_step_ring(ring, q, kn, vn)
        assert np.allclose(got, ref, rtol=0, atol=1e-13), step
    assert [ring.length(b) for b in range(B)] == [27, 34]


def test_ring_compaction_equals_row_by_row_appends_and_bulk_append():
    g = rng(32)
    n_sink, window = 2, 4
    k, v = g.standard_normal((17, 1, 3)), g.standard_normal((17, 1, 3))
    full = O.KVCache(1, 1, 3)
    full.append(0, k, v)
    a = O.RingKVCache(1, 1, 3, n_sink, window)
    O.compact_to_ring(full, a)
    b_ = O.RingKVCache(1, 1, 3, n_sink, window)
    for r in range(17):
        b_.append(0, k[r:r + 1], v[r:r + 1])
    c = O.RingKVCache(1, 1, 3, n_sink, window)
    c.append(0, k[:9], v[:9])
    c.append(0, k[9:], v[9:])
    for other in (b_, c):
        assert np.array_equal(a.pos[0], other.pos[0]) and np.array_equal(a.k[0], other.k[0]) and np.array_equal(a.v[0], other.v[0])
    assert a.pos[0].tolist() == [0, 1, 14, 15, 16, 13]      # rows 2..5 hold the p with (p - 2) % 4 = 0..3


# ----------------------------------------------------------------------------- block-granular mask (App. C.3)

def test_block_one_is_the_token_exact_mask():
    for n_sink, window in [(3, 5), (0, 7), (16, 16)]:
        assert np.array_equal(O.mask_matrix(50, 50, SA, n_sink, window, block=1), O.mask_matrix(50, 50, SA, n_sink, window))


@pytest.mark.parametrize("n,n_sink,window,block", [(96, 8, 16, 8), (100, 5, 20, 8), (70, 0, 9, 4), (128, 128, 64, 64), (40, 3, 1, 4)])
def test_block_is_the_minimum_unit_of_sparsity(n, n_sink, window, block):
    """Off the diagonal every block x block tile of the mask is all-kept or all-dropped; the diagonal tile is
    the causal triangle; the kept block columns of block row R are the first ceil(n_sink / block) and the
    ceil(window / block) most recent, counted without overlap (closed form); written without O.visible."""
    m = O.mask_matrix(n, n, SA, n_sink, window, block)
    sb, wb = math.ceil(n_sink / block), math.ceil(window / block)
    for R in range(math.ceil(n / block)):
        rows = slice(R * block, min((R + 1) * block, n))
        kept = 0
        for Cb in range(R + 1):
            cols = slice(Cb * block, min((Cb + 1) * block, n))
            tile = m[rows, cols]
            if Cb == R:
                assert np.array_equal(tile, np.tril(np.ones(tile.shape, dtype=bool)))
                kept += 1
            else:
                assert tile.all() or not tile.any()
                assert tile.all() == (Cb < sb or R - Cb < wb)
                kept += int(tile.all())
        assert kept == min(R + 1, wb) + max(0, min(sb, R + 1 - wb))
        assert not m[rows, (R + 1) * block:].any()                      # nothing from the future


def test_block_granular_attention_matches_brute_force():
    """Pure-Python enumeration of (i, j) pairs with the block rule spelled out from scratch."""
    g = rng(40)
    n, d, n_sink, window, block = 23, 4, 3, 6, 4
    q, k, v = g.standard_normal((n, 2, d)), g.standard_normal((n, 1, d)), g.standard_normal((n, 1, d))
    out = O.attention(q, k, v, SA, n_sink, window, block=block)
    sink_blocks, window_blocks = 1, 2                                     # ceil(3 / 4), ceil(6 / 4)
    for i in range(n):
        for h in range(2):
            num, den = np.zeros(d), 0.0
            for j in range(i + 1):
                if j // block < sink_blocks or i // block - j // block < window_blocks:
                    w = math.exp(float(q[i, h] @ k[j, 0]) / math.sqrt(d))
                    num += w * v[j, 0]
                    den += w
            assert np.allclose(out[i, h], num / den, rtol=0, atol=1e-12)
    # the row form agrees with the matrix form
    for i in (0, 3, 4, 11, 22):
        assert np.allclose(O.attention_row(q[i], k[:, 0], v[:, 0], i, SA, n_sink, window, block=block), out[i], rtol=0, atol=1e-13)


def test_block_granular_decode_equals_last_prefill_row():
    g = rng(41)
    n, n_sink, window, block = 37, 5, 9, 4
    q, k, v = g.standard_normal((n, 4, 8)), g.standard_normal((n, 2, 8)), g.standard_normal((n, 2, 8))
    whole = O.attention(q, k, v, SA, n_sink, window, block=block)
    cache = O.KVCache(1, 2, 8)
    cache.append(0, k[:-1], v[:-1])
    step = O.decode_step(cache, q[-1][None], k[-1][None], v[-1][None], [SA], n_sink, window, block=block)
    assert np.allclose(step[0], whole[-1], rtol=0, atol=1e-13)


# ----------------------------------------------------------------------------- block-sparse mask (Eq. 2 over key blocks)

def brute_force_block_sparse(q, k, v, bm, blk):
    """Pure-Python enumeration: pair (i, j) counts iff j <= i and (its block pair is kept or is the diagonal)."""
    n_q, hq, d = q.shape
    n_kv, hkv, _ = k.shape
    g = hq // hkv
    pos0 = n_kv - n_q
    out = np.zeros((n_q, hq, d))
    for r in range(n_q):
        i = pos0 + r
        for h in range(hq):
            num = [0.0] * d
            den = 0.0
            for j in range(n_kv):
                if j > i:
                    continue
                if not (bm[i // blk - pos0 // blk][j // blk] or i // blk == j // blk):
                    continue
                sc = sum(q[r, h, t] * k[j, h // g, t] for t in range(d)) / math.sqrt(d)
                w = math.exp(sc)
                den += w
                for t in range(d):
                    num[t] += w * v[j, h // g, t]
            out[r, h] = [x / den for x in num]
    return out


@pytest.mark.parametrize("n_q,n_kv", [(19, 19), (7, 19), (1, 19), (12, 20)])
def test_block_sparse_attention_matches_brute_force(n_q, n_kv):
    blk = 4
    q, k, v = make_qkv(61, n_q, n_kv, 4, 2, 3)
    n_kb = -(-n_kv // blk)
    n_qb = (n_kv - 1) // blk - (n_kv - n_q) // blk + 1
    bm = rng(62).random((n_qb, n_kb)) < 0.4
    got = O.attention(q, k, v, FA, 0, 1, block_mask=bm, mask_block=blk)
    assert np.abs(got - brute_force_block_sparse(q, k, v, bm, blk)).max() < 1e-12
    # per-head masks: head h uses its own matrix
    bmh = rng(63).random((4, n_qb, n_kb)) < 0.5
    got_h = O.attention(q, k, v, FA, 0, 1, block_mask=bmh, mask_block=blk)
    for h in range(4):
        one = O.attention(q, k, v, FA, 0, 1, block_mask=bmh[h], mask_block=blk)
        assert np.array_equal(got_h[:, h], one[:, h])


def test_block_sparse_row_form_matches_matrix_form():
    blk, n = 4, 37
    q, k, v = make_qkv(65, n, n, 3, 1, 5)
    nb = -(-n // blk)
    bm = rng(66).random((nb, nb)) < 0.35
    full = O.attention(q, k, v, FA, 0, 1, block_mask=bm, mask_block=blk)
    for i in (0, 3, 4, 17, 36):
        row = O.attention_row(q[i], k[:, 0], v[:, 0], i, FA, 0, 1, block_row=bm[i // blk], mask_block=blk)
        assert np.abs(row - full[i]).max() < 1e-13


def test_block_mask_all_true_is_fa_and_sink_window_blocks_are_block_granular_sa():
    blk, n = 8, 100
    q, k, v = make_qkv(64, n, n, 4, 2, 8)
    nb = -(-n // blk)
    assert np.array_equal(O.attention(q, k, v, FA, 0, 1, block_mask=np.ones((nb, nb), bool), mask_block=blk),
                          O.attention(q, k, v, FA, 0, 1))
    # the streaming pattern written as a block mask: first ceil(n_sink/blk) blocks + the ceil(window/blk) newest
    n_sink, window = 10, 20
    bi, bj = np.arange(nb)[:, None], np.arange(nb)[None, :]
    bm = (bj < -(-n_sink // blk)) | (bi - bj < -(-window // blk))
    assert np.array_equal(O.attention(q, k, v, FA, 0, 1, block_mask=bm, mask_block=blk),
                          O.attention(q, k, v, SA, n_sink, window, block=blk))
    # an all-false mask still keeps every query's own block (nothing else)
    diag_only = O.attention(q, k, v, FA, 0, 1, block_mask=np.zeros((nb, nb), bool), mask_block=blk)
    assert np.array_equal(diag_only, O.attention(q, k, v, FA, 0, 1, block_mask=np.eye(nb, dtype=bool), mask_block=blk))
    assert np.array_equal(diag_only[:blk], O.attention(q, k, v, FA, 0, 1)[:blk])    # block row 0 is plain causal


# ----------------------------------------------------------------------------- XAttention block selection (this build's reading)

def xa_mass_independent(q, k, stride, blk):
    """The same masses from a different formulation: the sampled pairs are those with
    (i + j) % stride == stride - 1 (the antidiagonals of the stride x stride squares), found by scanning the
    whole causal score matrix."""
    n, d = q.shape
    n_sq = -(-n // stride)
    tot = np.zeros((n_sq, n_sq))
    cnt = np.zeros((n_sq, n_sq))
    for i in range(n):
        for j in range(i + 1):
            if (i + j) % stride == stride - 1:
                tot[i // stride, j // stride] += float(q[i] @ k[j]) / math.sqrt(d)
                cnt[i // stride, j // stride] += 1
    per = blk // stride
    n_blk = -(-n // blk)
    mass = np.zeros((n_blk, n_blk))
    for a in range(n_sq):
        cols = [b for b in range(a + 1) if cnt[a, b] > 0]
        e = np.array([tot[a, b] / cnt[a, b] for b in cols])
        w = np.exp(e - e.max())
        w /= w.sum()
        rows_in_block = min(per, n_sq - (a // per) * per)
        for b, x in zip(cols, w):
            mass[a // per, b // per] += x / rows_in_block
    return mass


@pytest.mark.parametrize("n,stride,blk", [(64, 4, 8), (61, 4, 8), (50, 2, 4), (96, 16, 32)])
def test_xa_block_mass_against_independent_scan(n, stride, blk):
    r = rng(71)
    q, k = r.standard_normal((n, 6)), r.standard_normal((n, 6))
    mass = O.xa_block_mass(q, k, stride, blk)
    assert np.abs(mass - xa_mass_independent(q, k, stride, blk)).max() < 1e-12
    assert np.abs(mass.sum(axis=1) - 1.0).max() < 1e-12                 # a query block's masses sum to one
    assert (np.triu(mass, 1) == 0).all()                                # nothing above the block diagonal
    # strided form (what a fast kernel computes): square (a, b) is one dot product of the stride query rows
    # in order against the stride key rows in inverse order, over stride * D numbers
    if n % stride == 0:
        qr = q.reshape(n // stride, stride * 6)
        kr = k.reshape(n // stride, stride, 6)[:, ::-1].reshape(n // stride, stride * 6)
        e = (qr @ kr.T) / math.sqrt(6) / stride
        a, b = 3, 1                                                      # an off-diagonal square: all samples causal
        s = (q @ k.T) / math.sqrt(6)
        assert abs(e[a, b] - np.mean([s[stride * a + t, stride * b + stride - 1 - t] for t in range(stride)])) < 1e-12


def test_xa_constant_inputs_closed_form():
    """Equal scores everywhere: row a of the squares spreads its probability evenly over its a + 1 squares."""
    n, stride, blk = 64, 4, 16
    q = np.ones((n, 3))
    k = np.ones((n, 3))
    mass = O.xa_block_mass(q, k, stride, blk)
    per = blk // stride
    for bi in range(n // blk):
        for bj in range(bi + 1):
            expect = sum(len([b for b in range(per * bj, per * (bj + 1)) if b <= a]) / (a + 1)
                         for a in range(per * bi, per * (bi + 1))) / per
            assert abs(mass[bi, bj] - expect) < 1e-12


def test_xa_select_threshold_limits_monotonicity_and_a_dominant_key():
    n, stride, blk = 128, 4, 16
    r = rng(72)
    q, k = r.standard_normal((n, 8)), r.standard_normal((n, 8))
    nb = n // blk
    tri = np.tril(np.ones((nb, nb), bool))
    assert np.array_equal(O.xa_select(q, k, stride, 1.0, blk), tri)     # everything with mass is needed to reach 1
    keep0, mass = O.xa_select(q, k, stride, 1e-9, blk, return_mass=True)
    for bi in range(nb):                                                # only the heaviest block, and the diagonal
        assert set(np.nonzero(keep0[bi])[0]) == {int(np.argmax(mass[bi, :bi + 1])), bi}
    prev = keep0
    for t in (0.3, 0.6, 0.9, 0.99):
        cur, m = O.xa_select(q, k, stride, t, blk, return_mass=True)
        assert (cur | ~prev).all()                                      # a larger threshold never drops a block
        for bi in range(nb):
            kept = m[bi][cur[bi]].sum()
            assert kept >= t - 1e-12                                    # the kept blocks reach the threshold ...
            off_diag = cur[bi].copy()
            off_diag[bi] = False
            if off_diag.any():                                          # ... and the blocks strictly heavier than the
                lightest = m[bi][off_diag].min()                        # lightest kept one would not have reached it
                assert m[bi, :bi + 1][m[bi, :bi + 1] > lightest].sum() < t
        prev = cur
    # one key every query points at: its block takes the mass, and the selection is that block plus the diagonal
    k2 = 0.01 * r.standard_normal((n, 8))
    q2 = np.tile(np.array([3.0] + [0.0] * 7), (n, 1))
    for j in range(16, 32):                                             # every key of block 1, so that each sampled line meets one
        k2[j] = np.array([8.0] + [0.0] * 7)
    sel = O.xa_select(q2, k2, stride, 0.9, blk)
    for bi in range(2, nb):
        assert set(np.nonzero(sel[bi])[0]) == {1, bi}
