"""CPU oracle for the Flux Attention inference hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 NumPy: the definitions written out, no tiling, no online
softmax, no fusion.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this file; the product (the HIP
library and its Python binding) never does, and nothing here imports the
product.

What it follows (paper sections / equations):

* Full Attention, Eq. (1) of Sec. 2.1: ``O_r = Softmax(Q K^T) V`` per head,
  causal, with the usual 1/sqrt(d) scale the paper omits "for clarity".
* Sparse Attention, Eq. (2) of Sec. 2.1: the same softmax over a subset of the
  history.  The subset is the streaming one of Sec. 4.1 / App. C.3: the first
  ``n_sink`` positions plus the ``window`` most recent positions (the query's
  own position counts as the most recent).  App. C.3 sets a block size that is
  "the minimum unit of sparsity": ``block`` > 1 rounds both sets to whole blocks.
* Grouped-query attention: query head ``h`` reads KV head ``h // (Hq // Hkv)``.
* Layer Router, Sec. 3.1: prefix/suffix pooling of the first and last ``pool``
  token rows (App. C.1: 100 + 100) into one mean vector, Context Encoder
  ``Linear -> SiLU``, Router Head ``Linear`` to two logits ``(pi_FA, pi_SA)``,
  hard decision by argmax with ``r_hard = 0`` meaning SA.
* Route once in prefill, reuse the decision for every decode step, Sec. 3.3.
* Sparse-decode residency, Sec. 3.3: a sparse layer keeps only the K/V rows its
  kernel needs (the sinks and the last ``window`` positions); ``RingKVCache``
  stores exactly those and ``decode_step_ring`` attends over what is stored.
* Model Sparsity Ratio, Eq. (3) of Sec. 2.3, at layer granularity.
* Block-sparse attention, Eq. (2) with an arbitrary set of key BLOCKS per query block (the substrate the
  other sparse modes of Sec. 4.1 need): ``attention(..., block_mask=...)``.  A block of 64 positions is
  "the minimum unit of sparsity" (App. C.3).
* XAttention block selection (the XA mode of Sec. 4.1; Table 3: stride 16, threshold 0.9, selection mode
  "Inverse", block 64): ``xa_block_mass`` and ``xa_select``.  The paper names the method ("Block Sparse
  Attention with Antidiagonal Scoring") and its parameters and nothing else, so what is computed here is
  THIS BUILD'S READING of those words, written out in the two functions' docstrings; its agreement with
  the paper's own XA kernels is parity-unpinned (the functions themselves are pinned, see below).

Conventions: ``mode`` 1 = FA, 0 = SA (the paper's ``r_hard``).  All arrays are
float64; bf16 inputs are widened exactly by ``bf16_to_f64`` first.  Positions
are absolute and 0-based; the ``n_q`` queries of a call are the last ``n_q``
positions of the ``n_kv`` cached ones.

Pins (tests/test_oracle_pins.py): closed-form visible counts, window >= length
equals FA, rows of P sum to one, constant-V and constant-K special cases, shift
invariance, brute-force enumeration on 8-token cases, a textbook dense
formula, GQA by head repetition, decode == last prefill row, a hand-computed
router, argmax flip and tie; for the ring residency: stored positions against
their closed form, equality with the full-cache SA decode step by step across
several wrap-arounds, and compaction of a prompt against row-by-row appends;
for the block mask: brute force, the all-true lower triangle equals FA bit for
bit, the sink + window block pattern equals the block-granular SA bit for bit;
for the XA selection: brute-force element sampling against the strided form,
masses that sum to one, closed forms for constant inputs, threshold limits and
monotonicity.  Every function is pinned against the mathematics it states; what
is parity-unpinned is whether ``xa_block_mass`` / ``xa_select`` are the paper's
XA (it defines neither).
"""
from __future__ import annotations

import numpy as np

FA, SA = 1, 0


def bf16_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------- mask

def visible(i, j, mode: int, n_sink: int, window: int, block: int = 1):
    """Whether query position ``i`` attends key position ``j`` (broadcasts).

    FA: every ``j <= i``.  SA: ``j <= i`` and (``j`` is one of the first
    ``n_sink`` positions or ``j`` is among the ``window`` most recent, i.e.
    ``i - j < window``).

    ``block`` > 1 is the block-granular form of App. C.3, where a block of
    ``block`` positions is the minimum unit of sparsity: positions are grouped
    into blocks of ``block``, the sinks are the first ``ceil(n_sink / block)``
    blocks, the window is the ``ceil(window / block)`` most recent blocks (the
    query's own block counts), and a block pair is kept or dropped as a whole,
    except that the causal order still holds inside the diagonal block.
    ``block`` = 1 is the token-exact form above.
    """
    i = np.asarray(i)
    j = np.asarray(j)
    causal = j <= i
    if mode == FA:
        return causal
    bi, bj = i // block, j // block
    sink_blocks = -(-n_sink // block)
    window_blocks = -(-window // block)
    return causal & ((bj < sink_blocks) | (bi - bj < window_blocks))


def mask_matrix(n_q: int, n_kv: int, mode: int, n_sink: int, window: int, block: int = 1) -> np.ndarray:
    """Explicit boolean mask [n_q, n_kv]; row r is query position ``n_kv - n_q + r``."""
    i = (n_kv - n_q + np.arange(n_q))[:, None]
    j = np.arange(n_kv)[None, :]
    return visible(i, j, mode, n_sink, window, block)


BLOCK = 64          # positions per block of a block mask (App. C.3: "the minimum unit of sparsity")


def block_mask_matrix(n_q: int, n_kv: int, block_mask: np.ndarray, block: int = BLOCK) -> np.ndarray:
    """Explicit boolean mask [n_q, n_kv] of a block-sparse pattern.

    Positions are grouped into blocks of ``block``; query position ``i`` (row
    ``r`` is position ``n_kv - n_q + r``) sees key ``j`` iff ``j <= i`` and the
    pair (block of i, block of j) is kept.  ``block_mask[rq, bj]`` is the keep
    flag of key block ``bj`` for the query block ``(n_kv - n_q) // block + rq``
    (row 0 is the block of the call's first query).  The block that holds the
    query's own position is always kept, whatever the flag says: every query
    must see at least itself.
    """
    pos0 = n_kv - n_q
    i = (pos0 + np.arange(n_q))[:, None]
    j = np.arange(n_kv)[None, :]
    bi, bj = i // block, j // block
    bm = np.asarray(block_mask, dtype=bool)
    keep = bm[bi - pos0 // block, bj] | (bi == bj)
    return (j <= i) & keep


# --------------------------------------------------------------------------- attention

def softmax_rows(s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Row-wise softmax of ``s`` restricted to ``mask`` (max-subtracted, fp64)."""
    s = np.where(mask, s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    p = np.where(mask, np.exp(s - m), 0.0)
    return p / p.sum(axis=-1, keepdims=True)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mode: int, n_sink: int, window: int,
              scale: float | None = None, return_probs: bool = False, block: int = 1, block_mask=None,
              mask_block: int = BLOCK):
    """One sequence, one layer, explicit mask matrix.

    q [n_q, Hq, D], k and v [n_kv, Hkv, D] (fp64).  Returns out [n_q, Hq, D]
    (and P [Hq, n_q, n_kv] if asked).  With ``block_mask`` (one keep matrix
    [query blocks, key blocks] for all heads, or [Hq, query blocks, key blocks])
    the visible set is the block-sparse one of ``block_mask_matrix`` with blocks
    of ``mask_block`` positions, and ``mode``, ``n_sink``, ``window``, ``block``
    are not used.
    """
    n_q, hq, d = q.shape
    n_kv, hkv, _ = k.shape
    assert hq % hkv == 0 and n_q <= n_kv
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    mask = mask_matrix(n_q, n_kv, mode, n_sink, window, block) if block_mask is None else None
    out = np.empty((n_q, hq, d), dtype=np.float64)
    probs = np.empty((hq, n_q, n_kv), dtype=np.float64) if return_probs else None
    for h in range(hq):
        kh = k[:, h // g, :]
        vh = v[:, h // g, :]
        s = scale * (q[:, h, :] @ kh.T)
        if block_mask is not None:
            bm = np.asarray(block_mask)
            mask = block_mask_matrix(n_q, n_kv, bm[h] if bm.ndim == 3 else bm, mask_block)
        p = softmax_rows(s, mask)
        out[:, h, :] = p @ vh
        if return_probs:
            probs[h] = p
    return (out, probs) if return_probs else out


def attention_row(q_row: np.ndarray, k: np.ndarray, v: np.ndarray, i: int, mode: int, n_sink: int,
                  window: int, scale: float | None = None, block: int = 1, block_row=None,
                  mask_block: int = BLOCK) -> np.ndarray:
    """One query position ``i`` of one KV-head group, predicate evaluated along the row.

    q_row [G, D] (the G query heads sharing this KV head), k and v [>= i+1, D].
    Returns [G, D].  Same definition as ``attention``; used where the mask
    matrix would not fit.  ``block_row`` (keep flags per key block, the row of a
    block mask that belongs to position ``i``'s query block) selects the
    block-sparse visible set instead of ``mode``.
    """
    d = q_row.shape[-1]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    j = np.arange(i + 1)
    if block_row is None:
        keep = visible(i, j, mode, n_sink, window, block)
    else:
        bj = j // mask_block
        keep = np.asarray(block_row, dtype=bool)[bj] | (bj == i // mask_block)
    kk = k[: i + 1][keep]
    vv = v[: i + 1][keep]
    s = scale * (q_row @ kk.T)                        # [G, n_visible]
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return p @ vv


class KVCache:
    """One layer's contiguous K/V history for a ragged batch (lists of fp64 arrays)."""

    def __init__(self, batch: int, n_kv_heads: int, head_dim: int):
        self.k = [np.zeros((0, n_kv_heads, head_dim)) for _ in range(batch)]
        self.v = [np.zeros((0, n_kv_heads, head_dim)) for _ in range(batch)]

    def append(self, b: int, k_new: np.ndarray, v_new: np.ndarray) -> None:
        self.k[b] = np.concatenate([self.k[b], k_new], axis=0)
        self.v[b] = np.concatenate([self.v[b], v_new], axis=0)

    def length(self, b: int) -> int:
        return self.k[b].shape[0]


def prefill(cache: KVCache, q_list, k_list, v_list, modes, n_sink: int, window: int, scale=None, block: int = 1):
    """Append each sequence's new K/V rows, then attend with its new queries (Sec. 3.3).

    ``modes[b]`` is that sequence's cached decision for this layer.
    """
    outs = []
    for b, (q, k, v) in enumerate(zip(q_list, k_list, v_list)):
        cache.append(b, k, v)
        outs.append(attention(q, cache.k[b], cache.v[b], int(modes[b]), n_sink, window, scale, block=block))
    return outs


def decode_step(cache: KVCache, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, modes,
                n_sink: int, window: int, scale=None, block: int = 1) -> np.ndarray:
    """One autoregressive step: q [B, Hq, D], k_new/v_new [B, Hkv, D] -> out [B, Hq, D]."""
    out = np.empty_like(q)
    for b in range(q.shape[0]):
        cache.append(b, k_new[b][None], v_new[b][None])
        out[b] = attention(q[b][None], cache.k[b], cache.v[b], int(modes[b]), n_sink, window, scale, block=block)[0]
    return out


# --------------------------------------------------------------------------- sparse-decode residency

class RingKVCache:
    """K/V storage of a SPARSE layer in the sparse-decode configuration of Sec. 3.3: per sequence
    ``n_sink + window`` rows and nothing else.

    Row ``p`` for ``p < n_sink`` holds position ``p`` for ever; position ``p >= n_sink`` is written
    to row ``n_sink + (p - n_sink) % window`` and so overwrites the position that left the window.
    ``pos[b][row]`` remembers which position a row holds (-1 = never written).
    """

    def __init__(self, batch: int, n_kv_heads: int, head_dim: int, n_sink: int, window: int):
        self.n_sink, self.window = n_sink, window
        rows = n_sink + window
        self.k = [np.zeros((rows, n_kv_heads, head_dim)) for _ in range(batch)]
        self.v = [np.zeros((rows, n_kv_heads, head_dim)) for _ in range(batch)]
        self.pos = [np.full(rows, -1, dtype=np.int64) for _ in range(batch)]
        self.len = [0] * batch

    def row_of(self, p: int) -> int:
        return p if p < self.n_sink else self.n_sink + (p - self.n_sink) % self.window

    def append(self, b: int, k_new: np.ndarray, v_new: np.ndarray) -> None:
        """Rows one after the other, each at the next position."""
        for r in range(k_new.shape[0]):
            p = self.len[b]
            row = self.row_of(p)
            self.k[b][row] = k_new[r]
            self.v[b][row] = v_new[r]
            self.pos[b][row] = p
            self.len[b] = p + 1

    def length(self, b: int) -> int:
        return self.len[b]

    def stored(self, b: int):
        """(positions, K rows, V rows) of everything stored for sequence b, in position order."""
        rows = np.nonzero(self.pos[b] >= 0)[0]
        rows = rows[np.argsort(self.pos[b][rows])]
        return self.pos[b][rows], self.k[b][rows], self.v[b][rows]


def decode_step_ring(cache: RingKVCache, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, scale=None) -> np.ndarray:
    """One sparse-layer decode step on the minimal cache: append the new row, then the query at the
    newest position attends to EVERY stored row (Eq. 2: they are exactly its visible set).

    q [B, Hq, D], k_new/v_new [B, Hkv, D] -> out [B, Hq, D].
    """
    n_b, hq, d = q.shape
    hkv = k_new.shape[1]
    group = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty_like(q)
    for b in range(n_b):
        cache.append(b, k_new[b][None], v_new[b][None])
        _, kk, vv = cache.stored(b)
        for h in range(hq):
            s = scale * (kk[:, h // group] @ q[b, h])
            pr = np.exp(s - s.max())
            out[b, h] = (pr / pr.sum()) @ vv[:, h // group]
    return out


def compact_to_ring(full: KVCache, ring: RingKVCache) -> None:
    """After the prompt has been prefilled on full K/V (the decision is known only then), keep what
    a sparse layer needs: the same state as appending the prompt to an empty ring row by row."""
    for b in range(len(full.k)):
        ring.append(b, full.k[b], full.v[b])


# --------------------------------------------------------------------------- XAttention block selection

def xa_block_mass(q: np.ndarray, k: np.ndarray, stride: int = 16, block: int = BLOCK, scale: float | None = None,
                  blocks=None):
    """Approximate attention mass of every (query block, key block) pair of ONE head from antidiagonal samples.

    The reading taken of "Block Sparse Attention with Antidiagonal Scoring", stride 16, selection mode
    "Inverse", block 64 (Sec. 4.1, Table 3), for a whole prompt (``n`` queries at positions 0..n-1 over the
    same ``n`` keys; q, k [n, D]):

    1. The scaled score matrix ``scale * q k^T`` is cut into squares of ``stride x stride`` positions.  Of
       square (a, b) (query positions ``stride*a ..``, key positions ``stride*b ..``) only the ANTIDIAGONAL
       is looked at: row offset r against column offset ``stride - 1 - r`` (the query rows taken in inverse
       order against the key columns: the "Inverse" mode), and of those samples only the causal ones
       (key position <= query position).  ``e[a, b]`` is the MEAN of the square's causal samples (the
       "normalisation" App. C.3 mentions: the sampled sum over the number of samples); squares without a
       causal sample (b > a) do not exist.
    2. Each row ``a`` of ``e`` is turned into probabilities over its existing squares b <= a by a softmax:
       the approximate attention of those ``stride`` queries at a granularity of ``stride`` keys.
    3. The mass of the block pair (I, J) is the sum of those probabilities over the squares inside it
       (``block / stride`` rows by ``block / stride`` columns), divided by the number of rows of ``e`` the
       query block has, so that the masses of one query block sum to one.

    Returns ``mass`` [n_qblocks, n_kblocks] (fp64; zero above the block diagonal).  ``n`` need not be a
    multiple of ``block`` or ``stride``: trailing positions form shorter squares and blocks.  ``blocks``
    (query block indices) limits the work to those rows of the result; the others stay zero.
    """
    n, d = q.shape
    assert k.shape == (n, d) and block % stride == 0
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    n_sq = -(-n // stride)
    per = block // stride
    n_blk = -(-n // block)
    mass = np.zeros((n_blk, n_blk))
    r = np.arange(stride)
    for bi in (range(n_blk) if blocks is None else blocks):
        rows_a = range(per * bi, min(per * (bi + 1), n_sq))          # the rows of e this query block has
        for a in rows_a:
            i = stride * a + r                                      # query positions of square row a, one per offset
            j = stride * np.arange(a + 1)[None, :] + (stride - 1 - r)[:, None]   # their antidiagonal partners, per square
            ok = (i[:, None] < n) & (j < n) & (j <= i[:, None])     # inside the prompt and causal
            ic, jc = np.minimum(i, n - 1), np.minimum(j, n - 1)
            smp = scale * np.einsum("rd,rbd->rb", q[ic], k[jc])     # the sampled scores, [offset, square]
            cnt = ok.sum(axis=0)
            e = np.where(cnt > 0, np.where(ok, smp, 0.0).sum(axis=0) / np.maximum(cnt, 1), -np.inf)
            w = np.where(cnt > 0, np.exp(e - e[cnt > 0].max()), 0.0)
            p = w / w.sum()                                         # softmax over the squares of row a
            for bj in range(bi + 1):
                mass[bi, bj] += p[per * bj: per * (bj + 1)].sum() / len(rows_a)
    return mass


def xa_select(q: np.ndarray, k: np.ndarray, stride: int = 16, threshold: float = 0.9, block: int = BLOCK,
              scale: float | None = None, return_mass: bool = False, blocks=None):
    """Key blocks every query block of ONE head keeps (Table 3: threshold 0.9).

    For query block I the key blocks are taken in descending order of ``xa_block_mass`` until the masses
    taken reach ``threshold``; every block whose mass equals that of the last one taken is kept as well (so
    the result does not depend on how equal masses are ordered).  The diagonal block (the queries' own
    positions) is always kept.  Returns a boolean matrix [n_qblocks, n_kblocks] to be used as the
    ``block_mask`` of ``attention`` (only the rows ``blocks`` if given; the others stay empty).
    """
    mass = xa_block_mass(q, k, stride, block, scale, blocks)
    n_blk = mass.shape[0]
    keep = np.zeros((n_blk, n_blk), dtype=bool)
    for bi in (range(n_blk) if blocks is None else blocks):
        m = mass[bi, : bi + 1]
        order = np.argsort(-m, kind="stable")
        csum = np.cumsum(m[order])
        cut = int(np.searchsorted(csum, threshold * csum[-1], side="left"))    # first prefix reaching the threshold
        cut = min(cut, bi)
        keep[bi, : bi + 1] = m >= m[order[cut]]
        keep[bi, bi] = True
    return (keep, mass) if return_mass else keep


# --------------------------------------------------------------------------- router

def pooled_rows(n_rows: int, pool: int) -> np.ndarray:
    """Indices of the token rows that enter the pooling (Sec. 3.1, App. C.1).

    The first ``pool`` and the last ``pool`` rows, each row once; every row if
    the two stretches meet or overlap, or if ``pool`` is 0 (the "Full" setting
    of App. D.2).
    """
    if pool <= 0 or n_rows <= 2 * pool:
        return np.arange(n_rows)
    return np.concatenate([np.arange(pool), np.arange(n_rows - pool, n_rows)])


def silu(x):
    return x / (1.0 + np.exp(-x))


def router(x: np.ndarray, pool: int, w1: np.ndarray, b1, w2: np.ndarray, b2):
    """Layer Router for one sequence.

    x [S, hidden]; w1 [inner, hidden]; w2 [2, inner]; biases or None.
    Returns (logits [2] = (pi_FA, pi_SA), mode) with mode 1 = FA when
    ``pi_FA >= pi_SA`` (argmax, first index wins a tie), else 0 = SA.
    """
    p = x[pooled_rows(x.shape[0], pool)].mean(axis=0)
    h = w1 @ p
    if b1 is not None:
        h = h + b1
    h = silu(h)
    logits = w2 @ h
    if b2 is not None:
        logits = logits + b2
    mode = FA if int(np.argmax(logits)) == 0 else SA
    return logits, mode


def model_sparsity_ratio(modes) -> float:
    """Eq. (3) at layer granularity: the fraction of (layer, sequence) slots routed to SA."""
    modes = np.asarray(modes)
    return float(np.mean(modes == SA))
