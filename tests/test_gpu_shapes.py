"""Seeded sweep over odd shapes through the C ABI against the oracle: group sizes that do not fill an MFMA
column block, windows shorter than a key tile, no sinks, sinks longer than the prompt, chunk boundaries off
every tile edge, both head sizes, both launch shapes of the prefill kernel, token-exact and block-granular masks,
ragged batches with mixed modes.
Every case is small enough for the explicit-mask oracle; the draw is fixed by the case number."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as O
from tests import helpers as H
from tests.test_gpu_parity import Layer, FA, SA

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    from paper_2604_07394_amd import binding
    return binding


@pytest.fixture(scope="module")
def ctx(F):
    c = F.flux_create(0, 0)
    yield c
    F.flux_destroy(c)


HEADS = [(1, 1), (2, 1), (3, 1), (4, 2), (5, 1), (6, 2), (7, 1), (8, 8), (16, 1), (20, 2), (12, 4)]


@pytest.mark.parametrize("case", range(24))
def test_odd_shapes(F, ctx, case):
    rng = np.random.default_rng(1000 + case)
    hq, hkv = HEADS[case % len(HEADS)]
    d = 64 if case % 3 == 0 else 128
    batch = int(rng.integers(1, 5))
    lens = [int(x) for x in rng.integers(1, 700, size=batch)]
    n_sink = int(rng.choice([0, 1, 5, 16, 70, 900]))
    window = int(rng.choice([1, 7, 64, 130, 300]))
    block = int(rng.choice([1, 1, 16, 64]))
    modes = [int(x) for x in rng.integers(0, 2, size=batch)]
    # (head dimension 128: a cache as large as the bound that chooses the launch shape of long prompts, see below)
    lay = Layer(F, ctx, 2000 + case, batch, hq, hkv, d, 720 if d == 64 else 32768, n_sink, window, scales=bool(case % 2), block=block)
    # prefill in two chunks with a cut anywhere (possibly empty for some sequences)
    first = [int(rng.integers(0, n + 1)) for n in lens]
    what = f"case {case}: heads {hq}/{hkv} D {d} lens {lens} cut {first} sinks {n_sink} window {window} block {block} modes {modes}"
    for part in (first, [n - f for n, f in zip(lens, first)]):
        if sum(part) == 0:
            continue
        qb, kb, vb = lay.new_tokens(part)
        lay.append(kb, vb, part)
        got, ref = lay.prefill(qb, part, modes)
        H.assert_close(got, ref, what + " prefill")
        if d == 128:
            # the launch shape of long prompts (256 query rows and eight waves per workgroup), chosen by the host's
            # bound on the prompt length, which may be larger than needed: the same results bit for bit
            wide, _ = lay.prefill(qb, part, modes, max_q_len=32768, want_ref=False)
            assert np.array_equal(wide, got), what + " prefill, launch shape of long prompts"
    for step in range(2):
        qb, kb, vb = lay.new_tokens([1] * batch)
        lay.append(kb, vb, [1] * batch)
        got, ref = lay.decode(qb.reshape(batch, hq, d), modes)
        H.assert_close(got, ref, what + f" decode {step}")
    assert F.flux_last_device_status(ctx) == 0
