"""The C ABI without a GPU: the library loads, exports every symbol include/flux.h declares, and
rejects bad arguments on the host before anything could be launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def F():
    lib = os.path.join(ROOT, "paper_2604_07394_amd", "lib", "libflux.so")
    if not os.path.exists(lib):
        from paper_2604_07394_amd import build
        build.build_all()
    from paper_2604_07394_amd import binding
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flux.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flux_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(F):
    names = declared_symbols()
    assert set(names) == set(F.EXPORTS)
    lib = C.CDLL(F.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_texts(F):
    assert F.flux_strerror(0) == "ok"
    assert "invalid" in F.flux_strerror(F.FLUX_EINVAL)
    assert "capacity" in F.flux_strerror(F.FLUX_ECAPACITY)
    assert "workspace" in F.flux_strerror(F.FLUX_EWORKSPACE)


def test_workspace_needed_is_host_arithmetic(F):
    cfg = F.attn_cfg(32, 8, 128, 128, 4096)
    small = F.flux_workspace_needed(cfg, 1, 4096)
    big = F.flux_workspace_needed(cfg, 8, 131072 + 128)
    assert 0 < small < big < (1 << 30)
    assert F.flux_workspace_needed(F.attn_cfg(32, 5, 128, 0, 1), 1, 100) == 0       # bad head ratio
    assert F.flux_workspace_needed(cfg, 0, 100) == 0
    # split-K partials: at most 1024 + (sequence, KV head) pairs units of group x (D + 2) floats whatever the
    # lengths, fewer when even the longest list has few 256-key chunks
    fixed = F.flux_workspace_needed(cfg, 1, 1) - 8 * 1 * 4 * 130 * 4
    assert big - fixed == (1024 + 8 * 8) * 4 * 130 * 4
    assert F.flux_workspace_needed(cfg, 8, 1 << 22) == big              # no growth with the length
    assert small - fixed == 8 * 16 * 4 * 130 * 4                         # 8 pairs x 16 chunks of 256 keys


@pytest.fixture()
def nodev(F):
    ctx = F.flux_create(-1, 0)          # a context without a device: validation only
    yield ctx
    F.flux_destroy(ctx)


def cache_struct(F, **kw):
    d = dict(k=4096, v=8192, stride_b=128 * 64 * 2, stride_h=128 * 64, stride_t=128, kv_len=256, batch=1, capacity=64)
    d.update(kw)
    return F.FluxKVCache(d["k"], d["v"], d["stride_b"], d["stride_h"], d["stride_t"], d["kv_len"], d["batch"], d["capacity"])


def rc_of(F, fn, *a):
    try:
        fn(*a)
    except F.FluxError as e:
        return e.code
    return 0


def test_attention_argument_validation(F, nodev):
    good = F.attn_cfg(8, 2, 128, 4, 16)
    kc = cache_struct(F)
    args = lambda cfg=good, cache=kc, q=4096, mq=8, mk=32, mode=512, out=1024: (nodev, cfg, q, 768, mq, mk, cache, mode, out)
    # a fully valid call gets past validation and then reports the missing device
    assert rc_of(F, F.flux_attn_prefill, *args()) == F.FLUX_EHIP
    assert rc_of(F, F.flux_attn_prefill, *args(cfg=F.attn_cfg(8, 3, 128, 4, 16))) == F.FLUX_EINVAL      # Hq % Hkv
    assert rc_of(F, F.flux_attn_prefill, *args(cfg=F.attn_cfg(8, 2, 96, 4, 16))) == F.FLUX_EINVAL       # head_dim
    assert rc_of(F, F.flux_attn_prefill, *args(cfg=F.attn_cfg(8, 2, 128, -1, 16))) == F.FLUX_EINVAL     # sinks
    assert rc_of(F, F.flux_attn_prefill, *args(cfg=F.attn_cfg(8, 2, 128, 4, 0))) == F.FLUX_EINVAL       # window
    assert rc_of(F, F.flux_attn_prefill, *args(cfg=F.attn_cfg(8, 2, 128, 4, 16, out_dtype=3))) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_prefill, *args(q=None)) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_prefill, *args(q=4100)) == F.FLUX_EINVAL                                # alignment
    assert rc_of(F, F.flux_attn_prefill, *args(mode=None)) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_prefill, *args(mq=40, mk=32)) == F.FLUX_EINVAL                          # more queries than keys
    assert rc_of(F, F.flux_attn_prefill, *args(mk=65)) == F.FLUX_ECAPACITY
    assert rc_of(F, F.flux_attn_prefill, *args(cache=cache_struct(F, stride_t=64))) == F.FLUX_EINVAL    # stride < D
    assert rc_of(F, F.flux_attn_prefill, *args(cache=cache_struct(F, stride_t=132))) == F.FLUX_EINVAL   # 16-byte rule
    assert rc_of(F, F.flux_attn_prefill, *args(cache=cache_struct(F, stride_t=(1 << 22) + 8))) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_prefill, *args(cache=cache_struct(F, k=None))) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_prefill, None, good, 4096, 768, 8, 32, kc, 512, 1024) == F.FLUX_EINVAL  # no context

    dargs = lambda cfg=good, cache=kc, mk=32: (nodev, cfg, 4096, mk, cache, 512, 1024)
    assert rc_of(F, F.flux_attn_decode, *dargs()) == F.FLUX_EHIP
    assert rc_of(F, F.flux_attn_decode, *dargs(mk=-1)) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_decode, *dargs(mk=100)) == F.FLUX_ECAPACITY
    assert rc_of(F, F.flux_attn_decode, *dargs(cfg=F.attn_cfg(8, 0, 128, 4, 16))) == F.FLUX_EINVAL

    # the fused decode step: the arguments of flux_attn_decode plus the appended rows
    fargs = lambda cfg=good, cache=kc, mk=32, kn=8192, vn=12288: (nodev, cfg, 4096, kn, vn, mk, cache, 512, 1024)
    assert rc_of(F, F.flux_attn_decode_append, *fargs()) == F.FLUX_EHIP
    assert rc_of(F, F.flux_attn_decode_append, *fargs(mk=0)) == F.FLUX_EINVAL      # the appended row is always attended
    assert rc_of(F, F.flux_attn_decode_append, *fargs(mk=100)) == F.FLUX_ECAPACITY
    assert rc_of(F, F.flux_attn_decode_append, *fargs(kn=None)) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_decode_append, *fargs(vn=12296)) == F.FLUX_EINVAL  # 16-byte alignment
    assert rc_of(F, F.flux_attn_decode_append, *fargs(cfg=F.attn_cfg(8, 3, 128, 4, 16))) == F.FLUX_EINVAL


def test_append_and_router_argument_validation(F, nodev):
    kc = cache_struct(F)
    ok = (nodev, kc, 2, 128, 4096, 8192, 256, 10, 10)
    assert rc_of(F, F.flux_kv_append, *ok) == F.FLUX_EHIP
    assert rc_of(F, F.flux_kv_append, nodev, kc, 2, 128, 4096, 8192, 256, 100, 65) == F.FLUX_ECAPACITY
    assert rc_of(F, F.flux_kv_append, nodev, kc, 2, 128, 4096, 8192, 256, 5, 6) == F.FLUX_EINVAL        # max_new > total
    assert rc_of(F, F.flux_kv_append, nodev, kc, 2, 100, 4096, 8192, 256, 5, 5) == F.FLUX_EINVAL        # head_dim
    assert rc_of(F, F.flux_kv_append, nodev, kc, 2, 128, None, 8192, 256, 5, 5) == F.FLUX_EINVAL

    r_ok = (nodev, 4096, 256, 2, 4096, 100, 8192, None, 16384, None, 256, 512, None)
    assert rc_of(F, F.flux_router, *r_ok) == F.FLUX_EHIP
    bad_hidden = list(r_ok); bad_hidden[4] = 4100
    assert rc_of(F, F.flux_router, *bad_hidden) == F.FLUX_EINVAL
    bad_inner = list(r_ok); bad_inner[10] = 0
    assert rc_of(F, F.flux_router, *bad_inner) == F.FLUX_EINVAL
    bad_pool = list(r_ok); bad_pool[5] = -1
    assert rc_of(F, F.flux_router, *bad_pool) == F.FLUX_EINVAL
    no_out = list(r_ok); no_out[11] = None
    assert rc_of(F, F.flux_router, *no_out) == F.FLUX_EINVAL
    huge = list(r_ok); huge[3] = 4096
    assert rc_of(F, F.flux_router, *huge) == F.FLUX_EWORKSPACE


def test_ring_argument_validation(F, nodev):
    good = F.attn_cfg(8, 2, 128, 4, 16)
    ring = cache_struct(F, capacity=20)                      # exactly n_sink + window rows
    full = cache_struct(F, capacity=64)
    ok = (nodev, ring, 2, 128, 4, 16, 4096, 8192, 256, 100, 100)
    assert rc_of(F, F.flux_kv_append_ring, *ok) == F.FLUX_EHIP                   # any number of rows may be appended
    assert rc_of(F, F.flux_kv_append_ring, nodev, ring, 2, 128, 4, 17, 4096, 8192, 256, 5, 5) == F.FLUX_ECAPACITY
    assert rc_of(F, F.flux_kv_append_ring, nodev, ring, 2, 128, -1, 16, 4096, 8192, 256, 5, 5) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_kv_append_ring, nodev, ring, 2, 128, 4, 0, 4096, 8192, 256, 5, 5) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_kv_append_ring, nodev, ring, 2, 128, 4, 16, None, 8192, 256, 5, 5) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_kv_append_ring, nodev, ring, 2, 96, 4, 16, 4096, 8192, 256, 5, 5) == F.FLUX_EINVAL

    assert rc_of(F, F.flux_kv_compact_ring, nodev, full, ring, 2, 128, 4, 16) == F.FLUX_EHIP
    assert rc_of(F, F.flux_kv_compact_ring, nodev, full, ring, 2, 128, 5, 16) == F.FLUX_ECAPACITY
    assert rc_of(F, F.flux_kv_compact_ring, nodev, full, cache_struct(F, capacity=20, batch=2), 2, 128, 4, 16) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_kv_compact_ring, nodev, cache_struct(F, k=None), ring, 2, 128, 4, 16) == F.FLUX_EINVAL

    assert rc_of(F, F.flux_attn_decode_ring, nodev, good, 4096, ring, 1024) == F.FLUX_EHIP
    assert rc_of(F, F.flux_attn_decode_ring, nodev, F.attn_cfg(8, 2, 128, 4, 17), 4096, ring, 1024) == F.FLUX_ECAPACITY
    assert rc_of(F, F.flux_attn_decode_ring, nodev, good, None, ring, 1024) == F.FLUX_EINVAL
    assert rc_of(F, F.flux_attn_decode_ring, nodev, good, 4100, ring, 1024) == F.FLUX_EINVAL


def test_block_size_validation(F, nodev):
    kc = cache_struct(F)
    call = lambda blk: rc_of(F, F.flux_attn_decode, nodev, F.attn_cfg(8, 2, 128, 4, 16, 0.0, 0, blk), 4096, 32, kc, 512, 1024)
    assert call(0) == F.FLUX_EHIP and call(1) == F.FLUX_EHIP and call(64) == F.FLUX_EHIP
    assert call(48) == F.FLUX_EINVAL and call(-64) == F.FLUX_EINVAL and call(1 << 17) == F.FLUX_EINVAL


def test_window_and_sinks_near_the_largest_int_do_not_wrap(F, nodev):
    """'SA sees everything' (Eq. 2 degenerating to Eq. 1) is naturally written as window = INT32_MAX.  With a
    block size above one the window is rounded up to whole blocks; that rounding must not wrap: a ring cache
    can never hold such a window (FLUX_ECAPACITY, not a negative row count that passes), and the plain calls
    stay valid."""
    big = (1 << 31) - 1
    kc = cache_struct(F)
    for blk in (0, 64, 65536):
        assert rc_of(F, F.flux_attn_decode, nodev, F.attn_cfg(8, 2, 128, 4, big, 0.0, 0, blk), 4096, 32, kc, 512, 1024) == F.FLUX_EHIP
        assert rc_of(F, F.flux_attn_decode, nodev, F.attn_cfg(8, 2, 128, big, 16, 0.0, 0, blk), 4096, 32, kc, 512, 1024) == F.FLUX_EHIP
        assert rc_of(F, F.flux_attn_decode_ring, nodev, F.attn_cfg(8, 2, 128, 4, big, 0.0, 0, blk), 4096, kc, 1024) == F.FLUX_ECAPACITY
        assert rc_of(F, F.flux_attn_decode_ring, nodev, F.attn_cfg(8, 2, 128, big, 16, 0.0, 0, blk), 4096, kc, 1024) == F.FLUX_ECAPACITY
        assert F.flux_workspace_needed(F.attn_cfg(8, 2, 128, big, big, 0.0, 0, blk), 2, 4096) > 0


def test_blocksparse_argument_validation(F, nodev):
    good = F.attn_cfg(8, 2, 128, 0, 1)
    kc = cache_struct(F)
    call = lambda **kw: rc_of(F, F.flux_attn_prefill_blocksparse, nodev, kw.get("cfg", good), 4096, 768, kw.get("mq", 32),
                              kw.get("mk", 64), kc, 512, kw.get("mask", 2048), kw.get("heads", 1), kw.get("nq", 2),
                              kw.get("nk", 1), 1024)
    assert call() == F.FLUX_EHIP                                   # 32 queries somewhere in a 64-position cache
    assert call(nq=1) == F.FLUX_EHIP                               # (whether they span two blocks is seen on the device)
    assert call(mq=64, mk=64, nq=0) == F.FLUX_EINVAL
    assert call(mask=None) == F.FLUX_EINVAL
    assert call(heads=3) == F.FLUX_EINVAL                          # one matrix for all heads, or one per query head
    assert call(heads=8) == F.FLUX_EHIP
    assert call(nk=0) == F.FLUX_EINVAL
    assert call(mq=64, mk=64, nq=1, nk=1) == F.FLUX_EHIP           # a whole prompt: the queries start on a block boundary
    assert call(mq=64, mk=64, nq=1, nk=1) == F.FLUX_EHIP
    assert call(mk=64, nk=1) == F.FLUX_EHIP
    assert call(mk=65, nk=1) == F.FLUX_ECAPACITY                   # beyond the cache capacity of the fixture
    assert call(cfg=F.attn_cfg(8, 3, 128, 0, 1)) == F.FLUX_EINVAL


def test_xa_select_argument_validation(F, nodev):
    good = F.attn_cfg(8, 2, 128, 0, 1)
    kc = cache_struct(F)
    call = lambda **kw: rc_of(F, F.flux_xa_select, nodev, kw.get("cfg", good), 4096, 768, 64, 64, kc, kw.get("stride", 16),
                              kw.get("thr", 0.9), kw.get("mask", 2048), kw.get("nq", 1), kw.get("nk", 1))
    assert call() == F.FLUX_EHIP
    assert call(stride=8) == F.FLUX_EINVAL                          # the stride of Table 3 is the one built
    assert call(thr=0.0) == F.FLUX_EINVAL and call(thr=1.5) == F.FLUX_EINVAL and call(thr=float("nan")) == F.FLUX_EINVAL
    assert call(thr=1.0) == F.FLUX_EHIP
    assert call(mask=None) == F.FLUX_EINVAL
    assert call(nq=0) == F.FLUX_EINVAL and call(nk=0) == F.FLUX_EINVAL
    assert call(nk=4097) == F.FLUX_EINVAL                           # more key blocks than the kernel's LDS holds
    assert call(cfg=F.attn_cfg(8, 2, 96, 0, 1)) == F.FLUX_EINVAL
