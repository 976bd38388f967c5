"""Pins for the oracle's paged-KV gather/scatter: numpy fancy indexing as the library special
case, round-trip identities, untouched neighbours and the edge cases."""
import numpy as np
import pytest

import oracle
from workloads import Geometry


def _pool(g, seed=0):
    return np.random.default_rng(seed).integers(0, 256, size=g.pool_bytes, dtype=np.uint8)


@pytest.mark.parametrize("n_seg,seg_bytes,n_pages", [(1, 4096, 40), (6, 256, 33), (61, 1152, 20),
                                                      (3, 16, 9), (1, 16, 1)])
def test_gather_equals_fancy_indexing(n_seg, seg_bytes, n_pages):
    g = Geometry(n_seg, seg_bytes, n_pages)
    pool = _pool(g)
    rng = np.random.default_rng(1)
    ids = rng.integers(0, n_pages, size=25).astype(np.int32)           # duplicates allowed
    st = np.full(25 * g.blk_bytes, 0xEE, dtype=np.uint8)
    assert oracle.kv_gather(pool, g.as_tuple(), ids, None, st, g.blk_bytes) == 0
    planes = pool.reshape(n_seg, n_pages, seg_bytes)
    want = planes[:, ids, :].transpose(1, 0, 2).reshape(-1)            # block = segments in plane order
    assert np.array_equal(st, want)


def test_round_trips_and_idempotence():
    g = Geometry(5, 512, 64)
    pool = _pool(g, 2)
    keep = pool.copy()
    rng = np.random.default_rng(3)
    ids = rng.permutation(64)[:40].astype(np.int32)
    slots = rng.permutation(50)[:40].astype(np.int32)
    stride = g.blk_bytes + 64                                           # padded staging blocks
    st = np.full(50 * stride, 0x11, dtype=np.uint8)
    oracle.kv_gather(pool, g.as_tuple(), ids, slots, st, stride)
    assert np.array_equal(pool, keep)                                   # gather does not write the pool
    planes = pool.reshape(5, 64, 512)
    planes[:, ids, :] = 0xA5
    oracle.kv_scatter(pool, g.as_tuple(), ids, slots, st, stride)
    assert np.array_equal(pool, keep)                                   # scatter(gather) = identity
    oracle.kv_scatter(pool, g.as_tuple(), ids, slots, st, stride)
    assert np.array_equal(pool, keep)                                   # idempotent
    # padding bytes between staging blocks and unused slots are untouched
    s2 = st.reshape(50, stride)
    assert np.all(s2[:, g.blk_bytes:] == 0x11)
    unused = np.setdiff1d(np.arange(50), slots)
    assert np.all(s2[unused] == 0x11)
    # gather(scatter(staging, pi), pi) = staging for a permutation pi
    st_b = np.random.default_rng(4).integers(0, 256, size=40 * g.blk_bytes, dtype=np.uint8)
    pi = rng.permutation(64)[:40].astype(np.int32)
    oracle.kv_scatter(pool, g.as_tuple(), pi, None, st_b, g.blk_bytes)
    back = np.zeros_like(st_b)
    oracle.kv_gather(pool, g.as_tuple(), pi, None, back, g.blk_bytes)
    assert np.array_equal(back, st_b)
    others = np.setdiff1d(np.arange(64), pi)                            # unnamed pages unchanged
    assert np.array_equal(pool.reshape(5, 64, 512)[:, others], keep.reshape(5, 64, 512)[:, others])


def test_holes_bad_pages_and_empty():
    g = Geometry(2, 64, 10)
    pool = _pool(g, 5)
    keep = pool.copy()
    ids = np.array([3, -1, 10, 7, 2**31 - 1, -7], dtype=np.int32)
    st = np.full(6 * g.blk_bytes, 0x77, dtype=np.uint8)
    assert oracle.kv_gather(pool, g.as_tuple(), ids, None, st, g.blk_bytes) == 2
    s2 = st.reshape(6, -1)
    assert np.all(s2[[1, 2, 4, 5]] == 0x77)
    planes = pool.reshape(2, 10, 64)
    assert np.array_equal(s2[0], planes[:, 3].reshape(-1)) and np.array_equal(s2[3], planes[:, 7].reshape(-1))
    assert oracle.kv_scatter(pool, g.as_tuple(), ids, None, st, g.blk_bytes) == 2
    assert np.array_equal(pool, keep)
    assert oracle.kv_gather(pool, g.as_tuple(), ids[:0], None, st, g.blk_bytes) == 0
    with pytest.raises(ValueError):
        oracle.kv_gather(pool, g.as_tuple(), ids, None, st, g.blk_bytes - 16)   # stride too small


def test_strided_pool_descriptor():
    """A pool whose planes and pages are padded: only seg_bytes of each (plane, page) move."""
    n_seg, n_pages, seg, pstride = 3, 7, 48, 64
    sstride = n_pages * pstride + 32
    pool = np.random.default_rng(6).integers(0, 256, size=n_seg * sstride, dtype=np.uint8)
    geom = (n_seg, sstride, pstride, seg, n_pages)
    ids = np.array([6, 0, 3], dtype=np.int32)
    st = np.zeros(3 * n_seg * seg, dtype=np.uint8)
    oracle.kv_gather(pool, geom, ids, None, st, n_seg * seg)
    for i, p in enumerate(ids):
        for s in range(n_seg):
            a = s * sstride + p * pstride
            assert np.array_equal(st[(i * n_seg + s) * seg:(i * n_seg + s + 1) * seg], pool[a:a + seg])
