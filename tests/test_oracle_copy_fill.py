"""Pins for the oracle's copies of partly filled blocks: numpy slicing as the plain definition, the
clamping and rounding rule, untouched remainders on both sides, and whole segments as the special
case that must equal the plain copy."""
import numpy as np
import pytest

import oracle
from workloads import Geometry


def _pool(g, seed=0):
    return np.random.default_rng(seed).integers(0, 256, size=g.pool_bytes, dtype=np.uint8)


@pytest.mark.parametrize("n_seg,seg_bytes,n_pages", [(1, 4096, 40), (6, 256, 33), (61, 1152, 20), (3, 16, 9)])
def test_gather_fill_equals_slicing(n_seg, seg_bytes, n_pages):
    g = Geometry(n_seg, seg_bytes, n_pages)
    pool = _pool(g)
    rng = np.random.default_rng(7)
    n = 30
    ids = rng.integers(0, n_pages, size=n).astype(np.int32)
    fill = (rng.integers(0, seg_bytes // 16 + 1, size=n) * 16).astype(np.int32)
    fill[0], fill[1] = 0, seg_bytes                                     # nothing, and everything
    st = np.full(n * g.blk_bytes, 0xEE, dtype=np.uint8)
    assert oracle.kv_gather_fill(pool, g.as_tuple(), ids, None, fill, st, g.blk_bytes) == 0
    planes = pool.reshape(n_seg, n_pages, seg_bytes)
    want = np.full((n, n_seg, seg_bytes), 0xEE, dtype=np.uint8)
    for i in range(n):
        want[i, :, :fill[i]] = planes[:, ids[i], :fill[i]]              # the first fill bytes of every segment
    assert np.array_equal(st, want.reshape(-1))


def test_fill_is_clamped_and_rounded_down_to_16():
    g = Geometry(2, 256, 8)
    pool = _pool(g, 1)
    ids = np.arange(6, dtype=np.int32)
    fill = np.array([-5, 15, 16, 31, 250, 100000], dtype=np.int32)
    moved = [0, 0, 16, 16, 240, 256]
    st = np.full(6 * g.blk_bytes, 0x11, dtype=np.uint8)
    oracle.kv_gather_fill(pool, g.as_tuple(), ids, None, fill, st, g.blk_bytes)
    got = st.reshape(6, 2, 256)
    planes = pool.reshape(2, 8, 256)
    for i, m in enumerate(moved):
        assert np.array_equal(got[i, :, :m], planes[:, i, :m]) and np.all(got[i, :, m:] == 0x11)


def test_scatter_fill_leaves_the_rest_of_the_page_alone_and_inverts_the_gather():
    g = Geometry(4, 512, 32)
    pool = _pool(g, 2)
    keep = pool.copy()
    rng = np.random.default_rng(3)
    ids = rng.permutation(32)[:20].astype(np.int32)
    slots = rng.permutation(25)[:20].astype(np.int32)
    fill = (rng.integers(0, 33, size=20) * 16).astype(np.int32)
    stride = g.blk_bytes + 32
    st = np.full(25 * stride, 0x22, dtype=np.uint8)
    oracle.kv_gather_fill(pool, g.as_tuple(), ids, slots, fill, st, stride)
    assert np.array_equal(pool, keep)
    planes = pool.reshape(4, 32, 512)
    for i in range(20):
        planes[:, ids[i], :fill[i]] = 0xA5                              # wipe exactly what was staged
    oracle.kv_scatter_fill(pool, g.as_tuple(), ids, slots, fill, st, stride)
    assert np.array_equal(pool, keep)                                   # scatter(gather) = identity
    st2 = st.reshape(25, stride)
    assert np.all(st2[:, g.blk_bytes:] == 0x22)                         # padding untouched
    # a scatter writes the first fill bytes of each segment and nothing else of the page
    pool[:] = 0
    oracle.kv_scatter_fill(pool, g.as_tuple(), ids, slots, fill, st, stride)
    kp = keep.reshape(4, 32, 512)
    for i in range(20):
        assert np.array_equal(planes[:, ids[i], :fill[i]], kp[:, ids[i], :fill[i]])
        assert np.all(planes[:, ids[i], fill[i]:] == 0)
    assert np.all(planes[:, np.setdiff1d(np.arange(32), ids)] == 0)


def test_whole_segments_and_null_fill_equal_the_plain_copy_and_holes_are_skipped():
    g = Geometry(3, 128, 10)
    pool = _pool(g, 4)
    ids = np.array([3, -1, 9, 10, 0, 2**31 - 1], dtype=np.int32)
    a = np.full(6 * g.blk_bytes, 0x33, dtype=np.uint8)
    b, c = a.copy(), a.copy()
    assert oracle.kv_gather(pool, g.as_tuple(), ids, None, a, g.blk_bytes) == 2
    assert oracle.kv_gather_fill(pool, g.as_tuple(), ids, None, None, b, g.blk_bytes) == 2
    assert oracle.kv_gather_fill(pool, g.as_tuple(), ids, None, np.full(6, 128, np.int32), c, g.blk_bytes) == 2
    assert np.array_equal(a, b) and np.array_equal(a, c)
    assert oracle.kv_gather_fill(pool, g.as_tuple(), ids[:0], None, ids[:0], a, g.blk_bytes) == 0
