"""Pins for the oracle's index rebuild: the copy answers every question the source answers
(contents, usage, victims, matches), the source is untouched, and a smaller destination keeps
exactly `capacity` of the keys."""
import numpy as np

import oracle


def _filled(rng, n_slots, n_keys):
    ix = oracle.Index(n_slots)
    k = rng.choice(np.arange(1, 10 * n_keys, dtype=np.uint64), size=n_keys, replace=False)
    v = rng.integers(0, 1 << 40, size=n_keys, dtype=np.uint64)
    ix.insert(k, v)
    ix.touch(k[: n_keys // 2], 5)
    ix.touch(k[: n_keys // 4], 9)
    ix.evict(k[::7])
    return ix, k, v


def test_copy_equals_source_in_every_observable():
    rng = np.random.default_rng(1)
    src, k, v = _filled(rng, 1024, 600)
    before = (src.dump(), src.select_victims(2, 8), src.count())
    dst = oracle.Index(1024)
    dst.insert(np.array([77777], dtype=np.uint64), np.array([1], dtype=np.uint64))   # wiped by the rebuild
    c = src.rebuild_into(dst)
    assert list(c) == [src.count(), 0, 0]
    for a, b in zip(dst.dump(), before[0]):
        assert np.array_equal(a, b)
    for protect, epoch in ((1, 1), (2, 8), (2, 100), (3, 6), (255, 1 << 20)):
        for a, b in zip(dst.select_victims(protect, epoch), src.select_victims(protect, epoch)):
            assert np.array_equal(a, b)
    # the source still answers as before
    after = (src.dump(), src.select_victims(2, 8), src.count())
    assert after[2] == before[2]
    for x, y in zip(after[0] + after[1], before[0] + before[1]):
        assert np.array_equal(x, y)
    # a dict written out by hand agrees
    want = {int(a): int(b) for a, b in zip(k, v)}
    for a in k[::7]:
        del want[int(a)]
    dk, dv = dst.dump()
    assert {int(a): int(b) for a, b in zip(dk, dv)} == want
    # lookups through the copy
    blk_off = np.array([0, len(k)], dtype=np.int64)
    va, ma = src.match(k, blk_off)
    vb, mb = dst.match(k, blk_off)
    assert np.array_equal(va, vb) and np.array_equal(ma, mb) and int(ma[0]) == 0   # k[0] was evicted


def test_resize_up_and_down():
    rng = np.random.default_rng(2)
    src, k, v = _filled(rng, 512, 400)
    live = src.count()
    big = oracle.Index(4096)
    assert list(src.rebuild_into(big)) == [live, 0, 0] and big.count() == live
    small = oracle.Index(64)
    c = src.rebuild_into(small)
    assert list(c) == [64, 0, live - 64] and small.count() == 64
    sk, sv = small.dump()
    full = dict(zip(*[x.tolist() for x in src.dump()]))
    assert all(full[a] == b for a, b in zip(sk.tolist(), sv.tolist()))            # a subset, values kept
    empty = oracle.Index(64)
    assert list(empty.rebuild_into(small)) == [0, 0, 0] and small.count() == 0
