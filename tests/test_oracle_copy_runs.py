"""Pins for the oracle's run-wise copies (pools whose segments are not contiguous): numpy
transposition for a token-major pool, agreement with the plain copies when a segment is one run,
identities, holes and bad pages, untouched bytes."""
import numpy as np

import oracle


def _token_major(S, T, run, n_pages):
    """[page][token][segment][run bytes] -> (n_seg, n_run, seg_stride, page_stride, run_stride, run_bytes, n_pages)"""
    return (S, T, run, T * S * run, S * run, run, n_pages)


def test_token_major_pool_is_a_transposition():
    rng = np.random.default_rng(0)
    for S, T, run, n_pages, n in ((4, 16, 64, 20, 13), (61, 64, 1152, 5, 5), (3, 5, 16, 9, 9), (1, 7, 48, 6, 4)):
        pool = rng.integers(0, 256, size=n_pages * T * S * run, dtype=np.uint8)
        ids = rng.permutation(n_pages)[:n].astype(np.int32)
        blk = S * T * run
        staging = np.zeros(n * blk, dtype=np.uint8)
        assert oracle.kv_gather_runs(pool, _token_major(S, T, run, n_pages), ids, None, staging, blk) == 0
        want = pool.reshape(n_pages, T, S, run)[ids].transpose(0, 2, 1, 3)      # [entry][segment][token][bytes]
        assert np.array_equal(staging.reshape(n, S, T, run), want)
        # and back into an empty pool: exactly the gathered pages, nothing else
        pool2 = np.zeros_like(pool)
        assert oracle.kv_scatter_runs(pool2, _token_major(S, T, run, n_pages), ids, None, staging, blk) == 0
        want2 = np.zeros_like(pool).reshape(n_pages, T * S * run)
        want2[ids] = pool.reshape(n_pages, -1)[ids]
        assert np.array_equal(pool2.reshape(n_pages, -1), want2)


def test_one_run_per_segment_is_the_plain_copy():
    rng = np.random.default_rng(1)
    S, seg, n_pages, n = 6, 96, 15, 11
    pool = rng.integers(0, 256, size=S * n_pages * seg, dtype=np.uint8)
    ids = rng.permutation(n_pages)[:n].astype(np.int32)
    slots = rng.permutation(n).astype(np.int32)
    plain = (S, n_pages * seg, seg, seg, n_pages)                     # layer-major: plane s, page p
    runs = (S, 1, n_pages * seg, seg, 0, seg, n_pages)
    a = np.zeros(n * S * seg + 64, dtype=np.uint8)
    b = np.zeros_like(a)
    oracle.kv_gather(pool, plain, ids, slots, a, S * seg)
    oracle.kv_gather_runs(pool, runs, ids, slots, b, S * seg)
    assert np.array_equal(a, b) and a.any()


def test_holes_bad_pages_slots_and_padding():
    rng = np.random.default_rng(2)
    S, T, run, n_pages = 2, 3, 32, 10
    g = _token_major(S, T, run, n_pages)
    pool = rng.integers(1, 256, size=n_pages * T * S * run, dtype=np.uint8)
    ids = np.array([4, -1, 10, 0, 7], dtype=np.int32)
    slots = np.array([2, 0, 1, 4, 3], dtype=np.int32)
    blk, stride = S * T * run, S * T * run + 16
    staging = np.full(5 * stride, 0xEE, dtype=np.uint8)
    assert oracle.kv_gather_runs(pool, g, ids, slots, staging, stride) == 1
    st = staging.reshape(5, stride)
    assert np.all(st[:, blk:] == 0xEE) and np.all(st[0] == 0xEE) and np.all(st[1] == 0xEE)   # slots of the hole / bad page
    for p, q in ((4, 2), (0, 4), (7, 3)):
        assert np.array_equal(st[q, :blk].reshape(S, T, run), pool.reshape(n_pages, T, S, run)[p].transpose(1, 0, 2))
    keep = pool.copy()
    pool[:] = 0
    assert oracle.kv_scatter_runs(pool, g, ids, slots, staging, stride) == 1
    back = pool.reshape(n_pages, -1)
    for p in (4, 0, 7):
        assert np.array_equal(back[p], keep.reshape(n_pages, -1)[p])
    assert not back[[1, 2, 3, 5, 6, 8, 9]].any()
    assert oracle.kv_gather_runs(pool, g, ids[:0], None, staging, stride) == 0
