"""Pins for the oracle's index and prefix match: a dict model under random op sequences, the
capacity rule, and match length against a brute-force token comparison."""
import numpy as np
import pytest

import oracle
from workloads import make_workload, make_tokens

NO = np.uint64(0xFFFFFFFFFFFFFFFF)


def test_random_op_sequences_against_a_dict():
    rng = np.random.default_rng(0)
    for n_slots in (8, 16, 64):
        ix = oracle.Index(n_slots)
        model = {}
        ins = upd = full = ev = miss = 0
        universe = rng.integers(1, 2**63, size=3 * n_slots, dtype=np.uint64)
        for step in range(300):
            op = rng.integers(0, 3)
            k = rng.choice(universe, size=rng.integers(0, 9), replace=False)
            if op == 0:
                v = rng.integers(0, 2**40, size=len(k), dtype=np.uint64)
                ix.insert(k, v)
                for kk, vv in zip(k, v):
                    if int(kk) in model:
                        model[int(kk)] = int(vv); upd += 1
                    elif len(model) >= n_slots:
                        full += 1
                    else:
                        model[int(kk)] = int(vv); ins += 1
            elif op == 1:
                got = ix.evict(k)
                for kk, g in zip(k, got):
                    if int(kk) in model:
                        assert int(g) == model.pop(int(kk)); ev += 1
                    else:
                        assert g == NO; miss += 1
            else:
                vals, mlen = ix.match(k, [0, len(k)])
                want = [model.get(int(kk), int(NO)) for kk in k]
                assert [int(x) for x in vals] == want
                fm = next((j for j, w in enumerate(want) if w == int(NO)), len(k))
                assert int(mlen[0]) == fm
            assert ix.count() == len(model)
        dk, dv = ix.dump()
        assert [int(x) for x in dk] == sorted(model)
        assert [int(x) for x in dv] == [model[k] for k in sorted(model)]
        assert list(ix.counters_insert) == [ins, upd, full]
        assert list(ix.counters_evict) == [ev, miss]


def test_capacity_and_reserved_keys():
    ix = oracle.Index(8)
    keys = np.arange(1, 13, dtype=np.uint64)
    ix.insert(keys, keys * np.uint64(10))
    assert list(ix.counters_insert) == [8, 0, 4] and ix.count() == 8
    ix.insert(keys[:8], keys[:8])                       # all present: upsert works when full
    assert list(ix.counters_insert) == [8, 8, 4]
    got = ix.evict(keys[:2])
    assert list(got) == [1, 2]
    ix.insert(keys[10:12], keys[10:12])                 # room again after the eviction
    assert list(ix.counters_insert) == [10, 8, 4] and ix.count() == 8
    ix.insert(np.array([0, NO], dtype=np.uint64), np.array([5, 5], dtype=np.uint64))
    assert list(ix.counters_insert) == [10, 8, 6]
    assert list(ix.evict(np.array([0, NO], dtype=np.uint64))) == [NO, NO]
    v, m = ix.match(np.array([0, NO, 3], dtype=np.uint64), [0, 3])
    assert list(v) == [NO, NO, 3] and m[0] == 0


def test_duplicates_in_one_insert_batch():
    ix = oracle.Index(64)
    k = np.array([5, 5, 7, 5], dtype=np.uint64)
    ix.insert(k, np.array([1, 1, 2, 1], dtype=np.uint64))
    assert list(ix.counters_insert) == [2, 2, 0] and ix.count() == 2
    ix.insert(k, np.array([1, 1, 2, 1], dtype=np.uint64))
    assert list(ix.counters_insert) == [2, 6, 0]


def _brute_match(wl, indexed_requests):
    """match_len[r] = max over indexed q of min(floor(LCP(r,q)/B), n_q, n_r), by comparing tokens."""
    B = wl.block_size
    out = np.zeros(wl.n_req, dtype=np.int32)
    for r in range(wl.n_req):
        tr = wl.tokens[wl.tok_off[r]:wl.tok_off[r + 1]]
        n_r = len(tr) // B
        best = 0
        for q in indexed_requests:
            tq = wl.tokens[wl.tok_off[q]:wl.tok_off[q + 1]]
            m = min(len(tr), len(tq))
            neq = np.flatnonzero(tr[:m] != tq[:m])
            lcp = int(neq[0]) if len(neq) else m
            best = max(best, min(lcp // B, len(tq) // B, n_r))
        out[r] = best
    return out


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_match_length_equals_brute_force_token_comparison(cfg):
    wl = make_workload(cfg, "small")
    h = oracle.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, 0)
    indexed = list(range(0, wl.n_req, 2))               # every other request is cached
    ix = oracle.Index(1 << 16)
    for q in indexed:
        hq = h[wl.blk_off[q]:wl.blk_off[q + 1]]
        ix.insert(hq, np.arange(len(hq), dtype=np.uint64) + np.uint64(q << 20))
    vals, mlen = ix.match(h, wl.blk_off)
    assert np.array_equal(mlen, _brute_match(wl, indexed))
    for q in indexed:                                   # fully cached request: all present
        assert mlen[q] == wl.blk_off[q + 1] - wl.blk_off[q]
        assert not np.any(vals[wl.blk_off[q]:wl.blk_off[q + 1]] == NO)


def test_match_monotonicity_and_first_miss():
    tok, tok_off, blk_off = make_tokens(2, 0, 8)
    h = oracle.block_hash(tok, tok_off, blk_off, 16, 0)
    ix = oracle.Index(1 << 14)
    v, m = ix.match(h, blk_off)
    assert np.all(m == 0) and np.all(v == NO)           # empty index
    ix.insert(h, np.arange(len(h), dtype=np.uint64))
    v, m = ix.match(h, blk_off)
    assert np.array_equal(m, np.diff(blk_off).astype(np.int32))
    # evicting block k of request 3 caps its match at k, but later blocks still report values
    r, k = 3, 200                                       # block 200 is in the unshared tail
    key = h[blk_off[r] + k]
    ix.evict([key])
    v2, m2 = ix.match(h, blk_off)
    assert m2[r] == k and v2[blk_off[r] + k] == NO and v2[blk_off[r] + k + 1] != NO
    assert np.all(np.delete(m2, r) == np.delete(m, r))
    # re-inserting never lowers a match
    ix.insert([key], [123])
    v3, m3 = ix.match(h, blk_off)
    assert np.all(m3 >= m2) and v3[blk_off[r] + k] == 123
    # a request with zero blocks matches zero
    v4, m4 = ix.match(h[:0], [0, 0])
    assert list(m4) == [0]
