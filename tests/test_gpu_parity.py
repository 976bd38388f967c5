"""Parity of the HIP library (through its C ABI) with the CPU oracle, bit for bit, on small
inputs that still span several tiles and ragged tails, plus the edge cases."""
import numpy as np
import pytest

import oracle
from backends import HipBackend, HipIndex, OracleBackend, hip_hash_match
from workloads import Geometry, make_tokens, make_workload, flows

pytestmark = pytest.mark.gpu
NO = np.uint64(0xFFFFFFFFFFFFFFFF)


@pytest.fixture(scope="module")
def hip():
    return HipBackend()


# ---- block hash --------------------------------------------------------------------------------
def _ragged(rng, n_req, lo, hi, neg=False):
    lens = rng.integers(lo, hi + 1, size=n_req)
    tok_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(lens, out=tok_off[1:])
    if neg:
        tok = rng.integers(-2**31, 2**31, size=int(tok_off[-1]), dtype=np.int64).astype(np.int32)
    else:
        tok = rng.integers(0, 32000, size=int(tok_off[-1]), dtype=np.int32)
    return tok, tok_off, lens


@pytest.mark.parametrize("B", [16, 32, 64, 1, 5, 17, 100, 128, 1024])
def test_block_hash_ragged(hip, B):
    rng = np.random.default_rng(B)
    # lengths from below one block to many tiles (a tile is 1024 tokens), with ragged tails
    tok, tok_off, lens = _ragged(rng, 37, 0, max(40 * B, 5000), neg=True)
    lens[3] = 0
    lens[5] = B - 1 if B > 1 else 0
    lens[7] = B
    lens[9] = 4096 * 3 + B // 2
    np.cumsum(lens, out=tok_off[1:])
    tok = rng.integers(-2**31, 2**31, size=int(tok_off[-1]), dtype=np.int64).astype(np.int32)
    blk_off = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens // B, out=blk_off[1:])
    for seed in (0, 0xDEADBEEF12345678):
        want = oracle.block_hash(tok, tok_off, blk_off, B, seed)
        got = hip.block_hash(tok, tok_off, blk_off, B, seed)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_block_hash_configs_full_size(hip, cfg):
    wl = make_workload(cfg, "full")
    want = oracle.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, 0)
    got = hip.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, 0)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("B", [16, 32, 64])
def test_block_hash_many_requests(hip, B):
    """In a batch of thousands a request of up to 8 tiles (8192 tokens) is hashed by one wavefront
    (carry in registers, ragged tails), a longer one by the four wavefronts of its workgroup
    (carry through LDS): both sides of that boundary, and long requests of several rounds."""
    rng = np.random.default_rng(7 * B)
    tok, tok_off, lens = _ragged(rng, 5000, 0, 40 * B)
    lens[11] = 9000 + B // 3                      # long requests among the short ones
    lens[12] = 8192                               # exactly 8 tiles
    lens[13] = 8192 + B                           # one block more
    lens[14] = 8192 - 1
    lens[700] = 13 * 1024 + 5 * B + 3             # 14 tiles, the last one ragged
    lens[4999] = 33 * 1024 + B                    # 34 tiles: nine rounds of four wavefronts
    np.cumsum(lens, out=tok_off[1:])
    tok = rng.integers(0, 32000, size=int(tok_off[-1]), dtype=np.int32)
    blk_off = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens // B, out=blk_off[1:])
    want = oracle.block_hash(tok, tok_off, blk_off, B, 3)
    got = hip.block_hash(tok, tok_off, blk_off, B, 3)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("top", [200, 90])
def test_match_many_requests(top):
    """Thousands of short ragged requests in one call: four wavefronts per request (mean above 64
    blocks; requests of up to 64 blocks are left to the first of them) or one per request (mean
    below), each with a long request among them."""
    rng = np.random.default_rng(5 + top)
    keys = np.unique(rng.integers(1, 2**63, size=60000, dtype=np.uint64))
    gi, oi = HipIndex(1 << 16), oracle.Index(1 << 16)
    present = keys[: len(keys) // 2]
    for ix in (gi, oi):
        ix.insert(present, present >> np.uint64(7))
    sizes = rng.integers(0, top, size=5000)
    sizes[17], sizes[18], sizes[4999] = 1000, 64, 65
    blk_off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(sizes, out=blk_off[1:])
    h = rng.choice(keys, size=int(blk_off[-1]))
    lead = rng.random(len(h)) < 0.9                 # mostly present keys, so matches run long
    h[lead] = rng.choice(present, size=int(lead.sum()))
    gv, gm = gi.match(h, blk_off)
    ov, om = oi.match(h, blk_off)
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)
    assert om.max() > 64


@pytest.mark.parametrize("n_blocks,lg_slots", [((1 << 17) + 777, 16), ((1 << 20) + 333, 16), ((1 << 22) + 5, 16),
                                               ((1 << 20) + 333, 22)])
def test_match_large_batches(n_blocks, lg_slots):
    """Batches of 2^17 to 2^22 blocks over thousands of ragged requests; a table at load 0.75
    with tombstones gives long probe sequences. On the table of 2^22 slots the lookups of a tile
    whose last key is present go through the key words instead of the tags; the 3 % of absent keys
    strewn over the batch make that guess wrong for single keys of most tiles."""
    rng = np.random.default_rng(n_blocks)
    n_slots = 1 << lg_slots
    keys = np.unique(rng.integers(1, 2**63, size=n_slots + n_slots // 4, dtype=np.uint64))
    rng.shuffle(keys)
    present = keys[: int(n_slots * 0.75)]
    gi, oi = HipIndex(n_slots), oracle.Index(n_slots)
    for ix in (gi, oi):
        ix.insert(present, present ^ np.uint64(0x55))
    dropped = present[::9]
    assert np.array_equal(gi.evict(dropped), oi.evict(dropped))      # leaves tombstones behind
    sizes = rng.integers(0, 600, size=n_blocks // 300 + 1)
    sizes[-1] += n_blocks - sizes.sum() if sizes.sum() < n_blocks else 0
    sizes = sizes[np.cumsum(sizes) <= n_blocks]
    sizes = np.append(sizes, n_blocks - sizes.sum())
    blk_off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(sizes, out=blk_off[1:])
    h = rng.choice(keys, size=n_blocks)
    lead = rng.random(n_blocks) < 0.97
    h[lead] = rng.choice(present, size=int(lead.sum()))
    h[5] = 0
    h[6] = NO                                                        # reserved keys read as absent
    two = np.flatnonzero(sizes >= 2)[:2]                             # ... also as the last key of a request's last tile
    h[blk_off[two[0] + 1] - 1] = 0
    h[blk_off[two[1] + 1] - 1] = NO
    gv, gm = gi.match(h, blk_off)
    ov, om = oi.match(h, blk_off)
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)
    assert om.max() >= 8


def test_block_hash_golden_vector_and_empty(hip):
    t = np.arange(32, dtype=np.int32)
    got = hip.block_hash(t, [0, 32], [0, 2], 16, 0)
    assert [int(x) for x in got] == [0xF95A27A48F22F512, 0x7FDA0CD7157322A0]
    assert len(hip.block_hash(t[:0], [0], [0], 16, 0)) == 0
    assert len(hip.block_hash(t[:7], [0, 7], [0, 0], 16, 0)) == 0


# ---- index -------------------------------------------------------------------------------------
def _same_bucket_keys(rng, n_slots, n):
    """Keys whose home bucket (multiplicative hash, top bits) collide often: draw many, keep
    those falling into two buckets."""
    nb = max(n_slots // 8, 1)
    lg = int(np.log2(nb))
    keys = rng.integers(1, 2**63, size=200 * n, dtype=np.uint64)
    if lg == 0:
        return keys[:n]
    home = (keys * np.uint64(0x9E3779B97F4A7C15)) >> np.uint64(64 - lg)
    pick = keys[(home == home[0]) | (home == (home[0] + np.uint64(1)) % np.uint64(nb))]   # two home buckets
    return np.concatenate([pick[: n // 2], keys[: n - min(len(pick), n // 2)]])


@pytest.mark.parametrize("n_slots,seed", [(8, 0), (16, 0), (64, 0), (64, 1), (1024, 0), (1024, 1),
                                           (1024, 2), (1024, 3), (1024, 4), (1024, 5)])
def test_index_random_ops_against_oracle(n_slots, seed):
    """Random batches against the oracle's map. Half of the keys share two home buckets, so probe
    sequences run long, wrap around the table, and many concurrent inserts fight for the same
    tombstones (an insert that loses a claim must rescan, however often that happens)."""
    rng = np.random.default_rng(n_slots * 100 + seed)
    gi, oi = HipIndex(n_slots), oracle.Index(n_slots)
    universe = np.unique(_same_bucket_keys(rng, n_slots, 3 * n_slots))
    for step in range(120):
        op = rng.integers(0, 4)
        m = int(rng.integers(0, min(len(universe), n_slots // 2 + 3)))
        k = rng.choice(universe, size=m, replace=False)
        if op <= 1:
            if gi.count() + m > n_slots:      # which keys survive an overflow is unspecified
                continue
            v = rng.integers(0, 2**40, size=m, dtype=np.uint64)
            gi.insert(k, v)
            oi.insert(k, v)
        elif op == 2:
            assert np.array_equal(gi.evict(k), oi.evict(k))
        else:
            gv, gm = gi.match(k, [0, m])
            ov, om = oi.match(k, [0, m])
            assert np.array_equal(gv, ov) and np.array_equal(gm, om)
        assert gi.count() == oi.count()
    gk, gv = gi.dump()
    ok, ov = oi.dump()
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
    assert np.array_equal(gi.counters_insert, oi.counters_insert)
    assert np.array_equal(gi.counters_evict, oi.counters_evict)
    # every key that ever existed, looked up once more: the tags a lookup walks mirror the keys
    gv, gm = gi.match(universe, [0, len(universe)])
    ov, om = oi.match(universe, [0, len(universe)])
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)


def test_index_beyond_full_is_bounded_and_consistent():
    """A table larger than the probe bound, driven past its capacity: whatever was reported inserted
    is there with its value, the rest was counted full, absent keys are reported absent (each walk
    ends after 4,096 buckets instead of the whole table), and evicting everything empties it."""
    n_slots = 1 << 17
    rng = np.random.default_rng(99)
    gi = HipIndex(n_slots)
    keys = np.unique(rng.integers(1, 2**63, size=n_slots + 5000, dtype=np.uint64))
    rng.shuffle(keys)
    gi.insert(keys, keys >> np.uint64(7))
    ins, upd, full = [int(x) for x in gi.counters_insert]
    assert ins + full == len(keys) and upd == 0 and ins <= n_slots and ins >= int(0.999 * n_slots)
    assert gi.stats() == (ins, 0)
    v, _ = gi.match(keys, [0, len(keys)])
    found = v != NO
    assert int(found.sum()) == ins and np.array_equal(v[found], keys[found] >> np.uint64(7))
    absent = np.setdiff1d(rng.integers(1, 2**63, size=200000, dtype=np.uint64), keys)
    va, ma = gi.match(absent, [0, len(absent)])
    assert np.all(va == NO) and int(ma[0]) == 0
    out = gi.evict(keys)
    assert np.array_equal(out[found], keys[found] >> np.uint64(7)) and np.all(out[~found] == NO)
    assert gi.count() == 0


def _churn(rng, gi, oi, universe, n_slots, steps):
    for _ in range(steps):
        op = rng.integers(0, 5)
        m = int(rng.integers(0, min(len(universe), n_slots // 2 + 3)))
        k = rng.choice(universe, size=m, replace=False)
        if op <= 1:
            if gi.count() + m > n_slots:
                continue
            v = rng.integers(0, 2**40, size=m, dtype=np.uint64)
            gi.insert(k, v)
            oi.insert(k, v)
        elif op == 2:
            assert np.array_equal(gi.evict(k), oi.evict(k))
        elif op == 3:
            e = int(rng.integers(0, 50))
            gi.touch(k, e)
            oi.touch(k, e)
        else:
            gv, gm = gi.match(k, [0, m])
            ov, om = oi.match(k, [0, m])
            assert np.array_equal(gv, ov) and np.array_equal(gm, om)


def _same_index(gi, oi):
    for a, b in zip(gi.dump(), oi.dump()):
        assert np.array_equal(a, b)
    for protect, epoch in ((1, 1), (2, 25), (3, 60), (255, 1 << 20)):
        for a, b in zip(gi.select_victims(protect, epoch), oi.select_victims(protect, epoch)):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("n_slots,seed", [(64, 0), (1024, 0), (1024, 1), (4096, 0)])
def test_index_rebuild_compacts_and_keeps_everything(n_slots, seed):
    """Churn on crowded probe sequences leaves tombstones behind; the rebuilt table has none, holds
    the same keys, values and usage words as the oracle's copy, and goes on working like any index."""
    rng = np.random.default_rng(7000 + n_slots + seed)
    gi, oi = HipIndex(n_slots), oracle.Index(n_slots)
    universe = np.unique(_same_bucket_keys(rng, n_slots, 3 * n_slots))
    _churn(rng, gi, oi, universe, n_slots, 80)
    room = n_slots - n_slots // 16 - gi.count()           # fill up, then evict from the full buckets
    if room > 0:
        absent = np.setdiff1d(universe, oi.dump()[0])[:room]
        gi.insert(absent, absent >> np.uint64(5))
        oi.insert(absent, absent >> np.uint64(5))
    present = oi.dump()[0]
    assert np.array_equal(gi.evict(present[::3]), oi.evict(present[::3]))
    live, tombs = gi.stats()
    assert live == oi.count() and tombs > 0
    g2, o2 = HipIndex(n_slots), oracle.Index(n_slots)
    g2.insert(np.array([12345], dtype=np.uint64), np.array([1], dtype=np.uint64))   # wiped by the rebuild
    assert np.array_equal(gi.rebuild_into(g2), oi.rebuild_into(o2))
    assert g2.stats() == (live, 0)
    _same_index(g2, o2)
    _same_index(gi, oi)                                   # the source is only read
    assert gi.stats() == (live, tombs)
    _churn(rng, g2, o2, universe, n_slots, 60)            # the copy is a working index
    _same_index(g2, o2)
    # same call as a resize: up keeps everything, down keeps as many keys as fit
    g3, o3 = HipIndex(4 * n_slots), oracle.Index(4 * n_slots)
    assert np.array_equal(g2.rebuild_into(g3), o2.rebuild_into(o3))
    _same_index(g3, o3)
    small = max(8, n_slots // 8)
    g4, o4 = HipIndex(small), oracle.Index(small)
    cg, co = g3.rebuild_into(g4), o3.rebuild_into(o4)
    assert np.array_equal(cg, co) and g4.stats() == (o4.count(), 0)
    full = dict(zip(*[x.tolist() for x in o3.dump()]))
    gk, gv = g4.dump()
    assert len(set(gk.tolist())) == len(gk) and all(full[a] == b for a, b in zip(gk.tolist(), gv.tolist()))


def test_index_rebuild_rejects_itself():
    import paper_2504_03648_amd as aibx
    gi = HipIndex(64)
    with pytest.raises(aibx.AibxError) as e:
        aibx.aibx_index_rebuild(gi.h, gi.h)
    assert e.value.status == -1


def test_index_overflow_counts():
    """m > n_slots distinct keys into an empty table: exactly n_slots succeed, the rest are
    counted full; every survivor is found with its value."""
    for n_slots in (8, 64, 512):
        rng = np.random.default_rng(n_slots + 1)
        gi = HipIndex(n_slots)
        keys = np.unique(rng.integers(1, 2**63, size=2 * n_slots + 7, dtype=np.uint64))
        gi.insert(keys, keys >> np.uint64(3))
        assert list(gi.counters_insert) == [n_slots, 0, len(keys) - n_slots]
        assert gi.count() == n_slots
        v, _ = gi.match(keys, [0, len(keys)])
        found = v != NO
        assert found.sum() == n_slots and np.array_equal(v[found], keys[found] >> np.uint64(3))
        # a full table still updates present keys and still reports absent ones as missing
        gi.insert(keys[found][:5], np.arange(5, dtype=np.uint64))
        assert list(gi.counters_insert) == [n_slots, 5, len(keys) - n_slots]
        ev = gi.evict(keys)
        assert (ev != NO).sum() == n_slots and gi.count() == 0
        # tombstones everywhere: inserts must still succeed by reusing them
        gi.insert(keys[: n_slots // 2], keys[: n_slots // 2])
        assert gi.count() == n_slots // 2
        v, _ = gi.match(keys[: n_slots // 2], [0, n_slots // 2])
        assert np.array_equal(v, keys[: n_slots // 2])


def test_index_duplicates_and_reserved_keys():
    gi, oi = HipIndex(256), oracle.Index(256)
    k = np.array([5, 5, 7, 5, 9, 7, 5, 5, 5, 5, 11], dtype=np.uint64)
    v = k * np.uint64(100)
    for ix in (gi, oi):
        ix.insert(k, v)
        ix.insert(np.array([0, NO, 13], dtype=np.uint64), np.array([1, 2, 3], dtype=np.uint64))
    assert np.array_equal(gi.counters_insert, oi.counters_insert)
    assert list(gi.counters_insert) == [5, 7, 2]
    assert all(np.array_equal(a, b) for a, b in zip(gi.dump(), oi.dump()))
    q = np.array([0, NO, 5, 6], dtype=np.uint64)
    assert np.array_equal(gi.match(q, [0, 4])[0], oi.match(q, [0, 4])[0])
    assert np.array_equal(gi.evict(q), oi.evict(q))
    # duplicate keys in one evict batch: exactly one occurrence gets the value
    ev = gi.evict(np.array([7, 7, 7, 9], dtype=np.uint64))
    assert sorted(int(x) for x in ev[:3]) == [700, int(NO), int(NO)] and ev[3] == 900
    assert list(gi.counters_evict) == [3, 5]
    # duplicates with different values: any one of them may win
    gi.insert(np.array([21, 21, 21], dtype=np.uint64), np.array([1, 2, 3], dtype=np.uint64))
    assert int(gi.match(np.array([21], dtype=np.uint64), [0, 1])[0][0]) in (1, 2, 3)


def test_index_large_batch_with_shared_prefix_duplicates():
    """A batch shaped like the real preload: every block of every request, shared prefixes
    repeated, 100k+ keys in one call, then evict half and match."""
    tok, tok_off, blk_off = make_tokens(3, 0, 64)
    h = oracle.block_hash(tok, tok_off, blk_off, 16, 0)
    uniq, inv = np.unique(h, return_inverse=True)
    vals = (np.arange(len(uniq), dtype=np.uint64) + np.uint64(7))[inv]
    gi, oi = HipIndex(1 << 16), oracle.Index(1 << 16)
    for ix in (gi, oi):
        ix.insert(h, vals)
    assert np.array_equal(gi.counters_insert, oi.counters_insert)
    ev = uniq[::2]
    assert np.array_equal(gi.evict(ev), oi.evict(ev))
    gv, gm = gi.match(h, blk_off)
    ov, om = oi.match(h, blk_off)
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)
    assert gi.count() == oi.count()
    assert all(np.array_equal(a, b) for a, b in zip(gi.dump(), oi.dump()))
    gi.clear()
    assert gi.count() == 0


def test_two_block_sizes_and_two_seeds_share_one_index():
    """Engines with different page sizes (16- and 64-token blocks) and two tenants (hash seeds)
    index their blocks in ONE table: each population matches only its own entries, the lengths
    agree with the oracle's, evicting one population leaves the others whole, and the one-launch
    path sees the same state."""
    rng = np.random.default_rng(1664)
    tok, tok_off, lens = _ragged(rng, 40, 64, 3000)
    pops = [(16, 0), (64, 0), (16, 0xABCDEF), (64, 0xABCDEF), (24, 5)]     # (block size, seed)
    gi, oi = HipIndex(1 << 15), oracle.Index(1 << 15)
    hip = HipBackend()
    hs, bos = [], []
    for k, (B, seed) in enumerate(pops):
        bo = np.zeros(len(lens) + 1, dtype=np.int64)
        np.cumsum(lens // B, out=bo[1:])
        h = oracle.block_hash(tok, tok_off, bo, B, seed)
        assert np.array_equal(hip.block_hash(tok, tok_off, bo, B, seed), h)
        hs.append(h)
        bos.append(bo)
        keep = np.arange(len(h)) % 3 != 2 - (k % 2)                        # leave holes so lengths vary
        vals = (np.uint64(k) << np.uint64(32)) | np.arange(len(h), dtype=np.uint64)
        for ix in (gi, oi):
            ix.insert(h[keep], vals[keep])
    assert len(np.unique(np.concatenate(hs))) == sum(len(h) for h in hs)   # the populations never collide
    assert np.array_equal(gi.counters_insert, oi.counters_insert)

    def check():
        for (B, seed), h, bo in zip(pops, hs, bos):
            gv, gm = gi.match(h, bo)
            ov, om = oi.match(h, bo)
            assert np.array_equal(gv, ov) and np.array_equal(gm, om)
            present = gv != NO
            assert np.all((gv[present] >> np.uint64(32)) == np.uint64(pops.index((B, seed))))
            fh, fv, fm = hip_hash_match(gi, tok, tok_off, bo, B, seed)
            assert np.array_equal(fh, h) and np.array_equal(fv, ov) and np.array_equal(fm, om)
    check()
    assert np.array_equal(gi.evict(hs[1]), oi.evict(hs[1]))                # the 64-token blocks of tenant 0 go
    check()
    assert gi.count() == oi.count()
    assert all(np.array_equal(a, b) for a, b in zip(gi.dump(), oi.dump()))


def test_index_load_095_on_a_million_slots_matches_the_oracle():
    """The bound of 4,096 buckets per probe sequence is the one point where the table is not the
    oracle's abstract map. It must not bind where the map has room: a 2^20-slot table driven to a
    load factor of 0.95 in batches, with evictions in between (tombstones), reports exactly the
    oracle's counters, contents and lookups."""
    n_slots = 1 << 20
    rng = np.random.default_rng(95)
    keys = np.unique(rng.integers(1, 2**63, size=int(1.02 * n_slots), dtype=np.uint64))
    rng.shuffle(keys)
    gi, oi = HipIndex(n_slots), oracle.Index(n_slots)
    target = int(0.95 * n_slots)
    step = 1 << 17
    live_hi = 0
    for a in range(0, target, step):
        b = min(target, a + step)
        for ix in (gi, oi):
            ix.insert(keys[a:b], keys[a:b] ^ np.uint64(0x55))
        ev = keys[a:b][:: 16]                                               # evict a sixteenth again ...
        assert np.array_equal(gi.evict(ev), oi.evict(ev))
        for ix in (gi, oi):
            ix.insert(ev, ev + np.uint64(1))                                # ... and bring it back with new values
        live_hi = b
    assert np.array_equal(gi.counters_insert, oi.counters_insert)
    assert int(gi.counters_insert[2]) == 0 and gi.count() == oi.count() == target
    probe = np.concatenate([keys[:live_hi][:: 7], keys[target:]])          # present and absent keys
    bo = np.array([0, len(probe)], dtype=np.int64)
    gv, gm = gi.match(probe, bo)
    ov, om = oi.match(probe, bo)
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)
    assert all(np.array_equal(a, b) for a, b in zip(gi.dump(), oi.dump()))
    assert np.array_equal(gi.counters_evict, oi.counters_evict)


def test_key_word_search_walks_long_sequences_on_a_large_full_table():
    """Tables of 2^22 slots take a tile's lookups through the key words when the tile's last key is
    present. Here that guess holds for every tile while half of the other keys are absent, on a table
    at load 0.95 with tombstones: absent keys walk many full buckets of their probe sequence in the
    key words, present ones sit deep in theirs. Values and match lengths equal the oracle's."""
    n_slots = 1 << 22
    rng = np.random.default_rng(2295)
    keys = np.unique(rng.integers(1, 2**63, size=int(1.2 * n_slots), dtype=np.uint64))
    rng.shuffle(keys)
    target = int(0.95 * n_slots)
    present, absent = keys[:target], keys[target:]
    gi, oi = HipIndex(n_slots), oracle.Index(n_slots)
    for ix in (gi, oi):
        ix.insert(present, present >> np.uint64(3))
    gone = present[::16]
    assert np.array_equal(gi.evict(gone), oi.evict(gone))               # tombstones in full buckets
    back = gone[::2]
    for ix in (gi, oi):
        ix.insert(back, back + np.uint64(7))                             # half of them return, into tombstones
    assert np.array_equal(gi.counters_insert, oi.counters_insert) and int(gi.counters_insert[2]) == 0
    live = np.setdiff1d(present, gone[1::2])
    sizes = rng.integers(1, 200, size=3000)
    blk_off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(sizes, out=blk_off[1:])
    n = int(blk_off[-1])
    h = rng.choice(live, size=n)
    holes = rng.random(n) < 0.5
    h[holes] = rng.choice(np.concatenate([absent, gone[1::2]]), size=int(holes.sum()))
    for r in range(len(sizes)):                                          # the last key of every tile of every request is present
        ends = np.arange(blk_off[r] + 63, blk_off[r + 1], 64)
        ends = np.append(ends, blk_off[r + 1] - 1)
        h[ends] = rng.choice(live, size=len(ends))
    gv, gm = gi.match(h, blk_off)
    ov, om = oi.match(h, blk_off)
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)
    assert (ov == NO).sum() > n // 3 and (ov != NO).sum() > n // 3


def test_match_edge_cases():
    gi, oi = HipIndex(64), oracle.Index(64)
    keys = np.arange(1, 30, dtype=np.uint64)
    for ix in (gi, oi):
        ix.insert(keys[::2], keys[::2])
    # requests with 0 blocks, 1 block, exactly 64, 65 and 300 blocks (several tiles per request)
    sizes = [0, 1, 64, 65, 300, 0, 3]
    blk_off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(sizes, out=blk_off[1:])
    rng = np.random.default_rng(0)
    h = rng.choice(keys, size=int(blk_off[-1])).astype(np.uint64)
    h[blk_off[4]:blk_off[4] + 130] = 1          # a long matched run across tiles
    gv, gm = gi.match(h, blk_off)
    ov, om = oi.match(h, blk_off)
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)
    assert gm[4] >= 130


# ---- usage tracking and victim selection ------------------------------------------------------------
@pytest.mark.parametrize("n_slots,seed", [(64, 0), (1024, 0), (1024, 1), (1 << 16, 0)])
def test_eviction_policy_random_ops_against_oracle(n_slots, seed):
    rng = np.random.default_rng(n_slots + seed)
    gi, oi = HipIndex(n_slots), oracle.Index(n_slots)
    universe = np.unique(rng.integers(1, 2**63, size=2 * n_slots, dtype=np.uint64))
    for step in range(80):
        op = int(rng.integers(0, 6))
        m = int(rng.integers(0, max(2, n_slots // 3)))
        if op == 0:
            k = rng.choice(universe, size=m, replace=False)
            if gi.count() + m > n_slots:
                continue
            v = rng.integers(0, 2**40, size=m, dtype=np.uint64)
            gi.insert(k, v)
            oi.insert(k, v)
        elif op == 1:
            k = rng.choice(universe, size=m, replace=False)
            assert np.array_equal(gi.evict(k), oi.evict(k))
        elif op == 2 or op == 3:
            k = rng.choice(universe, size=3 * m, replace=True)       # duplicates: touched several times
            e = int(rng.integers(0, 40))
            gi.touch(k, e)
            oi.touch(k, e)
        elif op == 4 and step % 5 == 0:
            gi.age()
            oi.age()
        pc, be = int(rng.integers(0, 6)), int(rng.integers(0, 45))
        gk, gv = gi.select_victims(pc, be)
        ok, ov = oi.select_victims(pc, be)
        assert np.array_equal(gk, ok) and np.array_equal(gv, ov), (step, op)
    # saturation of the touch count
    k = universe[:1]
    for ix in (gi, oi):
        ix.insert(k, k)
        ix.touch(np.repeat(k, 700), 1)
    assert np.array_equal(gi.select_victims(255, 50)[0], oi.select_victims(255, 50)[0])
    assert np.array_equal(gi.select_victims(256, 50)[0], oi.select_victims(256, 50)[0])


def test_scan_does_not_push_out_reused_blocks_full_flow():
    """Config-2-shaped traffic: shared prefixes are touched by every request of their group each
    epoch, unique tails once; the victims must be exactly the old unique tails."""
    wl = make_workload(2, "small")
    h = oracle.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, 0)
    gi, oi = HipIndex(1 << 14), oracle.Index(1 << 14)
    uniq = np.unique(h)
    for ix in (gi, oi):
        ix.insert(uniq, uniq >> np.uint64(5))
        for r in range(wl.n_req):                       # request r arrives in epoch r + 1
            ix.touch(h[wl.blk_off[r]:wl.blk_off[r + 1]], r + 1)
    gk, gv = gi.select_victims(2, wl.n_req // 2 + 1)
    ok, ov = oi.select_victims(2, wl.n_req // 2 + 1)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
    shared = {int(x) for r in range(wl.n_req) for x in h[wl.blk_off[r]:wl.blk_off[r] + 2048 // wl.block_size]}
    assert len(ok) > 0 and not (set(int(x) for x in ok) & shared)


# ---- hash + match in one launch -------------------------------------------------------------------
@pytest.mark.parametrize("B,n_req,lg_slots", [(16, 37, 18), (32, 21, 18), (64, 19, 18), (16, 5000, 18), (64, 4500, 18),
                                              (24, 11, 18), (16, 37, 22), (32, 21, 22), (64, 4500, 22), (16, 5000, 22)])
def test_hash_match_equals_hash_then_match(B, n_req, lg_slots):
    """Few requests (8 wavefronts each), thousands (1 wavefront each, 4 for the long ones), and a
    block size that runs as two launches; half of the requests are indexed, a slice of their blocks
    evicted again (holes inside cached prefixes). Tables of 2^22 slots take the lookups of a tile
    through the key words where the tile's last block is present."""
    rng = np.random.default_rng(B * 7 + n_req)
    tok, tok_off, lens = _ragged(rng, n_req, 0, 30 * B if n_req > 1000 else 150 * B)
    lens[1] = 0
    lens[2] = B - 1
    # requests long enough to take several rounds of their workgroup's wavefronts, in large and small batches
    lens[6], lens[7], lens[8] = 8192 + 3 * B, 8192 + 3 * B + 40, 21 * 1024 + 7
    np.cumsum(lens, out=tok_off[1:])
    tok = rng.integers(0, 32000, size=int(tok_off[-1]), dtype=np.int32)
    # requests come in pairs that share a prefix of the first of the two
    for r in range(1, n_req, 2):
        k = min(int(lens[r]), int(lens[r - 1])) * 2 // 3
        tok[tok_off[r]:tok_off[r] + k] = tok[tok_off[r - 1]:tok_off[r - 1] + k]
    blk_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(lens // B, out=blk_off[1:])
    want_h = oracle.block_hash(tok, tok_off, blk_off, B, 11)
    gi, oi = HipIndex(1 << lg_slots), oracle.Index(1 << lg_slots)
    cached = np.concatenate([want_h[blk_off[r]:blk_off[r + 1]] for r in range(0, n_req, 2)] + [want_h[:0]])
    cached = np.unique(cached)
    for ix in (gi, oi):
        ix.insert(cached, cached >> np.uint64(9))
        ix.evict(cached[::17])
    want_v, want_m = oi.match(want_h, blk_off)
    h, v, m = hip_hash_match(gi, tok, tok_off, blk_off, B, 11)
    assert np.array_equal(h, want_h) and np.array_equal(v, want_v) and np.array_equal(m, want_m)
    if B != 24:
        h2, v2, m2 = hip_hash_match(gi, tok, tok_off, blk_off, B, 11, want_hashes=False, want_values=False)
        assert h2 is None and v2 is None and np.array_equal(m2, want_m)
    assert want_m.max() > 0


# ---- routing decision -----------------------------------------------------------------------------
@pytest.mark.parametrize("n_pods,num,den", [(1, 1, 2), (7, 0, 1), (7, 1, 2), (7, 9, 10), (63, 1, 3), (63, 2, 1)])
def test_route_parity(n_pods, num, den):
    import torch
    import paper_2504_03648_amd as aibx
    rng = np.random.default_rng(n_pods * 100 + num)
    n_req = 300
    sizes = rng.integers(0, 400, size=n_req)
    sizes[:4] = [0, 1, 64, 65]
    blk_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(sizes, out=blk_off[1:])
    n = int(blk_off[-1])
    all_pods = (1 << n_pods) - 1
    sets = np.zeros(n, dtype=np.uint64)
    for r in range(n_req):
        # a few pods hold a long prefix each, the rest is sparse noise
        k = int(sizes[r])
        row = rng.integers(0, 1 << min(n_pods, 62), size=k, dtype=np.uint64) & rng.integers(0, 1 << min(n_pods, 62), size=k, dtype=np.uint64)
        for p in rng.integers(0, n_pods, size=3):
            row[: int(rng.integers(0, k + 1))] |= np.uint64(1) << np.uint64(p)
        sets[blk_off[r]:blk_off[r + 1]] = row & np.uint64(all_pods)
    sets[rng.random(n) < 0.01] = NO
    load = rng.integers(0, 5, size=n_pods).astype(np.int32)
    want_pod, want_hit = oracle.route(sets, blk_off, n_pods, load, num, den)
    d_sets = torch.from_numpy(sets.view(np.int64).copy()).cuda()
    d_bo = torch.from_numpy(blk_off).cuda()
    d_load = torch.from_numpy(load).cuda()
    pod = torch.full((n_req,), -9, dtype=torch.int32, device="cuda")
    hit = torch.full((n_req,), -9, dtype=torch.int32, device="cuda")
    aibx.aibx_route(d_sets, d_bo, n_req, n, n_pods, d_load, num, den, pod, hit)
    assert np.array_equal(pod.cpu().numpy(), want_pod) and np.array_equal(hit.cpu().numpy(), want_hit)
    assert want_hit.max() > 64


@pytest.mark.parametrize("B,n_req,n_pods,num,den,lg_slots", [
    (16, 70, 7, 1, 2, 18), (32, 41, 63, 1, 3, 18), (64, 33, 5, 0, 1, 18), (16, 4500, 8, 1, 2, 18),
    (64, 4200, 3, 9, 10, 18), (16, 9, 1, 2, 1, 18), (16, 70, 7, 1, 2, 22), (64, 4200, 3, 9, 10, 22)])
def test_hash_match_route_equals_the_three_calls(B, n_req, n_pods, num, den, lg_slots):
    """Tokens in, pod out: the one-launch routing decision against the oracle's hash -> match ->
    route chain, on requests that share prefixes, with pods holding prefixes of every length
    (none, part of a tile, whole tiles, everything), zero-block requests, and both launch shapes
    (small batches share long requests between wavefronts; thousands of requests get one each)."""
    import torch
    import paper_2504_03648_amd as aibx
    rng = np.random.default_rng(B * 1000 + n_req)
    big = n_req >= 4096
    tok, tok_off, lens = _ragged(rng, n_req, 0, 700 if big else 6000)
    lens[:5] = [0, B - 1, B, 64 * B, 64 * B + 1][: min(5, n_req)]
    tok_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(lens, out=tok_off[1:])
    tok = rng.integers(0, 32000, size=int(tok_off[-1]), dtype=np.int32)
    for r in range(1, n_req, 3):                                       # every third request repeats its neighbour's start
        k = int(min(lens[r], lens[r - 1]) * rng.random())
        tok[tok_off[r]:tok_off[r] + k] = tok[tok_off[r - 1]:tok_off[r - 1] + k]
    blk_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(lens // B, out=blk_off[1:])
    h = oracle.block_hash(tok, tok_off, blk_off, B, 11)
    n = len(h)
    sets = np.zeros(n, dtype=np.uint64)                                # which pods hold block b of which request
    for r in range(n_req):
        n_r = int(blk_off[r + 1] - blk_off[r])
        for p in rng.integers(0, n_pods, size=3):
            L = int(rng.choice([0, n_r, rng.integers(0, n_r + 1), min(n_r, 64), min(n_r, 65)]))
            sets[blk_off[r]:blk_off[r] + L] |= np.uint64(1) << np.uint64(p)
    uniq, inv = np.unique(h, return_inverse=True)
    per_key = np.zeros(len(uniq), dtype=np.uint64)
    np.bitwise_or.at(per_key, inv, sets)                               # a shared block is held by the union
    present = per_key != 0
    gi, oi = HipIndex(1 << lg_slots), oracle.Index(1 << lg_slots)
    for ix in (gi, oi):
        ix.insert(uniq[present], per_key[present])
        ix.insert(rng.integers(1, 2**63, size=50000, dtype=np.uint64), np.full(50000, 1, dtype=np.uint64))
    load = rng.integers(0, 4, size=n_pods).astype(np.int32)
    values, _ = oi.match(h, blk_off)
    want_pod, want_hit = oracle.route(values, blk_off, n_pods, load, num, den)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    pod = torch.full((n_req,), -9, dtype=torch.int32, device="cuda")
    hit = torch.full((n_req,), -9, dtype=torch.int32, device="cuda")
    aibx.aibx_hash_match_route(gi.h, d(tok), d(tok_off), d(blk_off), n_req, n, B, 11, n_pods, d(load), num, den, pod, hit)
    assert np.array_equal(pod.cpu().numpy(), want_pod) and np.array_equal(hit.cpu().numpy(), want_hit)
    assert want_hit.max() > (64 if not big else 8) and (want_hit == 0).any()
    # and the three library calls in a row agree as well
    hh = torch.empty(n, dtype=torch.int64, device="cuda")
    vv = torch.empty(n, dtype=torch.int64, device="cuda")
    mm = torch.empty(n_req, dtype=torch.int32, device="cuda")
    pod3, hit3 = torch.empty_like(pod), torch.empty_like(hit)
    aibx.aibx_hash_match(gi.h, d(tok), d(tok_off), d(blk_off), n_req, n, B, 11, hh, vv, mm)
    aibx.aibx_route(vv, d(blk_off), n_req, n, n_pods, d(load), num, den, pod3, hit3)
    assert torch.equal(pod, pod3) and torch.equal(hit, hit3)


# ---- gather / scatter --------------------------------------------------------------------------
@pytest.mark.parametrize("n_seg,seg_bytes,n_pages,n", [
    (1, 262144, 40, 23), (64, 32768, 24, 17), (61, 73728, 12, 9), (5, 16, 50, 33),
    (3, 4096 + 16, 30, 30), (2, 8192, 30, 1), (7, 48, 9, 64), (1, 16, 1, 1), (4, 12288, 20, 11)])
def test_gather_scatter_parity(n_seg, seg_bytes, n_pages, n):
    g = Geometry(n_seg, seg_bytes, n_pages)
    rng = np.random.default_rng(n_seg * 1000 + n)
    host = rng.integers(0, 256, size=g.pool_bytes, dtype=np.uint8)
    ob, hb = OracleBackend(), HipBackend()
    ob.geom, ob.pool = g, host.copy()
    hb.pool_create(g, None, None, host_bytes=host.copy())
    stride = g.blk_bytes + (32 if n_seg == 5 else 0)
    n_slots = n + 3
    for be in (ob, hb):
        be.staging_create(n_slots, stride)
    ids = rng.integers(0, n_pages, size=n).astype(np.int32)
    if n > 4:
        ids[1] = -1
        ids[2] = n_pages           # bad page
        ids[3] = 2**31 - 1         # bad page
    slots = rng.permutation(n_slots)[:n].astype(np.int32)
    all_slots = np.arange(n_slots, dtype=np.int32)
    for sl in (None, slots):
        bo, bh = ob.gather(ids, sl), hb.gather(ids, sl)
        assert bo == bh == (2 if n > 4 else 0)
        assert np.array_equal(hb.staging.cpu().numpy(), ob.staging)      # whole staging, padding included
    # scatter distinct pages back from shuffled slots
    pages = rng.permutation(n_pages)[: min(n, n_pages)].astype(np.int32)
    sl = slots[: len(pages)]
    assert ob.scatter(pages, sl) == hb.scatter(pages, sl) == 0
    assert np.array_equal(hb.pool.cpu().numpy(), ob.pool)                # whole pool
    assert np.array_equal(hb.read_slots(all_slots), ob.read_slots(all_slots))
    hb.check_guards()                                                    # canaries around pool and staging intact


@pytest.mark.parametrize("n_seg,seg_bytes,n_pages,n", [(64, 32768, 24, 17), (61, 73728, 12, 9), (1, 262144, 20, 20),
                                                        (5, 48, 30, 33), (3, 4096 + 16, 30, 25), (2, 16, 4, 4)])
def test_partly_filled_blocks_parity(n_seg, seg_bytes, n_pages, n):
    """aibx_kv_gather_fill / _scatter_fill against the oracle: every fill from nothing to the whole
    segment, counts that are negative, not multiples of 16 or larger than a segment, holes and
    out-of-range pages; whole staging buffer and whole pool compared, canaries around both."""
    import torch
    import paper_2504_03648_amd as aibx
    g = Geometry(n_seg, seg_bytes, n_pages)
    rng = np.random.default_rng(n_seg * 31 + n)
    host = rng.integers(0, 256, size=g.pool_bytes, dtype=np.uint8)
    hb = HipBackend()
    hb.pool_create(g, None, None, host_bytes=host.copy())
    stride = g.blk_bytes + (48 if n_seg == 5 else 0)
    n_slots = n + 2
    hb.staging_create(n_slots, stride)
    hb.staging.fill_(0x5A)
    o_pool, o_st = host.copy(), np.full(n_slots * stride, 0x5A, dtype=np.uint8)
    ids = rng.permutation(n_pages)[:n].astype(np.int32) if n <= n_pages else rng.integers(0, n_pages, size=n).astype(np.int32)
    fill = (rng.integers(0, seg_bytes // 16 + 1, size=n) * 16).astype(np.int32)
    fill[0] = seg_bytes
    if n > 6:
        fill[1], fill[2], fill[3], fill[4] = 0, -7, seg_bytes + 4096, min(seg_bytes, 16 * 3) - 5
        ids[5] = -1
        ids[6] = n_pages
    slots = rng.permutation(n_slots)[:n].astype(np.int32)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    want_bad = oracle.kv_gather_fill(o_pool, g.as_tuple(), ids, slots, fill, o_st, stride)
    aibx.aibx_kv_gather_fill(hb.desc, d(ids), d(slots), d(fill), n, hb.staging, stride, bad)
    assert int(bad.item()) == want_bad == (1 if n > 6 else 0)
    assert np.array_equal(hb.staging.cpu().numpy(), o_st)
    assert np.array_equal(hb.pool.cpu().numpy(), o_pool)
    # scatter other bytes back into (distinct) pages, partly
    fresh = rng.integers(0, 256, size=n_slots * stride, dtype=np.uint8)
    o_st[:] = fresh
    hb.staging.copy_(torch.from_numpy(fresh))
    pages = rng.permutation(n_pages)[: min(n, n_pages)].astype(np.int32)
    k = len(pages)
    bad.zero_()
    assert oracle.kv_scatter_fill(o_pool, g.as_tuple(), pages, slots[:k], fill[:k], o_st, stride) == 0
    aibx.aibx_kv_scatter_fill(hb.desc, d(pages), d(slots[:k]), d(fill[:k]), k, hb.staging, stride, bad)
    assert int(bad.item()) == 0
    assert np.array_equal(hb.pool.cpu().numpy(), o_pool)
    assert np.array_equal(hb.staging.cpu().numpy(), o_st)
    # NULL fill = the plain copy
    aibx.aibx_kv_gather_fill(hb.desc, d(pages), d(slots[:k]), None, k, hb.staging, stride, bad)
    oracle.kv_gather(o_pool, g.as_tuple(), pages, slots[:k], o_st, stride)
    assert np.array_equal(hb.staging.cpu().numpy(), o_st)
    hb.check_guards()


def test_gather_then_scatter_is_identity_on_the_pool():
    g = Geometry(8, 32768, 300)
    hb = HipBackend()
    hb.pool_create(g, "bf16", 2)
    keep = hb.pool.clone()
    ids = np.random.default_rng(0).permutation(300)[:200].astype(np.int32)
    hb.staging_create(200, g.blk_bytes)
    assert hb.gather(ids, None) == 0
    hb.fill_pages(ids, 0xA5)
    assert not hb.t.equal(hb.pool, keep)
    assert hb.scatter(ids, None) == 0
    assert hb.t.equal(hb.pool, keep)


# ---- copies with a layout conversion ---------------------------------------------------------------
def _token_major(S, T, run, n_pages):
    return (S, T, run, T * S * run, S * run, run, n_pages)


@pytest.mark.parametrize("S,T,run,n_pages,n,pad", [
    (64, 16, 2048, 40, 23, 0),        # config-2 page seen token-major: runs of one token's K or V heads
    (61, 64, 1152, 9, 7, 0),          # MLA latent + rope key per token
    (64, 16, 1024, 30, 30, 64),       # fp8 bytes, padded staging blocks
    (3, 5, 16, 50, 33, 0), (1, 7, 48, 12, 12, 16), (2, 300, 4096 + 16, 6, 5, 0)])
def test_gather_scatter_runs_parity(S, T, run, n_pages, n, pad):
    import torch
    import paper_2504_03648_amd as aibx
    g = _token_major(S, T, run, n_pages)
    blk = S * T * run
    stride = blk + pad
    rng = np.random.default_rng(S * 100 + T)
    host_pool = rng.integers(0, 256, size=n_pages * blk, dtype=np.uint8)
    pool = torch.from_numpy(host_pool.copy()).cuda()
    desc = aibx.make_pool_runs_desc(pool, *g)
    ids = rng.permutation(n_pages)[:n].astype(np.int32)
    slots = rng.permutation(n).astype(np.int32)
    if n > 4:
        ids[1], ids[3] = -1, n_pages
    d_ids, d_slots = torch.from_numpy(ids).cuda(), torch.from_numpy(slots).cuda()
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    staging = torch.full((n * stride,), 0x5A, dtype=torch.uint8, device="cuda")
    aibx.aibx_kv_gather_runs(desc, d_ids, d_slots, n, staging, stride, bad)
    want = np.full(n * stride, 0x5A, dtype=np.uint8)
    n_bad = oracle.kv_gather_runs(host_pool, g, ids, slots, want, stride)
    assert np.array_equal(staging.cpu().numpy(), want) and int(bad.item()) == n_bad
    # scatter other bytes back through the same list
    fresh = rng.integers(0, 256, size=n * stride, dtype=np.uint8)
    staging.copy_(torch.from_numpy(fresh).cuda())
    aibx.aibx_kv_scatter_runs(desc, d_ids, d_slots, n, staging, stride, bad)
    n_bad += oracle.kv_scatter_runs(host_pool, g, ids, slots, fresh, stride)
    assert np.array_equal(pool.cpu().numpy(), host_pool) and int(bad.item()) == n_bad
    # without slot ids
    aibx.aibx_kv_gather_runs(desc, d_ids, None, n, staging, stride, None)
    oracle.kv_gather_runs(host_pool, g, ids, None, fresh, stride)
    assert np.array_equal(staging.cpu().numpy(), fresh)


def test_one_run_per_segment_equals_the_plain_copy():
    import torch
    import paper_2504_03648_amd as aibx
    g = Geometry(8, 32768, 60)
    hb = HipBackend()
    hb.pool_create(g, "bf16", 3)
    ids = torch.from_numpy(np.random.default_rng(4).permutation(60)[:41].astype(np.int32)).cuda()
    a = torch.zeros(41 * g.blk_bytes, dtype=torch.uint8, device="cuda")
    b = torch.zeros_like(a)
    aibx.aibx_kv_gather(hb.desc, ids, None, 41, a, g.blk_bytes)
    n_seg, seg_stride, page_stride, seg_bytes, n_pages = g.as_tuple()
    rd = aibx.make_pool_runs_desc(hb.pool, n_seg, 1, seg_stride, page_stride, 0, seg_bytes, n_pages)
    aibx.aibx_kv_gather_runs(rd, ids, None, 41, b, g.blk_bytes)
    assert torch.equal(a, b) and bool(a.any())


# ---- host tier ----------------------------------------------------------------------------------
@pytest.mark.parametrize("n_seg,seg_bytes,n,pad", [(6, 4096, 77, 0), (1, 65536, 40, 0), (64, 32768, 50, 0),
                                                   (3, 48, 33, 32), (2, 4096 + 16, 600, 16)])
def test_offload_to_host_and_onload_back(n_seg, seg_bytes, n, pad):
    import torch
    import paper_2504_03648_amd as aibx
    n_pages = max(200, n + 50)
    g = Geometry(n_seg, seg_bytes, n_pages)
    rng = np.random.default_rng(n_seg + n)
    host_pool = rng.integers(0, 256, size=g.pool_bytes, dtype=np.uint8)
    hb = HipBackend()
    hb.pool_create(g, None, None, host_bytes=host_pool.copy())
    ids = rng.permutation(n_pages)[:n].astype(np.int32)
    ids[3], ids[5] = -1, n_pages                           # a hole and a bad page
    d_ids = torch.from_numpy(ids).cuda()
    h_stride = g.blk_bytes + pad
    h_buf = torch.full((n * h_stride,), 0x3C, dtype=torch.uint8).pin_memory()
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    aibx.aibx_kv_offload(hb.desc, d_ids, n, h_buf, h_stride, bad)
    torch.cuda.synchronize()
    # the oracle's gather with slot i = entry i: skipped entries and the padding keep their bytes
    want = np.full(n * h_stride, 0x3C, dtype=np.uint8)
    assert oracle.kv_gather(host_pool, g.as_tuple(), ids, None, want, h_stride) == 1
    assert np.array_equal(h_buf.numpy(), want)
    assert int(bad.item()) == 1
    # wipe the moved pages, put other bytes where the skipped entries' host blocks are, onload
    moved = np.ones(n, dtype=bool)
    moved[[3, 5]] = False
    hb.fill_pages(ids[moved], 0xA5)
    aibx.aibx_kv_onload(hb.desc, d_ids, n, h_buf, h_stride, bad)
    torch.cuda.synchronize()
    assert np.array_equal(hb.pool.cpu().numpy(), host_pool)
    assert int(bad.item()) == 2
    # onload of other bytes against the oracle's scatter
    fresh = rng.integers(0, 256, size=n * h_stride, dtype=np.uint8)
    h_buf.copy_(torch.from_numpy(fresh))
    aibx.aibx_kv_onload(hb.desc, d_ids, n, h_buf, h_stride, None)
    torch.cuda.synchronize()
    assert oracle.kv_scatter(host_pool, g.as_tuple(), ids, None, fresh, h_stride) == 1
    assert np.array_equal(hb.pool.cpu().numpy(), host_pool)


def test_host_tier_refuses_memory_the_gpu_cannot_address():
    import torch
    import paper_2504_03648_amd as aibx
    g = Geometry(4, 4096, 64)
    hb = HipBackend()
    hb.pool_create(g, "bf16", 1)
    ids = torch.arange(8, dtype=torch.int32, device="cuda")
    pageable = torch.zeros(8 * g.blk_bytes, dtype=torch.uint8)
    pinned = torch.zeros(8 * g.blk_bytes, dtype=torch.uint8).pin_memory()
    keep = hb.pool.clone()
    for fn in (aibx.aibx_kv_offload, aibx.aibx_kv_onload):
        with pytest.raises(aibx.AibxError) as e:
            fn(hb.desc, ids, 8, pageable, g.blk_bytes)
        assert e.value.status == -1
        with pytest.raises(aibx.AibxError) as e:          # 1 GiB of host blocks claimed, 128 KiB allocated
            fn(hb.desc, ids, 8, pinned, 1 << 27)
        assert e.value.status == -1
    torch.cuda.synchronize()
    assert torch.equal(hb.pool, keep) and int(pinned.sum()) == 0
    aibx.aibx_kv_offload(hb.desc, ids, 8, pinned, g.blk_bytes)       # the library still works afterwards
    torch.cuda.synchronize()
    want = np.zeros(8 * g.blk_bytes, dtype=np.uint8)
    oracle.kv_gather(hb.pool.cpu().numpy(), g.as_tuple(), ids.cpu().numpy(), None, want, g.blk_bytes)
    assert np.array_equal(pinned.numpy(), want)


# ---- HIP graph capture ----------------------------------------------------------------------------
def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """Every entry point only launches kernels on the caller's stream (no allocation, no memset), so
    a sequence of calls can be captured once and replayed. Each replay is checked against the
    eager results, with eager work and synchronisations between the replays."""
    import torch
    import paper_2504_03648_amd as aibx
    wl = make_workload(2, "small")
    g = wl.geom
    d_tok = torch.from_numpy(wl.tokens).cuda()
    d_to, d_bo = torch.from_numpy(wl.tok_off).cuda(), torch.from_numpy(wl.blk_off).cuda()
    N, R = wl.n_blocks, wl.n_req
    h = torch.zeros(N, dtype=torch.int64, device="cuda")
    v = torch.zeros(N, dtype=torch.int64, device="cuda")
    m = torch.zeros(R, dtype=torch.int32, device="cuda")
    vals = torch.zeros(N, dtype=torch.int64, device="cuda")
    storage = torch.empty(aibx.aibx_index_storage_bytes(1 << 14), dtype=torch.uint8, device="cuda")
    ix = aibx.aibx_index_create(storage, 1 << 14)
    pool = torch.from_numpy(np.random.default_rng(0).integers(0, 256, size=g.pool_bytes, dtype=np.uint8)).cuda()
    desc = aibx.make_pool_desc(pool, *g.as_tuple())
    n = 300
    pages = torch.from_numpy(np.random.default_rng(1).permutation(g.n_pages)[:n].astype(np.int32)).cuda()
    back = torch.from_numpy(np.random.default_rng(2).permutation(g.n_pages)[:n].astype(np.int32)).cuda()
    staging = torch.zeros(n * g.blk_bytes, dtype=torch.uint8, device="cuda")
    staging2 = torch.zeros(n * g.blk_bytes, dtype=torch.uint8, device="cuda")
    fill = torch.from_numpy((np.random.default_rng(3).integers(0, g.seg_bytes // 16 + 1, size=n) * 16).astype(np.int32)).cuda()
    pod_load = torch.zeros(8, dtype=torch.int32, device="cuda")
    pod = torch.zeros(R, dtype=torch.int32, device="cuda")
    hit = torch.zeros(R, dtype=torch.int32, device="cuda")

    def sequence():
        aibx.aibx_index_clear(ix)
        aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, wl.block_size, 0, h)
        aibx.aibx_index_insert(ix, h, vals, N, None)
        aibx.aibx_index_evict(ix, evict_keys, evict_keys.numel(), ev, None)
        aibx.aibx_prefix_match(ix, h, d_bo, R, N, v, m)
        aibx.aibx_kv_gather(desc, pages, None, n, staging, g.blk_bytes, None)
        aibx.aibx_kv_scatter(desc, back, None, n, staging, g.blk_bytes, None)
        aibx.aibx_kv_gather_fill(desc, pages, None, fill, n, staging2, g.blk_bytes, None)
        aibx.aibx_hash_match_route(ix, d_tok, d_to, d_bo, R, N, wl.block_size, 0, 8, pod_load, 1, 2, pod, hit)

    # Requests share prefixes, so the batch repeats keys: values are a function of the key and the
    # evicted keys are distinct, which makes every output independent of the order of equal keys.
    aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, wl.block_size, 0, h)
    vals.copy_(h & 0xFFFF)
    evict_keys = torch.unique(h)[::3].contiguous()
    ev = torch.zeros_like(evict_keys)
    pool0 = pool.clone()
    sequence()
    torch.cuda.synchronize()
    want = [x.clone() for x in (h, v, m, ev, staging, pool, staging2, pod, hit)]
    assert int((v == -1).sum()) > 0 and int((v != -1).sum()) > 0

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    pool.copy_(pool0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sequence()
    for replay in range(3):
        for x in (h, v, ev, staging, staging2, pod, hit):
            x.zero_()                                   # eager work between the replays
        m.fill_(-1)
        pool.copy_(pool0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, w in zip((h, v, m, ev, staging, pool, staging2, pod, hit), want):
            assert torch.equal(got, w), replay
    aibx.aibx_index_destroy(ix)


# ---- whole flows on the small configs ----------------------------------------------------------
@pytest.mark.parametrize("cfg", [1, 3, 4])
def test_flow_match_roundtrip_small(cfg):
    wl = make_workload(cfg, "small")
    a = flows.flow_match_roundtrip(wl, OracleBackend())
    hb = HipBackend()
    b = flows.flow_match_roundtrip(wl, hb)
    assert flows.traces_equal(a, b) == []
    from workloads import fill_pool_numpy
    assert np.array_equal(hb.pool.cpu().numpy(), fill_pool_numpy(wl.geom, wl.kv_dtype, wl.cfg))


@pytest.mark.parametrize("layout", [None, "page-major"])
def test_flow_offload_onload_small(layout):
    wl = make_workload(2, "small", layout=layout)
    ob, hb = OracleBackend(), HipBackend()
    a = flows.flow_offload_onload(wl, ob)
    b = flows.flow_offload_onload(wl, hb)
    assert flows.traces_equal(a, b) == []
    assert np.array_equal(hb.pool.cpu().numpy(), ob.pool)
    assert np.array_equal(hb.staging.cpu().numpy(), ob.staging)
    hb.check_guards()


def test_flow_stress_small_two_streams():
    wl = make_workload(5, "small")
    ob, hb = OracleBackend(), HipBackend(two_streams=True)
    a = flows.flow_stress(wl, ob, n_rounds=6, q=512)
    b = flows.flow_stress(wl, hb, n_rounds=6, q=512)
    assert flows.traces_equal(a, b) == []
    assert np.array_equal(hb.pool.cpu().numpy(), ob.pool)
    assert np.array_equal(hb.staging.cpu().numpy(), ob.staging)
    hb.check_guards()
