"""Pins for the oracle's usage tracking and victim selection: a dict model, the rules one by one,
and the property the policy is named for (a one-off scan does not push out the reused blocks)."""
import numpy as np

import oracle


def test_rules_one_by_one():
    ix = oracle.Index(64)
    k = np.arange(1, 11, dtype=np.uint64)
    ix.insert(k, k * np.uint64(3))
    # nothing touched yet: count 0, last 0 -> all are victims for any protect_count >= 1, epoch >= 1
    vk, vv = ix.select_victims(1, 1)
    assert list(vk) == list(k) and list(vv) == [3 * x for x in range(1, 11)]
    assert len(ix.select_victims(0, 100)[0]) == 0 and len(ix.select_victims(5, 0)[0]) == 0
    ix.touch(k[:4], 7)                       # keys 1..4: count 1, last 7
    ix.touch(k[:2], 9)                       # keys 1,2:  count 2, last 9
    ix.touch(np.array([1, 1, 1, 99], dtype=np.uint64), 3)   # key 1: count 5, last stays 9; 99 absent
    assert list(ix.select_victims(2, 100)[0]) == [3, 4, 5, 6, 7, 8, 9, 10]   # count < 2
    assert list(ix.select_victims(2, 8)[0]) == [3, 4, 5, 6, 7, 8, 9, 10]     # ... and last < 8
    assert list(ix.select_victims(2, 7)[0]) == [5, 6, 7, 8, 9, 10]           # last 7 is not before 7
    assert list(ix.select_victims(6, 10)[0]) == list(k)
    assert list(ix.select_victims(5, 10)[0]) == list(k[1:])                  # key 1 has count 5
    ix.age()                                 # 5,2,1,1 -> 2,1,0,0
    assert list(ix.select_victims(2, 10)[0]) == list(k[1:])
    ix.age()
    assert list(ix.select_victims(1, 10)[0]) == list(k[1:])
    ix.age()
    assert list(ix.select_victims(1, 10)[0]) == list(k)
    # upsert keeps usage, evict + insert resets it
    ix.touch(k[:1], 20)
    ix.insert(k[:1], np.array([1234], dtype=np.uint64))
    assert 1 not in list(ix.select_victims(1, 20)[0])
    ix.evict(k[:1])
    ix.insert(k[:1], np.array([1], dtype=np.uint64))
    assert 1 in list(ix.select_victims(1, 1)[0])
    # saturation
    ix.touch(np.full(300, 2, dtype=np.uint64), 1)
    assert 2 in list(ix.select_victims(256, 100)[0]) and 2 not in list(ix.select_victims(255, 100)[0])


def test_random_sequences_against_a_dict_model():
    rng = np.random.default_rng(0)
    ix = oracle.Index(256)
    model = {}                               # key -> [value, count, last]
    universe = np.arange(1, 400, dtype=np.uint64)
    for step in range(300):
        op = rng.integers(0, 6)
        k = rng.choice(universe, size=rng.integers(0, 30), replace=(op == 2))
        if op == 0:
            v = rng.integers(0, 1000, size=len(k), dtype=np.uint64)
            ix.insert(k, v)
            for kk, vv in zip(k, v):
                if int(kk) in model:
                    model[int(kk)][0] = int(vv)
                elif len(model) < 256:
                    model[int(kk)] = [int(vv), 0, 0]
        elif op == 1:
            ix.evict(k)
            for kk in k:
                model.pop(int(kk), None)
        elif op == 2:
            e = int(rng.integers(0, 50))
            ix.touch(k, e)
            for kk in k:
                if int(kk) in model:
                    m = model[int(kk)]
                    m[1] = min(m[1] + 1, 255)
                    m[2] = max(m[2], e)
        elif op == 3 and step % 7 == 0:
            ix.age()
            for m in model.values():
                m[1] >>= 1
        else:
            pc, be = int(rng.integers(0, 5)), int(rng.integers(0, 60))
            vk, vv = ix.select_victims(pc, be)
            want = sorted(kk for kk, m in model.items() if m[1] < pc and m[2] < be)
            assert [int(x) for x in vk] == want
            assert [int(x) for x in vv] == [model[kk][0] for kk in want]


def test_a_one_off_scan_does_not_push_out_reused_blocks():
    ix = oracle.Index(1 << 12)
    hot = np.arange(1, 201, dtype=np.uint64)                 # a shared system prompt, reused every epoch
    ix.insert(hot, hot)
    epoch = 1
    for epoch in range(1, 6):
        ix.touch(hot, epoch)
    scan = np.arange(1000, 3000, dtype=np.uint64)            # one long request, seen once
    ix.insert(scan, scan)
    ix.touch(scan, 6)
    ix.touch(hot, 7)
    vk, _ = ix.select_victims(2, 8)                          # cold = touched at most once, older than now
    assert np.array_equal(vk, scan)
    # plain recency (protect everything younger than epoch 7) would have kept the scan instead
    lru_k, _ = ix.select_victims(256, 6)
    assert len(lru_k) == 0
