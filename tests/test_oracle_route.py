"""Pins for the oracle's routing decision: hand-worked cases, threshold and fallback rules, and
agreement with matching against one index per pod."""
import numpy as np
import pytest

import oracle

NO = np.uint64(0xFFFFFFFFFFFFFFFF)


def _sets(*bits):
    return np.array([NO if b is None else np.uint64(b) for b in bits], dtype=np.uint64)


def test_hand_worked_cases():
    # 3 pods. request 0: blocks held by {0,1}, {1}, {1,2}, {}  -> pod 1 holds 3 of 4
    # request 1: {2}, {2}, {0}                                  -> pod 2 holds 2 of 3
    # request 2: nothing cached                                 -> fallback
    # request 3: zero blocks                                    -> fallback
    sets = _sets(0b011, 0b010, 0b110, None, 0b100, 0b100, 0b001, None, 0b000)
    blk_off = [0, 4, 7, 9, 9]
    load = [5, 9, 1]
    pod, hit = oracle.route(sets, blk_off, 3, load, 1, 2)            # threshold 1/2
    assert list(pod) == [1, 2, 2, 2] and list(hit) == [3, 2, 0, 0]
    pod, hit = oracle.route(sets, blk_off, 3, load, 3, 4)            # 3/4: request 1 (2/3) falls back
    assert list(pod) == [1, 2, 2, 2] and list(hit) == [3, 2, 0, 0]   # least-loaded pod 2 happens to hold 2
    load = [0, 9, 1]
    pod, hit = oracle.route(sets, blk_off, 3, load, 3, 4)
    assert list(pod) == [1, 0, 0, 0] and list(hit) == [3, 0, 0, 0]
    pod, hit = oracle.route(sets, blk_off, 3, load, 5, 4)            # threshold above 1: always least-request
    assert list(pod) == [0, 0, 0, 0] and list(hit) == [1, 0, 0, 0]


def test_ties_go_to_the_less_loaded_then_lower_pod():
    sets = _sets(0b1111, 0b1110, 0b0110)          # pods 1 and 2 hold all three blocks
    pod, hit = oracle.route(sets, [0, 3], 4, [0, 7, 7, 0], 0, 1)
    assert list(pod) == [1] and list(hit) == [3]
    pod, hit = oracle.route(sets, [0, 3], 4, [0, 7, 6, 0], 0, 1)
    assert list(pod) == [2] and list(hit) == [3]


def test_agrees_with_one_index_per_pod():
    """len_p is the first-miss match length against an index holding only pod p's blocks."""
    rng = np.random.default_rng(0)
    n_pods, n_req = 5, 40
    sizes = rng.integers(0, 30, size=n_req)
    blk_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(sizes, out=blk_off[1:])
    n = int(blk_off[-1])
    keys = np.arange(1, n + 1, dtype=np.uint64)
    sets = rng.integers(0, 1 << n_pods, size=n).astype(np.uint64) | np.uint64(0b00100) * (rng.random(n) < 0.7)
    sets[rng.random(n) < 0.05] = NO
    per_pod = []
    for p in range(n_pods):
        ix = oracle.Index(1 << 12)
        held = (sets != NO) & ((sets >> np.uint64(p)) & np.uint64(1) == 1)
        ix.insert(keys[held], keys[held])
        per_pod.append(ix.match(keys, blk_off)[1])
    per_pod = np.array(per_pod)                                   # [pod, request]
    load = rng.integers(0, 4, size=n_pods).astype(np.int32)
    for num, den in [(0, 1), (1, 2), (1, 1)]:
        pod, hit = oracle.route(sets, blk_off, n_pods, load, num, den)
        best = per_pod.max(axis=0)
        for r in range(n_req):
            assert hit[r] == per_pod[pod[r], r]
            aware = sizes[r] > 0 and best[r] > 0 and best[r] * den >= num * sizes[r]
            cand = np.flatnonzero(per_pod[:, r] == best[r]) if aware else np.arange(n_pods)
            want = min(cand, key=lambda p: (load[p], p))
            assert pod[r] == want


def test_invalid_arguments():
    with pytest.raises(ValueError):
        oracle.route(_sets(1), [0, 1], 64, [0] * 64, 1, 2)
    with pytest.raises(ValueError):
        oracle.route(_sets(1), [0, 1], 1, [0], 1, 0)
