"""Op sequences of the five workloads, written once against a small backend protocol so that the
CPU oracle and the HIP library are driven by the same calls on the same inputs. This module only
decides WHICH keys, pages and slots each call names (bookkeeping on host arrays); the hashing,
probing and copying are done by the backend.

Backend protocol (all arrays host numpy):
  be.block_hash(tokens, tok_off, blk_off, block_size, seed) -> uint64[N]
  be.index_create(n_slots) -> ix with
      ix.insert(keys, values); ix.evict(keys) -> uint64[n]; ix.match(hashes, blk_off) ->
      (uint64[N], int32[R]); ix.count() -> int; ix.dump() -> (keys, values) sorted by key;
      ix.counters_insert (3), ix.counters_evict (2)
  be.pool_create(geom, kv_dtype, cfg); be.staging_create(n_blocks, stride)
  be.gather(page_ids, slot_ids) -> bad; be.scatter(page_ids, slot_ids) -> bad
  be.fill_pages(page_ids, byte)          (plain memset of whole pages; test plumbing)
  be.read_pages(page_ids) -> uint8[n, blk_bytes]; be.read_slots(slot_ids) -> uint8[n, blk_bytes]

Value encoding in the index: a plain page id = block lives in the HBM pool; STAGED | slot = block
was offloaded to that staging slot; ELSEWHERE | k = block is indexed but held by another tier.
"""
from __future__ import annotations

import numpy as np

from .configs import Workload, filler_keys, ops_rng

STAGED = np.uint64(1) << np.uint64(62)
ELSEWHERE = np.uint64(1) << np.uint64(61)
NO_VALUE = np.uint64(0xFFFFFFFFFFFFFFFF)
CANARY = 0xA5


def _distinct_in_order(h: np.ndarray):
    """Distinct keys by first appearance, their reference counts, and block -> rank."""
    uniq, first, inv, cnt = np.unique(h, return_index=True, return_inverse=True, return_counts=True)
    order = np.argsort(first, kind="stable")
    rank_of_uniq = np.empty(len(uniq), dtype=np.int64)
    rank_of_uniq[order] = np.arange(len(uniq))
    return uniq[order], cnt[order], rank_of_uniq[inv]


def preload_index(wl: Workload, be, h: np.ndarray):
    """Creates the index and inserts the workload's resident blocks (one call naming every block,
    duplicates included - they carry identical values) plus random filler keys up to the load
    factor. Returns (ix, dkeys, dvalues, refcnt)."""
    n_idx = wl.n_blocks if wl.preload_requests is None else int(wl.blk_off[wl.preload_requests])
    dkeys, refcnt, rank = _distinct_in_order(h[:n_idx])
    ranks = np.arange(len(dkeys), dtype=np.uint64)
    n_res = min(len(dkeys), wl.geom.n_pages)
    dvalues = ELSEWHERE | ranks
    dvalues[:n_res] = wl.page_perm[:n_res].astype(np.uint64)
    ix = be.index_create(wl.n_slots)
    ix.insert(h[:n_idx], dvalues[rank])
    n_fill = max(0, wl.n_live_target - len(dkeys))
    if n_fill:
        fk, fv = filler_keys(wl.cfg, n_fill)
        ix.insert(fk, fv)
    return ix, dkeys, dvalues, refcnt


def _batches(n: int, step: int):
    for i in range(0, n, step):
        yield i, min(n, i + step)


def flow_match_roundtrip(wl: Workload, be) -> dict:
    """Configs 1, 3, 4: hash, preload, match every request, then move every distinct matched
    resident block pool -> staging -> pool in batches; the freed pages are overwritten with a
    canary in between, so the pool ends bit-identical only if both copies are exact."""
    tr = {}
    h = be.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, wl.hash_seed)
    tr["hash"] = h
    ix, dkeys, dvalues, _ = preload_index(wl, be, h)
    values, mlen = ix.match(h, wl.blk_off)
    tr["values"], tr["match_len"] = values, mlen
    matched = np.zeros(wl.n_blocks, dtype=bool)
    for r in range(wl.n_req):
        matched[wl.blk_off[r]:wl.blk_off[r] + mlen[r]] = True
    v = values[matched]
    pages = np.unique(v[v < np.uint64(wl.geom.n_pages)]).astype(np.int32)
    pages = pages[ops_rng(wl.cfg, 1).permutation(len(pages))]
    tr["pages"] = pages
    be.pool_create(wl.geom, wl.kv_dtype, wl.cfg)
    be.staging_create(min(wl.batch_pages, max(len(pages), 1)), wl.geom.blk_bytes)
    probe = pages[:: max(1, len(pages) // 16)][:16]
    tr["before"] = be.read_pages(probe)
    staged = []
    for a, b in _batches(len(pages), wl.batch_pages):
        assert be.gather(pages[a:b], None) == 0
        be.fill_pages(pages[a:b], CANARY)
        staged.append(be.read_slots(np.arange(min(b - a, 4), dtype=np.int32)))
        assert be.scatter(pages[a:b], None) == 0
    tr["staged_samples"] = staged
    tr["after"] = be.read_pages(probe)
    tr["count"] = ix.count()
    tr["dump"] = ix.dump()
    tr["counters_insert"] = np.array(ix.counters_insert)
    return tr


def flow_offload_onload(wl: Workload, be) -> dict:
    """Config 2 (usable with any config's shapes): (1) hash and index every block; (2) gather the
    cold half of the resident blocks to staging, re-point their index values at the staging slots
    and overwrite their pool pages with a canary; (3) evict a tenth of the cold keys outright;
    (4) match every request, scatter the staged blocks that are still on a matched prefix into a
    shuffled set of the freed pages and re-point their values; (5) read everything back."""
    tr = {}
    g = wl.geom
    h = be.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, wl.hash_seed)
    tr["hash"] = h
    ix, dkeys, dvalues, refcnt = preload_index(wl, be, h)
    be.pool_create(g, wl.kv_dtype, wl.cfg)
    # (2) cold half: smallest (reference count, then key) among resident blocks
    res = np.flatnonzero(dvalues < np.uint64(g.n_pages))
    cold = res[np.lexsort((dkeys[res], refcnt[res]))][: len(res) // 2]
    cold_keys, cold_pages = dkeys[cold], dvalues[cold].astype(np.int32)
    tr["cold_keys"] = cold_keys
    n_cold = len(cold)
    be.staging_create(max(n_cold, 1), g.blk_bytes)
    original = {}
    sample = np.arange(0, n_cold, max(1, n_cold // 24))
    for i, blk in zip(sample, be.read_pages(cold_pages[sample])):
        original[int(i)] = blk
    slots = np.arange(n_cold, dtype=np.int32)
    for a, b in _batches(n_cold, wl.batch_pages):
        assert be.gather(cold_pages[a:b], slots[a:b]) == 0
    ix.insert(cold_keys, STAGED | slots.astype(np.uint64))
    be.fill_pages(cold_pages, CANARY)
    tr["staged"] = be.read_slots(slots[sample])
    # (3) drop 10 % of the cold keys from the cache altogether
    rng = ops_rng(wl.cfg, 2)
    dropped = cold_keys[rng.permutation(n_cold)[: n_cold // 10]]
    tr["evicted_values"] = ix.evict(dropped)
    # (4) match, then onload what is staged and on a matched prefix
    values, mlen = ix.match(h, wl.blk_off)
    tr["values"], tr["match_len"] = values, mlen
    on_prefix = np.zeros(wl.n_blocks, dtype=bool)
    for r in range(wl.n_req):
        on_prefix[wl.blk_off[r]:wl.blk_off[r] + mlen[r]] = True
    want = on_prefix & (values != NO_VALUE) & ((values & STAGED) != 0) & ((values >> np.uint64(63)) == 0)
    on_keys, first = np.unique(h[want], return_index=True)
    on_slots = (values[want][first] & ~STAGED).astype(np.int32)
    new_pages = cold_pages[rng.permutation(n_cold)[: len(on_keys)]]
    tr["onload_slots"], tr["onload_pages"] = on_slots, new_pages
    for a, b in _batches(len(on_keys), wl.batch_pages):
        assert be.scatter(new_pages[a:b], on_slots[a:b]) == 0
    ix.insert(on_keys, new_pages.astype(np.uint64))
    # (5) observable end state
    k = max(1, len(on_keys) // 24)
    tr["onloaded"] = be.read_pages(new_pages[::k])
    tr["onloaded_from"] = be.read_slots(on_slots[::k])
    left = np.setdiff1d(cold_pages, new_pages)
    tr["still_canary"] = be.read_pages(left[:: max(1, len(left) // 8)][:8])
    tr["original_of_sample"] = original
    tr["sample"] = sample
    tr["count"] = ix.count()
    tr["dump"] = ix.dump()
    tr["counters_insert"] = np.array(ix.counters_insert)
    tr["counters_evict"] = np.array(ix.counters_evict)
    return tr


def flow_stress(wl: Workload, be, n_rounds: int = 8, q: int = 4096, extra_tokens=None,
                page_span=None) -> dict:
    """Config 5: after the preload, rounds of {insert q new keys, evict the q oldest live real
    keys, probe about 4q block hashes}, while disjoint page batches are gathered and scattered
    (the backend may run those two on separate streams via be.gather_scatter_pair).
    extra_tokens = (tokens, tok_off, blk_off) of further requests of the same mix: their block
    hashes extend the supply of keys when n_rounds*q exceeds the batch's own distinct blocks.
    page_span: the copies use only this many pages of the pool (the first of a seeded permutation)
    and go round them again and again in batches of wl.batch_pages; by default every round takes
    fresh pages."""
    tr = {"round_values": [], "round_match_len": [], "round_evicted": []}
    g = wl.geom
    h = be.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, wl.hash_seed)
    tr["hash"] = h
    supply = h
    if extra_tokens is not None:
        h2 = be.block_hash(*extra_tokens, wl.block_size, wl.hash_seed)
        tr["hash_extra"] = h2
        supply = np.concatenate([h, h2])
    dkeys, _, rank = _distinct_in_order(supply)
    n_keys = len(dkeys)
    n_pre = max(0, n_keys - n_rounds * q)              # the tail is inserted round by round
    dvalues = ELSEWHERE | np.arange(n_keys, dtype=np.uint64)
    n_res = min(n_keys, g.n_pages)
    dvalues[:n_res] = wl.page_perm[:n_res].astype(np.uint64)
    ix = be.index_create(wl.n_slots)
    ix.insert(dkeys[:n_pre], dvalues[:n_pre])
    n_fill = max(0, wl.n_live_target - n_pre)
    if n_fill:
        ix.insert(*filler_keys(wl.cfg, n_fill))
    be.pool_create(g, wl.kv_dtype, wl.cfg)
    rng = ops_rng(wl.cfg, 3)
    page_order = rng.permutation(g.n_pages).astype(np.int32)
    if page_span is None:
        bp = min(wl.batch_pages, g.n_pages // (2 * n_rounds))
    else:
        page_order = page_order[:page_span]
        bp = min(wl.batch_pages, page_span // 2)
    span = len(page_order)
    be.staging_create(2 * bp, g.blk_bytes)
    req_order = rng.permutation(wl.n_req)
    probe_ptr, ins_ptr, ev_ptr = 0, n_pre, 0
    for t in range(n_rounds):
        a = ins_ptr
        ins_ptr = min(n_keys, ins_ptr + q)
        ix.insert(dkeys[a:ins_ptr], dvalues[a:ins_ptr])
        ev = dkeys[ev_ptr: ev_ptr + q]
        ev_ptr += len(ev)
        tr["round_evicted"].append(ix.evict(ev))
        # probe whole requests until about 4q blocks are named
        rs, nb = [], 0
        while nb < 4 * q and len(rs) < wl.n_req:
            r = int(req_order[probe_ptr % wl.n_req])
            probe_ptr += 1
            rs.append(r)
            nb += int(wl.blk_off[r + 1] - wl.blk_off[r])
        hp = np.concatenate([h[wl.blk_off[r]:wl.blk_off[r + 1]] for r in rs])
        bo = np.zeros(len(rs) + 1, dtype=np.int64)
        np.cumsum([wl.blk_off[r + 1] - wl.blk_off[r] for r in rs], out=bo[1:])
        v, m = ix.match(hp, bo)
        tr["round_values"].append(v)
        tr["round_match_len"].append(m)
        # copies: gather batch 2t into staging half A while staging half B is scattered over
        # batch 2t+1 (disjoint pages, disjoint slots)
        ga = np.take(page_order, np.arange((2 * t) * bp, (2 * t + 1) * bp), mode="wrap")
        sb = np.take(page_order, np.arange((2 * t + 1) * bp, (2 * t + 2) * bp), mode="wrap")
        slots_a = np.arange(bp, dtype=np.int32)
        slots_b = np.arange(bp, 2 * bp, dtype=np.int32)
        if t == 0:
            assert be.gather(sb[::-1].copy(), slots_b) == 0    # give half B defined contents
        bad = be.gather_scatter_pair(ga, slots_a, sb, slots_b)
        assert tuple(bad) == (0, 0)
    used = min(span, 2 * bp * n_rounds)
    tr["final_pages"] = be.read_pages(page_order[:used: max(1, used // 32)])
    tr["final_slots"] = be.read_slots(np.arange(0, 2 * bp, max(1, (2 * bp) // 16), dtype=np.int32))
    tr["count"] = ix.count()
    tr["dump"] = ix.dump()
    tr["counters_insert"] = np.array(ix.counters_insert)
    tr["counters_evict"] = np.array(ix.counters_evict)
    return tr


def traces_equal(a, b, path="") -> list:
    """Element-by-element comparison of two flow traces; returns the list of differing paths."""
    bad = []
    if isinstance(a, dict):
        if set(a) != set(b):
            return [f"{path}: keys {sorted(set(a) ^ set(b))}"]
        for k in a:
            bad += traces_equal(a[k], b[k], f"{path}/{k}")
    elif isinstance(a, (list, tuple)):
        if len(a) != len(b):
            return [f"{path}: length {len(a)} != {len(b)}"]
        for i, (x, y) in enumerate(zip(a, b)):
            bad += traces_equal(x, y, f"{path}[{i}]")
    else:
        x, y = np.asarray(a), np.asarray(b)
        if x.shape != y.shape or x.dtype != y.dtype or not np.array_equal(x, y):
            bad.append(f"{path}: arrays differ")
    return bad
