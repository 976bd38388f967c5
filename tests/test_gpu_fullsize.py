"""Parity at the workloads' full sizes, in the launch configuration the benchmark times: index
and match outputs are compared whole; page copies are checked on sampled entries that the oracle
recomputes one by one from the same input bytes, plus whole-pool checksums (exact integer sums)
for the gather -> scatter identity."""
import gc

import numpy as np
import pytest

import oracle
from backends import HipIndex, hip_hash_match
from workloads import Geometry, fill_pool_torch, filler_keys, make_workload

pytestmark = pytest.mark.gpu
NO = np.uint64(0xFFFFFFFFFFFFFFFF)


def _free():
    import torch
    gc.collect()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_index_and_match_full_size(cfg):
    wl = make_workload(cfg, "full")
    h = oracle.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, 0)
    n_idx = wl.n_blocks if wl.preload_requests is None else int(wl.blk_off[wl.preload_requests])
    uniq, inv = np.unique(h[:n_idx], return_inverse=True)
    vals = np.arange(len(uniq), dtype=np.uint64)[inv]
    gi, oi = HipIndex(wl.n_slots), oracle.Index(wl.n_slots)
    n_fill = max(0, wl.n_live_target - len(uniq))
    fk, fv = filler_keys(cfg, n_fill) if n_fill else (np.zeros(0, np.uint64), np.zeros(0, np.uint64))
    for ix in (gi, oi):
        ix.insert(h[:n_idx], vals)
        if n_fill:
            ix.insert(fk, fv)
    assert np.array_equal(gi.counters_insert, oi.counters_insert)
    rng = np.random.default_rng(cfg)
    ev = np.concatenate([uniq[rng.random(len(uniq)) < 0.15], fk[: len(fk) // 50]])
    assert np.array_equal(gi.evict(ev), oi.evict(ev))
    gv, gm = gi.match(h, wl.blk_off)
    ov, om = oi.match(h, wl.blk_off)
    assert np.array_equal(gv, ov) and np.array_equal(gm, om)
    assert gi.count() == oi.count()
    gk, gvv = gi.dump()
    ok, ovv = oi.dump()
    assert np.array_equal(gk, ok) and np.array_equal(gvv, ovv)
    assert np.array_equal(gi.counters_evict, oi.counters_evict)
    # the one-launch path on the same index state
    fh, fv, fm = hip_hash_match(gi, wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, 0)
    assert np.array_equal(fh, h) and np.array_equal(fv, ov) and np.array_equal(fm, om)
    # eviction policy at the full table size: every request touches its blocks in its own epoch
    for r in range(0, wl.n_req, max(1, wl.n_req // 64)):
        blk = h[wl.blk_off[r]:wl.blk_off[r + 1]]
        gi.touch(blk, r + 1)
        oi.touch(blk, r + 1)
    for pc, be in [(2, wl.n_req // 2 + 1), (1, 1)]:
        gk2, gv2 = gi.select_victims(pc, be)
        ok2, ov2 = oi.select_victims(pc, be)
        assert np.array_equal(gk2, ok2) and np.array_equal(gv2, ov2)
    gi.age()
    oi.age()
    gk2, _ = gi.select_victims(1, 1 << 20)
    ok2, _ = oi.select_victims(1, 1 << 20)
    assert np.array_equal(gk2, ok2)
    del gi
    _free()


def _plane_sums(torch, pool, g):
    return pool.view(torch.int64).view(g.n_seg, -1).sum(dim=1)


@pytest.mark.parametrize("cfg,layout", [(1, None), (2, None), (2, "page-major"), (3, None), (4, None),
                                        (5, None)])
def test_copy_full_size_sampled(cfg, layout):
    import torch
    import paper_2504_03648_amd as aibx
    wl = make_workload(cfg, "full", layout=layout)
    g = wl.geom
    n = min(wl.batch_pages, g.n_pages)
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device="cuda")
    fill_pool_torch(pool, wl.kv_dtype, cfg)
    staging = torch.full((n * g.blk_bytes,), 0x5A, dtype=torch.uint8, device="cuda")
    desc = aibx.make_pool_desc(pool, *g.as_tuple())
    rng = np.random.default_rng(100 + cfg)
    pages = rng.permutation(g.n_pages)[:n].astype(np.int32)
    slots = rng.permutation(n).astype(np.int32)
    d_pages, d_slots = torch.from_numpy(pages).cuda(), torch.from_numpy(slots).cuda()
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    sums0 = _plane_sums(torch, pool, g)
    planes = pool.view(g.n_seg, g.n_pages, g.seg_bytes)
    st2 = staging.view(n, g.blk_bytes)
    # sampled entries: first, last and random ones
    K = 24
    sample = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=K)]))
    d_sp = torch.from_numpy(pages[sample].astype(np.int64)).cuda()
    d_ss = torch.from_numpy(slots[sample].astype(np.int64)).cuda()
    cg = Geometry(g.n_seg, g.seg_bytes, len(sample))                  # compact host pool of the sample
    host_pool = planes[:, d_sp, :].contiguous().cpu().numpy().reshape(-1)

    aibx.aibx_kv_gather(desc, d_pages, d_slots, n, staging, g.blk_bytes, bad)
    torch.cuda.synchronize()
    want = np.zeros(len(sample) * g.blk_bytes, dtype=np.uint8)
    assert oracle.kv_gather(host_pool, cg.as_tuple(), np.arange(len(sample), dtype=np.int32), None, want,
                            g.blk_bytes) == 0
    got = st2[d_ss].cpu().numpy().reshape(-1)
    assert np.array_equal(got, want)
    assert torch.equal(_plane_sums(torch, pool, g), sums0)            # gather leaves the pool alone

    planes[:, torch.from_numpy(pages.astype(np.int64)).cuda(), :] = 0xA5     # canary over the moved pages
    assert not torch.equal(_plane_sums(torch, pool, g), sums0)
    aibx.aibx_kv_scatter(desc, d_pages, d_slots, n, staging, g.blk_bytes, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    canary_pool = np.full(cg.pool_bytes, 0xA5, dtype=np.uint8)
    assert oracle.kv_scatter(canary_pool, cg.as_tuple(), np.arange(len(sample), dtype=np.int32), None, got,
                             g.blk_bytes) == 0
    after = planes[:, d_sp, :].contiguous().cpu().numpy().reshape(-1)
    assert np.array_equal(after, canary_pool) and np.array_equal(after, host_pool)
    assert torch.equal(_plane_sums(torch, pool, g), sums0)            # scatter(gather) = identity
    del pool, staging, planes, st2
    _free()


def test_converting_copy_full_size_sampled():
    """Config 2's pool read as token-major pages, at the batch size bench.py --survey times: sampled
    blocks against the oracle, a checksum that every staged block is a permutation-free image of its
    page, and the scatter back restores the pool."""
    import torch
    import paper_2504_03648_amd as aibx
    wl = make_workload(2, "full")
    g = wl.geom
    S, T = g.n_seg, wl.block_size
    run = g.seg_bytes // T
    n = wl.batch_pages
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device="cuda")
    fill_pool_torch(pool, wl.kv_dtype, 2)
    geom = (S, T, run, g.blk_bytes, S * run, run, g.n_pages)
    rd = aibx.make_pool_runs_desc(pool, *geom)
    rng = np.random.default_rng(321)
    pages = rng.permutation(g.n_pages)[:n].astype(np.int32)
    d_pages = torch.from_numpy(pages).cuda()
    staging = torch.full((n * g.blk_bytes,), 0x5A, dtype=torch.uint8, device="cuda")
    aibx.aibx_kv_gather_runs(rd, d_pages, None, n, staging, g.blk_bytes)
    torch.cuda.synchronize()
    by_page = pool.view(g.n_pages, g.blk_bytes)
    sample = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=16)]))
    host_pool = by_page[torch.from_numpy(pages[sample].astype(np.int64)).cuda()].cpu().numpy().reshape(-1)
    cgeom = (S, T, run, g.blk_bytes, S * run, run, len(sample))
    want = np.zeros(len(sample) * g.blk_bytes, dtype=np.uint8)
    assert oracle.kv_gather_runs(host_pool, cgeom, np.arange(len(sample), dtype=np.int32), None, want, g.blk_bytes) == 0
    got = staging.view(n, g.blk_bytes)[torch.from_numpy(sample.astype(np.int64)).cuda()].cpu().numpy().reshape(-1)
    assert np.array_equal(got, want)
    # every block: the staged bytes are the page's bytes in another order (equal 64-bit word sums)
    sums_pool = by_page.view(torch.int64).view(g.n_pages, -1).sum(dim=1)[d_pages.long()]
    sums_stage = staging.view(torch.int64).view(n, -1).sum(dim=1)
    assert torch.equal(sums_pool, sums_stage)
    keep = by_page[d_pages.long()].clone()
    by_page[d_pages.long()] = 0
    aibx.aibx_kv_scatter_runs(rd, d_pages, None, n, staging, g.blk_bytes)
    torch.cuda.synchronize()
    assert torch.equal(by_page[d_pages.long()], keep)
