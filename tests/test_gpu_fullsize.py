"""Parity at the workloads' full sizes, in the launch configuration the benchmark times: index
and match outputs are compared whole; page copies are compared with the oracle plane by plane
(every entry of the batch on whole planes, every plane on sampled entries) and byte for byte on
the device against an independent index_select; the offload/onload flow of the 8B-shaped
workload and the insert/evict/probe rounds with two-stream copies of the stress workload run
against the oracle at the full index, batch and pool sizes."""
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
    # the routing decision straight from the tokens, values read as pod sets, at the batch's full size
    import torch
    import paper_2504_03648_amd as aibx
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    load = rng.integers(0, 4, size=8).astype(np.int32)
    pod = torch.full((wl.n_req,), -9, dtype=torch.int32, device="cuda")
    hit = torch.full((wl.n_req,), -9, dtype=torch.int32, device="cuda")
    for num, den in ((1, 2), (0, 1)):
        want_pod, want_hit = oracle.route(ov, wl.blk_off, 8, load, num, den)
        aibx.aibx_hash_match_route(gi.h, d(wl.tokens), d(wl.tok_off), d(wl.blk_off), wl.n_req, wl.n_blocks,
                                   wl.block_size, 0, 8, d(load), num, den, pod, hit)
        assert np.array_equal(pod.cpu().numpy(), want_pod) and np.array_equal(hit.cpu().numpy(), want_hit)
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


def _whole_planes(g, rng):
    """Planes compared whole, every entry of the batch: the first, the last and two random ones."""
    return sorted(set([0, g.n_seg - 1] + [int(x) for x in rng.integers(0, g.n_seg, size=2)]))


@pytest.mark.parametrize("cfg,layout", [(1, None), (2, None), (2, "page-major"), (3, None), (4, None),
                                        (5, None)])
def test_copy_full_size_every_entry(cfg, layout):
    """One gather and one scatter batch at the workload's full pool size, in the launch shape the
    benchmark times. Compared with the oracle: (a) EVERY entry of the batch on whole planes, plane
    by plane - the plane and the matching strided slice of the staging buffer are fetched with
    plain device-to-host copies and the oracle moves that plane's segments on the host; (b) every
    plane on sampled entries. Compared on the device, with torch's index_select as an independent
    reference: (c) every byte of the batch, all planes, and that nothing else in the pool moved."""
    import torch
    import paper_2504_03648_amd as aibx
    wl = make_workload(cfg, "full", layout=layout)
    g = wl.geom
    n = min(wl.batch_pages, g.n_pages)
    G = 4096                                                             # canary bytes around both buffers
    pool_buf = torch.full((g.pool_bytes + 2 * G,), 0xC3, dtype=torch.uint8, device="cuda")
    pool = pool_buf[G:G + g.pool_bytes]
    fill_pool_torch(pool, wl.kv_dtype, cfg)
    st_buf = torch.full((n * g.blk_bytes + 2 * G,), 0xC3, dtype=torch.uint8, device="cuda")
    staging = st_buf[G:G + n * g.blk_bytes]
    staging.fill_(0x5A)
    desc = aibx.make_pool_desc(pool, *g.as_tuple())
    rng = np.random.default_rng(100 + cfg)
    pages = rng.permutation(g.n_pages)[:n].astype(np.int32)
    slots = rng.permutation(n).astype(np.int32)
    d_pages, d_slots = torch.from_numpy(pages).cuda(), torch.from_numpy(slots).cuda()
    lp, ls = d_pages.long(), d_slots.long()
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    sums0 = _plane_sums(torch, pool, g)
    planes = pool.view(g.n_seg, g.n_pages, g.seg_bytes)
    st3 = staging.view(n, g.n_seg, g.seg_bytes)
    whole = _whole_planes(g, rng)
    one_plane = Geometry(1, g.seg_bytes, g.n_pages)                     # a plane seen as a pool of its own
    host_planes = {s: planes[s].cpu().numpy().reshape(-1) for s in whole}
    print(f"  cfg {cfg} {g.layout}: {n} entries; whole planes {whole} of {g.n_seg} "
          f"({len(whole) * one_plane.pool_bytes / 2**30:.2f} GiB on the host), staging {n * g.blk_bytes / 2**30:.2f} GiB",
          flush=True)
    # sampled entries, every plane: first, last and random ones
    sample = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=24)]))
    d_sp = torch.from_numpy(pages[sample].astype(np.int64)).cuda()
    d_ss = torch.from_numpy(slots[sample].astype(np.int64)).cuda()
    cg = Geometry(g.n_seg, g.seg_bytes, len(sample))                    # compact host pool of the sample
    host_pool = planes[:, d_sp, :].contiguous().cpu().numpy().reshape(-1)

    aibx.aibx_kv_gather(desc, d_pages, d_slots, n, staging, g.blk_bytes, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    for s in whole:                                                      # (a) every entry, plane by plane
        want = np.full(n * g.seg_bytes, 0x5A, dtype=np.uint8)
        assert oracle.kv_gather(host_planes[s], one_plane.as_tuple(), pages, slots, want, g.seg_bytes) == 0
        got = st3[:, s, :].cpu().numpy().reshape(-1)
        assert np.array_equal(got, want), f"gather, plane {s}"
    want = np.zeros(len(sample) * g.blk_bytes, dtype=np.uint8)           # (b) sampled entries, all planes
    assert oracle.kv_gather(host_pool, cg.as_tuple(), np.arange(len(sample), dtype=np.int32), None, want,
                            g.blk_bytes) == 0
    got = staging.view(n, g.blk_bytes)[d_ss].cpu().numpy().reshape(-1)
    assert np.array_equal(got, want)
    for s in range(g.n_seg):                                             # (c) every byte, on the device
        assert torch.equal(st3[:, s, :].index_select(0, ls), planes[s].index_select(0, lp)), f"gather, plane {s}"
    assert torch.equal(_plane_sums(torch, pool, g), sums0)               # gather leaves the pool alone

    planes[:, lp, :] = 0xA5                                              # canary over the moved pages
    assert not torch.equal(_plane_sums(torch, pool, g), sums0)
    aibx.aibx_kv_scatter(desc, d_pages, d_slots, n, staging, g.blk_bytes, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    for s in whole:                                                      # (a) the whole plane after the scatter
        want_plane = host_planes[s].copy()
        want_plane.reshape(g.n_pages, g.seg_bytes)[pages.astype(np.int64)] = 0xA5
        stage_s = st3[:, s, :].cpu().numpy().reshape(-1)
        assert oracle.kv_scatter(want_plane, one_plane.as_tuple(), pages, slots, stage_s, g.seg_bytes) == 0
        assert np.array_equal(planes[s].cpu().numpy().reshape(-1), want_plane), f"scatter, plane {s}"
        assert np.array_equal(want_plane, host_planes[s])                # which is the plane it started as
    canary_pool = np.full(cg.pool_bytes, 0xA5, dtype=np.uint8)           # (b)
    assert oracle.kv_scatter(canary_pool, cg.as_tuple(), np.arange(len(sample), dtype=np.int32), None, got,
                             g.blk_bytes) == 0
    after = planes[:, d_sp, :].contiguous().cpu().numpy().reshape(-1)
    assert np.array_equal(after, canary_pool) and np.array_equal(after, host_pool)
    for s in range(g.n_seg):                                             # (c)
        assert torch.equal(planes[s].index_select(0, lp), st3[:, s, :].index_select(0, ls)), f"scatter, plane {s}"
    assert torch.equal(_plane_sums(torch, pool, g), sums0)               # scatter(gather) = identity
    for buf in (pool_buf, st_buf):                                       # nothing written outside the buffers
        assert bool((buf[:G] == 0xC3).all()) and bool((buf[-G:] == 0xC3).all())
    del pool, staging, planes, st3, pool_buf, st_buf, host_planes
    _free()


def test_converting_copy_full_size_every_entry():
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
    # every block, every byte, on the device: torch's own transpose of the token-major pages
    for a in range(0, n, 1024):
        ids = d_pages[a:a + 1024].long()
        ref = by_page[ids].view(len(ids), T, S, run).permute(0, 2, 1, 3).contiguous().view(len(ids), -1)
        assert torch.equal(staging.view(n, g.blk_bytes)[a:a + 1024], ref)
    # whole segments of every entry against the oracle: segment s of all pages, fetched with plain copies
    for sgm in (0, S - 1, int(rng.integers(0, S))):
        seg_pool = by_page.view(g.n_pages, T, S, run)[:, :, sgm, :].contiguous().cpu().numpy().reshape(-1)
        sgeom = (1, T, run, T * run, run, run, g.n_pages)               # that segment alone, token-major
        want = np.zeros(n * g.seg_bytes, dtype=np.uint8)
        assert oracle.kv_gather_runs(seg_pool, sgeom, pages, None, want, g.seg_bytes) == 0
        got = staging.view(n, S, g.seg_bytes)[:, sgm, :].cpu().numpy().reshape(-1)
        assert np.array_equal(got, want), f"segment {sgm}"
    keep = by_page[d_pages.long()].clone()
    by_page[d_pages.long()] = 0
    aibx.aibx_kv_scatter_runs(rd, d_pages, None, n, staging, g.blk_bytes)
    torch.cuda.synchronize()
    assert torch.equal(by_page[d_pages.long()], keep)


# ---- whole flows at full size ------------------------------------------------------------------
def _page_sums(torch, hb):
    """Exact 64-bit word sums of every (plane, page) of the device pool."""
    g = hb.geom
    return hb.pool.view(torch.int64).view(g.n_seg, g.n_pages, -1).sum(dim=2)


def _compare_flow_end_state(torch, ob, hb, sums0):
    """Every page the flow named, byte for byte against the oracle's compact pool; every page it
    did not name still has its checksum; the whole staging buffer; the guard regions."""
    named = np.sort(ob.named_pages())
    for a in range(0, len(named), 1024):
        part = named[a:a + 1024]
        assert np.array_equal(hb.read_pages(part), ob.read_pages(part)), f"pages {a}.."
    sums1 = _page_sums(torch, hb)
    untouched = torch.ones(hb.geom.n_pages, dtype=torch.bool, device="cuda")
    untouched[torch.from_numpy(named).cuda()] = False
    assert torch.equal(sums0[:, untouched], sums1[:, untouched])
    step = 1 << 30
    for a in range(0, hb.staging.numel(), step):
        assert np.array_equal(hb.staging[a:a + step].cpu().numpy(), ob.staging[a:a + step]), f"staging byte {a}.."
    hb.check_guards()
    return len(named)


def test_flow_offload_onload_full_size():
    """The 8B-shaped workload's five steps at full size (64 x 4096 tokens, 2^20-slot index at load
    0.5, 20,000-page pool of 2 MiB blocks in 64 planes, one gather of the 4,608 cold blocks): every
    trace entry, the final index, every named page, the whole staging buffer and the untouched rest
    of the pool against the oracle. The oracle holds the named pages only (9 GiB of the 39 GiB)."""
    import torch
    from backends import CompactOracleBackend, HipBackend
    from workloads import flows
    wl = make_workload(2, "full")
    hb = HipBackend(device_fill=True)
    hb.pool_create(wl.geom, wl.kv_dtype, wl.cfg)
    sums0 = _page_sums(torch, hb)
    ob = CompactOracleBackend(fetch=hb.read_pages, capacity=4608 + 64)
    a = flows.flow_offload_onload(wl, ob)            # first: it fetches the pages it names while they are pristine
    b = flows.flow_offload_onload(wl, hb)
    assert flows.traces_equal(a, b) == []
    assert len(a["cold_keys"]) == 4608 and 0 < len(a["onload_slots"]) < 4608
    n_named = _compare_flow_end_state(torch, ob, hb, sums0)
    print(f"  {n_named} named pages ({n_named * wl.geom.blk_bytes / 2**30:.1f} GiB) and "
          f"{hb.staging.numel() / 2**30:.1f} GiB of staging compared whole", flush=True)
    del hb, ob
    _free()


def test_flow_stress_full_size_two_streams():
    """The stress workload at full size: 1,024 requests (216 k blocks), 2^24-slot index at load
    0.75, 64 rounds of {insert 4,096 new keys, evict the 4,096 oldest, probe about 16 k blocks},
    each round with a 4,096-page gather and a 4,096-page scatter in flight on two streams in the
    full 131,072-page pool (1 MiB blocks in 64 planes). The copies go round 16,384 of the pool's
    pages, which is what the oracle mirrors on the host (16 GiB + 8 GiB of staging); the key
    supply beyond the batch's own blocks comes from a second draw of the same request mix."""
    import torch
    from backends import CompactOracleBackend, HipBackend
    from workloads import flows
    from workloads.configs import make_tokens
    wl = make_workload(5, "full")
    extra = make_tokens(5, 1)
    span, rounds, q = 16384, 64, 4096
    hb = HipBackend(two_streams=True, device_fill=True)
    hb.pool_create(wl.geom, wl.kv_dtype, wl.cfg)
    sums0 = _page_sums(torch, hb)
    ob = CompactOracleBackend(fetch=hb.read_pages, capacity=span)
    a = flows.flow_stress(wl, ob, n_rounds=rounds, q=q, extra_tokens=extra, page_span=span)
    print("  oracle flow done", flush=True)
    b = flows.flow_stress(wl, hb, n_rounds=rounds, q=q, extra_tokens=extra, page_span=span)
    assert flows.traces_equal(a, b) == []
    ins, upd, full = [int(x) for x in a["counters_insert"]]
    assert full == 0 and ins >= wl.n_live_target + rounds * q - q
    assert all(len(e) == q for e in a["round_evicted"]) and int(a["counters_evict"][1]) == 0
    n_named = _compare_flow_end_state(torch, ob, hb, sums0)
    assert n_named == span
    del hb, ob
    _free()
