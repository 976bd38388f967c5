#!/usr/bin/env python3
"""Benchmark of the KV-cache hot path on one MI355X.

A step is one pass of the whole path over the Llama-3-8B-shaped workload (64 requests x 4096
tokens, 16-token blocks, 20,000-page pool of 2 MiB blocks in 64 planes, 2^20-slot index preloaded
to load 0.5): hash every request, index every block, gather the cold half of the resident blocks
to staging (offload), re-point and evict index entries, match every request, scatter the matched
staged blocks back into the pool (onload), update the index, and evict the batch's keys again so
that the next step starts from the same index. Every array the step reads is resident in HBM
before the clock starts.

Prints ONE JSON line. `value` = bytes read + written by the gathers and scatters of a step divided
by the whole step's time. `roofline` is the gather kernel against 8 TB/s. `hash_match` is the
scaled batch (the same request mix replicated until >= 4 Mi blocks) against its 152 B/block HBM
roofline. `cpu_baseline` is the CPU oracle on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
STAGED = np.uint64(1) << np.uint64(62)
NO_VALUE = np.uint64(0xFFFFFFFFFFFFFFFF)

# HBM bytes per gather launch from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by the same
# counters on a plain copy of known size; valid only for the kernel source it was taken on.
MEASURED_TRAFFIC = {"kvcopy_sha1": "20f0afe104144a6cf0209e213c9b28adfa0c9a1e",
                    "bytes_per_launch": 19327179779}


def _u64(t):
    return t.cpu().numpy().view(np.uint64)


def _dev_u64(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64).copy()).cuda()


def _kvcopy_sha1():
    p = os.path.join(ROOT, "paper_2504_03648_amd", "csrc", "kvcopy.hip")
    return hashlib.sha1(open(p, "rb").read()).hexdigest()


class Step:
    """Device-resident state and the call sequence of one step."""

    def __init__(self, torch, aibx, wl):
        from workloads import fill_pool_torch, filler_keys
        from workloads.configs import ops_rng
        self.t, self.a, self.wl = torch, aibx, wl
        g = wl.geom
        dev = "cuda"
        self.tokens = torch.from_numpy(wl.tokens).to(dev)
        self.tok_off = torch.from_numpy(wl.tok_off).to(dev)
        self.blk_off = torch.from_numpy(wl.blk_off).to(dev)
        self.N, self.R = wl.n_blocks, wl.n_req
        self.hash = torch.empty(self.N, dtype=torch.int64, device=dev)
        self.values = torch.empty(self.N, dtype=torch.int64, device=dev)
        self.mlen = torch.empty(self.R, dtype=torch.int32, device=dev)
        self.ev_out = None
        self.ev_g0 = self.ev_g1 = None
        self.pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=dev)
        fill_pool_torch(self.pool, wl.kv_dtype, wl.cfg)
        self.desc = aibx.make_pool_desc(self.pool, *g.as_tuple())
        self.storage = torch.empty(aibx.aibx_index_storage_bytes(wl.n_slots), dtype=torch.uint8, device=dev)
        self.ix = aibx.aibx_index_create(self.storage, wl.n_slots)
        self.counters = torch.zeros(8, dtype=torch.int64, device=dev)
        # ---- untimed planning pass: which keys / pages / slots each call names ----------------
        aibx.aibx_block_hash(self.tokens, self.tok_off, self.blk_off, self.R, self.N, wl.block_size,
                             wl.hash_seed, self.hash)
        h = _u64(self.hash)
        uniq, first, inv, cnt = np.unique(h, return_index=True, return_inverse=True, return_counts=True)
        order = np.argsort(first, kind="stable")
        rank_of_uniq = np.empty(len(uniq), dtype=np.int64)
        rank_of_uniq[order] = np.arange(len(uniq))
        dkeys, refcnt, rank = uniq[order], cnt[order], rank_of_uniq[inv]
        assert len(dkeys) <= g.n_pages
        dvalues = wl.page_perm[: len(dkeys)].astype(np.uint64)
        self.block_values = _dev_u64(torch, dvalues[rank])
        n_fill = max(0, wl.n_live_target - len(dkeys))
        fk, fv = filler_keys(wl.cfg, n_fill)
        self.fk, self.fv = _dev_u64(torch, fk), _dev_u64(torch, fv)
        cold = np.lexsort((dkeys, refcnt))[: len(dkeys) // 2]
        cold_keys, cold_pages = dkeys[cold], dvalues[cold].astype(np.int32)
        n_cold = len(cold)
        self.n_cold = n_cold
        self.staging = torch.empty(n_cold * g.blk_bytes, dtype=torch.uint8, device=dev)
        self.cold_keys = _dev_u64(torch, cold_keys)
        self.cold_pages = torch.from_numpy(cold_pages.copy()).to(dev)
        self.cold_slots = torch.arange(n_cold, dtype=torch.int32, device=dev)
        self.cold_vals = _dev_u64(torch, STAGED | np.arange(n_cold, dtype=np.uint64))
        rng = ops_rng(wl.cfg, 2)
        dropped = cold_keys[rng.permutation(n_cold)[: n_cold // 10]]
        self.dropped = _dev_u64(torch, dropped)
        self.ev_out = torch.empty(len(dropped), dtype=torch.int64, device=dev)
        # run the index part once to learn which staged blocks are on a matched prefix
        self.n_on = 0
        self.all_keys = _dev_u64(torch, dkeys)
        self.preload()
        self._front()
        aibx.aibx_prefix_match(self.ix, self.hash, self.blk_off, self.R, self.N, self.values, self.mlen)
        values, mlen = _u64(self.values), self.mlen.cpu().numpy()
        on_prefix = np.zeros(self.N, dtype=bool)
        for r in range(self.R):
            on_prefix[wl.blk_off[r]:wl.blk_off[r] + mlen[r]] = True
        want = on_prefix & (values != NO_VALUE) & ((values & STAGED) != 0) & ((values >> np.uint64(63)) == 0)
        on_keys, firsti = np.unique(h[want], return_index=True)
        on_slots = (values[want][firsti] & ~STAGED).astype(np.int32)
        new_pages = cold_pages[rng.permutation(n_cold)[: len(on_keys)]]
        self.n_on = len(on_keys)
        self.on_keys = _dev_u64(torch, on_keys)
        self.on_slots = torch.from_numpy(on_slots.copy()).to(dev)
        self.on_pages = torch.from_numpy(new_pages.copy()).to(dev)
        self.on_vals = _dev_u64(torch, new_pages.astype(np.uint64))
        self.plan_mlen = mlen.copy()
        self.copy_bytes = 2 * (self.n_cold + self.n_on) * g.blk_bytes
        self.gather_bytes = 2 * self.n_cold * g.blk_bytes
        self.ev_g0 = self.ev_g1 = None
        self.preload()            # the planning pass left the batch's keys in the index
        torch.cuda.synchronize()

    def preload(self):
        """Index state every step starts from: empty table plus the filler keys (load factor)."""
        a = self.a
        a.aibx_index_clear(self.ix)
        a.aibx_index_insert(self.ix, self.fk, self.fv, self.fk.numel(), self.counters[0:3])

    def _front(self):
        """Hash, index every block, offload the cold blocks, re-point and evict their entries."""
        a, wl = self.a, self.wl
        c = self.counters
        a.aibx_block_hash(self.tokens, self.tok_off, self.blk_off, self.R, self.N, wl.block_size,
                          wl.hash_seed, self.hash)
        a.aibx_index_insert(self.ix, self.hash, self.block_values, self.N, c[0:3])
        if self.ev_g0 is not None:
            self.ev_g0.record()
        a.aibx_kv_gather(self.desc, self.cold_pages, self.cold_slots, self.n_cold, self.staging,
                         wl.geom.blk_bytes, c[5:6])
        if self.ev_g1 is not None:
            self.ev_g1.record()
        a.aibx_index_insert(self.ix, self.cold_keys, self.cold_vals, self.n_cold, c[0:3])
        a.aibx_index_evict(self.ix, self.dropped, self.dropped.numel(), self.ev_out, c[3:5])

    def run(self, events=None):
        """One step, enqueued on the current stream. It ends by evicting the batch's own keys, so
        the index is back to the preloaded state (fillers only) for the next step."""
        a, wl = self.a, self.wl
        self.ev_g0, self.ev_g1 = events if events else (None, None)
        self._front()
        a.aibx_prefix_match(self.ix, self.hash, self.blk_off, self.R, self.N, self.values, self.mlen)
        a.aibx_kv_scatter(self.desc, self.on_pages, self.on_slots, self.n_on, self.staging,
                          wl.geom.blk_bytes, self.counters[6:7])
        a.aibx_index_insert(self.ix, self.on_keys, self.on_vals, self.n_on, self.counters[0:3])
        a.aibx_index_evict(self.ix, self.all_keys, self.all_keys.numel(), None, self.counters[3:5])


def time_calls(torch, fn, reps, warm=2):
    for _ in range(warm):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in evs)
    return ms[len(ms) // 2], ms[0]


def time_calls_cold(torch, fn, reps, flush):
    """Like time_calls, but a 1 GiB buffer is rewritten before every timed call, so that neither
    the L2s nor the Infinity Cache hold the call's inputs."""
    ms = []
    for _ in range(reps):
        flush.add_(1)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        ms.append(a.elapsed_time(b))
    ms.sort()
    return ms[len(ms) // 2]


def scaled_hash_match(torch, aibx, cfg, step, min_blocks):
    """Scaled batch: hash and match >= min_blocks blocks in one launch each, index unchanged."""
    from workloads import make_scaled_tokens
    tok, tok_off, blk_off = make_scaled_tokens(cfg, min_blocks)
    N, R = int(blk_off[-1]), len(blk_off) - 1
    d_tok = torch.from_numpy(tok).cuda()
    d_to, d_bo = torch.from_numpy(tok_off).cuda(), torch.from_numpy(blk_off).cuda()
    h = torch.empty(N, dtype=torch.int64, device="cuda")
    v = torch.empty(N, dtype=torch.int64, device="cuda")
    m = torch.empty(R, dtype=torch.int32, device="cuda")
    B = step.wl.block_size
    hash_ms, _ = time_calls(torch, lambda: aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h), 10)
    match_ms, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(step.ix, h, d_bo, R, N, v, m), 10)
    fused_ms, _ = time_calls(torch, lambda: aibx.aibx_hash_match(step.ix, d_tok, d_to, d_bo, R, N, B, 0, h, v, m), 10)
    per_block = 4 * B + 8 + 8 + 64 + 8
    t = (hash_ms + match_ms) * 1e-3
    rate = N / t
    fused_rate = N / (fused_ms * 1e-3)
    return {
        "fused_one_launch": {"ms": fused_ms, "blocks_per_s": fused_rate,
                             "roofline_frac": fused_rate * per_block / 1e9 / HBM_PEAK_GBPS},
        "workload": f"config {cfg} request mix replicated to {R} requests / {N} blocks / {len(tok)} tokens",
        "blocks_per_s": rate, "hash_ms": hash_ms, "match_ms": match_ms,
        "hash_GBps": N * (4 * B + 8) / (hash_ms * 1e-3) / 1e9,
        "match_Gprobes_per_s": N / (match_ms * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "achieved": rate * per_block / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": rate * per_block / 1e9 / HBM_PEAK_GBPS, "bytes_per_block": per_block},
    }


def cpu_baseline(wl, gpu_hash, gpu_mlen_fn):
    """The oracle on a bounded sample: hash+match of the whole native config, and gather+scatter
    of 512 blocks on a 1024-page host mirror of the pool. Also cross-checks the GPU's hashes."""
    import oracle
    from workloads import Geometry
    t0 = time.perf_counter()
    h = oracle.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, wl.hash_seed)
    t_hash = time.perf_counter() - t0
    checked = bool(np.array_equal(h, gpu_hash))
    ix = oracle.Index(wl.n_slots)
    ix.insert(h, np.arange(len(h), dtype=np.uint64))
    t0 = time.perf_counter()
    reps_m = 20
    for _ in range(reps_m):
        ix.match(h, wl.blk_off)
    t_match = (time.perf_counter() - t0) / reps_m
    g = Geometry(wl.geom.n_seg, wl.geom.seg_bytes, 1024)
    tile = np.random.default_rng(0).integers(0, 256, size=1 << 26, dtype=np.uint8)
    pool = np.tile(tile, g.pool_bytes // len(tile))
    n = 512
    staging = np.zeros(n * g.blk_bytes, dtype=np.uint8)
    ids = np.random.default_rng(1).permutation(g.n_pages)[:n].astype(np.int32)
    oracle.kv_gather(pool, g.as_tuple(), ids, None, staging, g.blk_bytes)        # touch pages once
    reps = 6
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.kv_gather(pool, g.as_tuple(), ids, None, staging, g.blk_bytes)
        oracle.kv_scatter(pool, g.as_tuple(), ids, None, staging, g.blk_bytes)
    t_copy = (time.perf_counter() - t0) / (2 * reps)
    return {
        "value": 2 * n * g.blk_bytes / t_copy / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"gather+scatter of {n} blocks of {g.blk_bytes} B on a {g.n_pages}-page host mirror, "
                  f"{reps} repetitions; hash+match of the native config ({wl.n_blocks} blocks)",
        "hash_match_blocks_per_s": wl.n_blocks / (t_hash + t_match),
        "gpu_hashes_equal_oracle": checked,
    }


def survey_config(torch, aibx, cfg, layout=None):
    """Per-config figures (not the headline line): copy bandwidth of one gather and one scatter
    batch at the config's geometry, two-stream gather+scatter, native-size call latencies, the
    scaled hash+match batch, and index update rates. Returns a dict."""
    from workloads import fill_pool_torch, filler_keys, make_scaled_tokens, make_workload
    wl = make_workload(cfg, "full", layout=layout)
    g = wl.geom
    out = {"config": cfg, "name": wl.name, "layout": g.layout, "n_seg": g.n_seg, "seg_bytes": g.seg_bytes,
           "blk_bytes": g.blk_bytes, "pool_GiB": g.pool_bytes / 2**30}
    n = min(wl.batch_pages, g.n_pages // 2)
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device="cuda")
    fill_pool_torch(pool, wl.kv_dtype, cfg)
    staging = torch.empty(2 * n * g.blk_bytes, dtype=torch.uint8, device="cuda")
    desc = aibx.make_pool_desc(pool, *g.as_tuple())
    rng = np.random.default_rng(cfg)
    perm = rng.permutation(g.n_pages).astype(np.int32)
    pa, pb = torch.from_numpy(perm[:n].copy()).cuda(), torch.from_numpy(perm[n:2 * n].copy()).cuda()
    sa = torch.arange(n, dtype=torch.int32, device="cuda")
    sb = torch.arange(n, 2 * n, dtype=torch.int32, device="cuda")
    traffic = 2 * n * g.blk_bytes
    ms, _ = time_calls(torch, lambda: aibx.aibx_kv_gather(desc, pa, sa, n, staging, g.blk_bytes), 7)
    out["gather_GBps"] = traffic / ms / 1e6
    ms, _ = time_calls(torch, lambda: aibx.aibx_kv_scatter(desc, pa, sa, n, staging, g.blk_bytes), 7)
    out["scatter_GBps"] = traffic / ms / 1e6
    out["batch_blocks"] = n
    if g.n_seg > 1 and g.seg_bytes % (16 * wl.block_size) == 0:
        # the same pool bytes read as token-major pages [page][token][segment][run]: the copy converts
        T, run = wl.block_size, g.seg_bytes // wl.block_size
        rd = aibx.make_pool_runs_desc(pool, g.n_seg, T, run, g.blk_bytes, g.n_seg * run, run, g.n_pages)
        ms, _ = time_calls(torch, lambda: aibx.aibx_kv_gather_runs(rd, pa, sa, n, staging, g.blk_bytes), 7)
        out["token_major"] = {"run_bytes": run, "runs_per_segment": T, "gather_GBps": traffic / ms / 1e6}
        ms, _ = time_calls(torch, lambda: aibx.aibx_kv_scatter_runs(rd, pa, sa, n, staging, g.blk_bytes), 7)
        out["token_major"]["scatter_GBps"] = traffic / ms / 1e6
    # gather and scatter of disjoint pages and slots on two streams, wall time from a common start
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    walls = []
    for _ in range(6):
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1, e2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        s1.wait_event(e0)
        s2.wait_event(e0)
        aibx.aibx_kv_gather(desc, pa, sa, n, staging, g.blk_bytes, None, s1)
        aibx.aibx_kv_scatter(desc, pb, sb, n, staging, g.blk_bytes, None, s2)
        e1.record(s1)
        e2.record(s2)
        torch.cuda.synchronize()
        walls.append(max(e0.elapsed_time(e1), e0.elapsed_time(e2)))
    out["two_stream_gather_scatter_GBps"] = 2 * traffic / sorted(walls)[len(walls) // 2] / 1e6
    # host tier: offload / onload of 1024 blocks straight between the pool and pinned host memory
    nh = min(1024, n)
    h_buf = torch.empty(nh * g.blk_bytes, dtype=torch.uint8).pin_memory()
    h_buf.zero_()                                     # first touch of the pinned pages is not timed

    def wall(fn):
        ts = []
        for _ in range(5):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        return sorted(ts)[2]
    t_off = wall(lambda: aibx.aibx_kv_offload(desc, pa, nh, h_buf, g.blk_bytes))
    t_on = wall(lambda: aibx.aibx_kv_onload(desc, pa, nh, h_buf, g.blk_bytes))
    t_d2h = wall(lambda: h_buf.copy_(staging[: h_buf.numel()], non_blocking=True))
    t_h2d = wall(lambda: staging[: h_buf.numel()].copy_(h_buf, non_blocking=True))
    # gathers on a second stream while an offload / onload runs: the rate they keep, and the transfer's
    def beside(fn):
        k = max(2, min(64, int(1.2 * (nh * g.blk_bytes / 55e9) / (ms_alone * 1e-3))))
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(k)]
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0.record(s1)
        fn(desc, pa, nh, h_buf, g.blk_bytes, None, s1)
        t1.record(s1)
        for a, b in evs:
            a.record(s2)
            aibx.aibx_kv_gather(desc, pb, sb, n, staging, g.blk_bytes, None, s2)
            b.record(s2)
        torch.cuda.synchronize()
        span, used, rates = t0.elapsed_time(t1), 0.0, []
        for a, b in evs:
            used += a.elapsed_time(b)
            if used <= span:
                rates.append(traffic / a.elapsed_time(b) / 1e6)
        rates.sort()
        return {"transfer_GBps": nh * g.blk_bytes / span / 1e6, "gathers_inside": len(rates),
                "gather_median_GBps": rates[len(rates) // 2] if rates else None,
                "gather_min_GBps": rates[0] if rates else None}
    ms_alone, _ = time_calls(torch, lambda: aibx.aibx_kv_gather(desc, pb, sb, n, staging, g.blk_bytes), 5)
    b_off, b_on = beside(aibx.aibx_kv_offload), beside(aibx.aibx_kv_onload)
    hb = nh * g.blk_bytes
    out["host_tier"] = {"blocks": nh, "offload_GBps": hb / t_off / 1e9, "onload_GBps": hb / t_on / 1e9,
                        "plain_d2h_copy_GBps": hb / t_d2h / 1e9, "plain_h2d_copy_GBps": hb / t_h2d / 1e9,
                        "gather_alone_GBps": traffic / ms_alone / 1e6,
                        "beside_offload": b_off, "beside_onload": b_on}
    del h_buf
    del pool, staging
    torch.cuda.empty_cache()
    # index + hash at native size
    B = wl.block_size
    d_tok = torch.from_numpy(wl.tokens).cuda()
    d_to, d_bo = torch.from_numpy(wl.tok_off).cuda(), torch.from_numpy(wl.blk_off).cuda()
    N, R = wl.n_blocks, wl.n_req
    h = torch.empty(N, dtype=torch.int64, device="cuda")
    v = torch.empty(N, dtype=torch.int64, device="cuda")
    m = torch.empty(R, dtype=torch.int32, device="cuda")
    storage = torch.empty(aibx.aibx_index_storage_bytes(wl.n_slots), dtype=torch.uint8, device="cuda")
    ix = aibx.aibx_index_create(storage, wl.n_slots)
    aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h)
    vals = torch.arange(N, dtype=torch.int64, device="cuda")
    c = torch.zeros(5, dtype=torch.int64, device="cuda")
    aibx.aibx_index_insert(ix, h, vals, N, c[0:3])
    n_fill = max(0, wl.n_live_target - int(c[0].item()))
    fk, fv = filler_keys(cfg, max(n_fill, 1))
    fk, fv = _dev_u64(torch, fk), _dev_u64(torch, fv)
    if n_fill:
        aibx.aibx_index_insert(ix, fk, fv, n_fill, c[0:3])
    ms_h, _ = time_calls(torch, lambda: aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h), 20)
    ms_m, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(ix, h, d_bo, R, N, v, m), 20)
    flush = torch.zeros(1 << 27, dtype=torch.int64, device="cuda")
    cold_h = time_calls_cold(torch, lambda: aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h), 7, flush)
    cold_m = time_calls_cold(torch, lambda: aibx.aibx_prefix_match(ix, h, d_bo, R, N, v, m), 7, flush)
    cold_f = time_calls_cold(torch, lambda: aibx.aibx_hash_match(ix, d_tok, d_to, d_bo, R, N, B, 0, None, v, m), 7,
                             flush)
    ms_f, _ = time_calls(torch, lambda: aibx.aibx_hash_match(ix, d_tok, d_to, d_bo, R, N, B, 0, None, v, m), 20)
    del flush
    # hash -> insert -> match -> evict of the batch's keys: four launches, eager and as one HIP graph
    ev_all = torch.empty(N, dtype=torch.int64, device="cuda")

    def metadata_sequence():
        aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h)
        aibx.aibx_index_insert(ix, h, vals, N, c[0:3])
        aibx.aibx_prefix_match(ix, h, d_bo, R, N, v, m)
        aibx.aibx_index_evict(ix, h, N, ev_all, c[3:5])
    ms_seq, _ = time_calls(torch, metadata_sequence, 20)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            metadata_sequence()
    torch.cuda.synchronize()
    ms_graph, _ = time_calls(torch, graph.replay, 20)
    del graph
    aibx.aibx_index_insert(ix, h, vals, N, c[0:3])    # the sequence ends with the batch evicted
    out["native"] = {"metadata_sequence_4_launches_us": ms_seq * 1e3,
                     "metadata_sequence_graph_replay_us": ms_graph * 1e3,
                     "requests": R, "blocks": N, "hash_us": ms_h * 1e3, "match_us": ms_m * 1e3,
                     "hash_match_one_launch_us": ms_f * 1e3, "cold_cache_hash_us": cold_h * 1e3,
                     "cold_cache_match_us": cold_m * 1e3, "cold_cache_hash_match_one_launch_us": cold_f * 1e3}
    # update rates: evict then re-insert q filler keys (rounds of the 1:1:4 mix use q = 4096)
    if n_fill >= 1 << 16:
        q = 1 << 16
        ev = torch.empty(q, dtype=torch.int64, device="cuda")

        def churn():
            aibx.aibx_index_evict(ix, fk[:q], q, ev, c[3:5])
            aibx.aibx_index_insert(ix, fk[:q], fv[:q], q, c[0:3])
        ms_c, _ = time_calls(torch, churn, 10)
        out["evict_plus_insert_Mkeys_per_s"] = 2 * q / ms_c / 1e3
        q = 4096
        n_probe = min(N, 4 * q)
        r_probe = int(np.searchsorted(wl.blk_off, n_probe, side="right")) - 1
        n_probe = int(wl.blk_off[r_probe])

        def mix_round():
            aibx.aibx_index_insert(ix, fk[:q], fv[:q], q, c[0:3])
            aibx.aibx_index_evict(ix, fk[:q], q, ev[:q], c[3:5])
            aibx.aibx_prefix_match(ix, h, d_bo, r_probe, n_probe, v, m)
        if r_probe > 0:
            ms_r, _ = time_calls(torch, mix_round, 20)
            out["mix_1_1_4_round_us"] = ms_r * 1e3
            out["mix_1_1_4_Mops_per_s"] = (2 * q + n_probe) / ms_r / 1e3
    # eviction policy: touch the batch's blocks, then one victim scan over the whole table
    ms_t, _ = time_calls(torch, lambda: aibx.aibx_index_touch(ix, h, N, 5), 10)
    cap = wl.n_slots
    vk = torch.empty(cap, dtype=torch.int64, device="cuda")
    vv = torch.empty(cap, dtype=torch.int64, device="cuda")
    vn = torch.zeros(1, dtype=torch.int64, device="cuda")
    ms_v, _ = time_calls(torch, lambda: aibx.aibx_index_select_victims(ix, 2, 3, vk, vv, cap, vn), 10)
    n_vict = int(vn.item())
    table_bytes = wl.n_slots * 20
    out["eviction_policy"] = {"touch_Mkeys_per_s": N / ms_t / 1e3, "victim_scan_us": ms_v * 1e3,
                              "victims": n_vict, "victim_scan_GBps": (table_bytes + 16 * n_vict) / ms_v / 1e6,
                              "victim_scan_frac_of_hbm_peak": (table_bytes + 16 * n_vict) / ms_v / 1e6 / HBM_PEAK_GBPS}
    del vk, vv
    # scaled batch
    tok, to, bo = make_scaled_tokens(cfg, 4 << 20)
    Ns, Rs = int(bo[-1]), len(bo) - 1
    d_tok, d_to, d_bo = torch.from_numpy(tok).cuda(), torch.from_numpy(to).cuda(), torch.from_numpy(bo).cuda()
    h = torch.empty(Ns, dtype=torch.int64, device="cuda")
    v = torch.empty(Ns, dtype=torch.int64, device="cuda")
    m = torch.empty(Rs, dtype=torch.int32, device="cuda")
    ms_h, _ = time_calls(torch, lambda: aibx.aibx_block_hash(d_tok, d_to, d_bo, Rs, Ns, B, 0, h), 10)
    ms_m, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(ix, h, d_bo, Rs, Ns, v, m), 10)
    ms_f, _ = time_calls(torch, lambda: aibx.aibx_hash_match(ix, d_tok, d_to, d_bo, Rs, Ns, B, 0, h, v, m), 10)
    # match lengths only (what a routing decision needs): no hashes, no per-block values written, and the
    # kernels stop working on a request behind its first miss
    ms_len, _ = time_calls(torch, lambda: aibx.aibx_hash_match(ix, d_tok, d_to, d_bo, Rs, Ns, B, 0, None, None, m), 10)
    ms_mlen, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(ix, h, d_bo, Rs, Ns, None, m), 10)
    per = 4 * B + 8 + 8 + 64 + 8
    rate = Ns / ((ms_h + ms_m) * 1e-3)
    out["scaled"] = {"requests": Rs, "blocks": Ns, "hash_ms": ms_h, "match_ms": ms_m, "blocks_per_s": rate,
                     "roofline_frac": rate * per / 1e9 / HBM_PEAK_GBPS, "bytes_per_block": per,
                     "lengths_only_one_launch_ms": ms_len, "lengths_only_match_ms": ms_mlen,
                     "mean_match_fraction": float(m.float().sum().item()) / Ns,
                     "one_launch_ms": ms_f, "one_launch_roofline_frac": Ns / (ms_f * 1e-3) * per / 1e9 / HBM_PEAK_GBPS,
                     "index_slots": wl.n_slots, "load_factor": wl.load_factor}
    # routing decision on the scaled batch: values read as pod sets (low 8 bits), 8 pods
    pod_sets = torch.where(v == -1, v, v & 0xFF)
    load = torch.zeros(8, dtype=torch.int32, device="cuda")
    pod = torch.empty(Rs, dtype=torch.int32, device="cuda")
    hit = torch.empty(Rs, dtype=torch.int32, device="cuda")
    ms_r, _ = time_calls(torch, lambda: aibx.aibx_route(pod_sets, d_bo, Rs, Ns, 8, load, 1, 2, pod, hit), 10)
    out["route"] = {"requests": Rs, "us": ms_r * 1e3, "Mrequests_per_s": Rs / ms_r / 1e3}
    # turnover, then compaction: evict fillers and insert fresh keys in rounds of 65,536 (a third of
    # the table's keys at most), look at the tombstones left behind, rebuild into a second table
    q = 1 << 16
    rounds = min(64, n_fill // (3 * q))
    if rounds > 0:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(cfg)
        ev = torch.empty(q, dtype=torch.int64, device="cuda")
        for r in range(rounds):
            fresh = torch.randint(1, 2**62, (q,), dtype=torch.int64, device="cuda", generator=gen)
            aibx.aibx_index_evict(ix, fk[r * q:(r + 1) * q], q, ev, c[3:5])
            aibx.aibx_index_insert(ix, fresh, fresh, q, c[0:3])
        st = torch.zeros(2, dtype=torch.int64, device="cuda")
        aibx.aibx_index_stats(ix, st)
        live, tombs = st.tolist()
        ms_before, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(ix, h, d_bo, Rs, Ns, v, m), 10)
        storage2 = torch.empty(aibx.aibx_index_storage_bytes(wl.n_slots), dtype=torch.uint8, device="cuda")
        ix2 = aibx.aibx_index_create(storage2, wl.n_slots)
        ms_rb, _ = time_calls(torch, lambda: aibx.aibx_index_rebuild(ix, ix2), 5, warm=1)
        aibx.aibx_index_stats(ix2, st)
        live2, tombs2 = st.tolist()
        ms_after, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(ix2, h, d_bo, Rs, Ns, v, m), 10)
        out["rebuild"] = {"turnover_keys": rounds * q, "live": live, "tombstones": tombs, "rebuild_ms": ms_rb,
                          "rebuild_Mkeys_per_s": live / ms_rb / 1e3, "live_after": live2, "tombstones_after": tombs2,
                          "scaled_match_ms_before": ms_before, "scaled_match_ms_after": ms_after}
        aibx.aibx_index_destroy(ix2)
    aibx.aibx_index_destroy(ix)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload (2 = the one the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-scaled", action="store_true")
    ap.add_argument("--survey", action="store_true",
                    help="instead of the headline line, print one JSON line per config (both pool "
                         "layouts) with copy bandwidths, call latencies and index rates")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain elementwise kernel that reads and writes the staging "
                         "buffer once (known HBM bytes), for scaling profiler counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path runs on ONE GPU (no sharding, no collectives); use --gpus 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    import paper_2504_03648_amd as aibx
    from workloads import make_workload
    torch.cuda.set_device(0)
    if args.survey:
        for cfg, layout in [(1, None), (2, None), (2, "page-major"), (3, None), (3, "page-major"), (4, None),
                            (4, "page-major"), (5, None), (5, "page-major")]:
            print(json.dumps(survey_config(torch, aibx, cfg, layout)), flush=True)
        return
    wl = make_workload(args.config, "full")
    step = Step(torch, aibx, wl)
    for _ in range(args.warmup):
        step.run()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step.run(evs[k])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    gather_ms = sum(a.elapsed_time(b) for a, b in evs) / args.steps
    assert np.array_equal(step.mlen.cpu().numpy(), step.plan_mlen)
    g = wl.geom
    value = step.copy_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = step.gather_bytes / (gather_ms * 1e-3) / 1e9
    # what a library device-to-device copy of the same volume reaches on this GPU, for context
    src, dst = step.staging, step.pool[: step.staging.numel()]
    plain_ms, _ = time_calls(torch, lambda: dst.copy_(src), 5)
    plain_gbps = 2 * src.numel() / (plain_ms * 1e-3) / 1e9
    traffic = None
    if MEASURED_TRAFFIC["kvcopy_sha1"] == _kvcopy_sha1():
        traffic = MEASURED_TRAFFIC["bytes_per_launch"]
    out = {
        "metric": "kv_gather_scatter_hbm_GBps", "value": value, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] {wl.name}", "requests": wl.n_req,
                   "tokens": int(wl.tok_off[-1]), "blocks": wl.n_blocks, "block_size": wl.block_size,
                   "blk_bytes": g.blk_bytes, "n_seg": g.n_seg, "pool_pages": g.n_pages,
                   "index_slots": wl.n_slots, "gathered_blocks": step.n_cold, "scattered_blocks": step.n_on},
        "pct_of_peak": 100.0 * value / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "kernel": "kv_copy_kernel<gather>",
                     "bytes_per_launch": step.gather_bytes, "avg_launch_ms": gather_ms,
                     "plain_d2d_copy_GBps": plain_gbps},
    }
    if args.calibrate:
        cal = step.staging.view(torch.int64)
        cal.add_(1)
        torch.cuda.synchronize()
        out["calibration"] = {"kernel": "torch elementwise add_ (int64)", "bytes_read": cal.numel() * 8,
                              "bytes_written": cal.numel() * 8}
    if not args.no_scaled:
        out["hash_match"] = scaled_hash_match(torch, aibx, args.config, step, 4 << 20)
        out["hash_match_blocks_per_s"] = out["hash_match"]["blocks_per_s"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, _u64(step.hash), None)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
