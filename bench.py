#!/usr/bin/env python3
"""Benchmark of the KV-cache hot path on one MI355X.

Headline (default --config 3, the largest workload that fits one GPU): the Llama-3-70B-shaped
workload - 256 requests of 2,048..8,192 tokens, 16-token blocks, a 160 GiB pool of 5 MiB blocks in
160 planes, a 2^22-slot index at load 0.7. A step is one pass of the whole path over one batch:
hash every request, index every block, match every request, gather one batch of 4,096 pages into
the 20 GiB staging buffer (offload), scatter it back into the pool (onload), and evict the batch's
keys again so that the next step starts from the same index. (--config 2 runs the 8B-shaped
offload/onload flow, --config 5 one round of the stress mix with the two copies on two streams.)
Every array the step reads is resident in HBM before the clock starts.

Prints ONE JSON line. `value` = bytes read + written by the gathers and scatters of a step divided
by the whole step's time. `roofline` is the gather kernel and `roofline_scatter` the scatter kernel
against 8 TB/s, each timed with HIP events inside the timed steps. `per_config` holds, for each of
the five workloads: gather, scatter and two-stream bandwidth at its pool geometry, native-size call
latencies, and the scaled hash+match batch (>= 4 Mi blocks) at three matched fractions, against the
152 B/block (344 B at 64-token blocks) roofline and against the bytes the kernels ask for, with a
random-read calibration on tables of the same size. `cpu_baseline` is the CPU oracle on a bounded
sample of the headline workload, on one thread and on all cores.
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
COPY_KERNEL = {"gather": "aibx::kv_copy_xcd_kernel<true, 256, false>",
               "scatter": "aibx::kv_copy_xcd_kernel<false, 256, false>"}

# HBM bytes per gather and per scatter launch of the headline workload from two rocprofv3 --pmc runs
# (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for a plain elementwise
# kernel of known size (--calibrate); valid only for the kernel source they were taken on.
MEASURED_TRAFFIC = {"kvcopy_sha1": "f7993a4a54130c5281bdd6484a450703775ef58d", "config": 3,
                    "bytes_per_launch": 42951846523, "scatter_bytes_per_launch": 42948969970}


def _u64(t):
    return t.cpu().numpy().view(np.uint64)


def _dev_u64(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64).copy()).cuda()


def _kvcopy_sha1():
    p = os.path.join(ROOT, "paper_2504_03648_amd", "csrc", "kvcopy.hip")
    return hashlib.sha1(open(p, "rb").read()).hexdigest()


def _roofline(bytes_per_launch, ms, kernel, **extra):
    gbps = bytes_per_launch / (ms * 1e-3) / 1e9
    d = {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
         "traffic": None, "kernel": kernel, "bytes_per_launch": int(bytes_per_launch), "avg_launch_ms": ms}
    d.update(extra)
    return d


class StepBase:
    """Device-resident state shared by the steps: tokens, hash/value/length arrays, pool, index."""

    def __init__(self, torch, aibx, wl):
        from workloads import fill_pool_torch
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
        self.pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=dev)
        fill_pool_torch(self.pool, wl.kv_dtype, wl.cfg)
        self.desc = aibx.make_pool_desc(self.pool, *g.as_tuple())
        self.storage = torch.empty(aibx.aibx_index_storage_bytes(wl.n_slots), dtype=torch.uint8, device=dev)
        self.ix = aibx.aibx_index_create(self.storage, wl.n_slots)
        self.counters = torch.zeros(8, dtype=torch.int64, device=dev)
        self.events = None                       # (gather start, gather end, scatter start, scatter end)
        aibx.aibx_block_hash(self.tokens, self.tok_off, self.blk_off, self.R, self.N, wl.block_size,
                             wl.hash_seed, self.hash)
        self.host_hash = _u64(self.hash)

    def _distinct(self):
        """Distinct keys of the batch by first appearance, reference counts, block -> rank."""
        h = self.host_hash
        uniq, first, inv, cnt = np.unique(h, return_index=True, return_inverse=True, return_counts=True)
        order = np.argsort(first, kind="stable")
        rank_of_uniq = np.empty(len(uniq), dtype=np.int64)
        rank_of_uniq[order] = np.arange(len(uniq))
        return uniq[order], cnt[order], rank_of_uniq[inv]

    def _fillers(self, n_real):
        from workloads import filler_keys
        n_fill = max(0, self.wl.n_live_target - n_real)
        fk, fv = filler_keys(self.wl.cfg, max(n_fill, 1))
        self.n_fill = n_fill
        self.fk, self.fv = _dev_u64(self.t, fk), _dev_u64(self.t, fv)

    def preload(self):
        """Index state every step starts from: empty table plus the filler keys (load factor)."""
        a = self.a
        a.aibx_index_clear(self.ix)
        if self.n_fill:
            a.aibx_index_insert(self.ix, self.fk, self.fv, self.n_fill, self.counters[0:3])

    def _mark(self, k):
        if self.events is not None:
            self.events[k].record()

    def check(self):
        pass


class BatchStep(StepBase):
    """Workloads 1, 3 and 4: hash, index and match every request, then move one batch of pages
    pool -> staging -> pool; the step ends by evicting the batch's keys."""

    def __init__(self, torch, aibx, wl):
        super().__init__(torch, aibx, wl)
        g = wl.geom
        dkeys, _, rank = self._distinct()
        n_res = min(len(dkeys), g.n_pages)
        dvalues = (np.uint64(1) << np.uint64(61)) | np.arange(len(dkeys), dtype=np.uint64)   # held by another tier
        dvalues[:n_res] = wl.page_perm[:n_res].astype(np.uint64)
        self.block_values = _dev_u64(torch, dvalues[rank])
        self.all_keys = _dev_u64(torch, dkeys)
        self._fillers(len(dkeys))
        self.n_batch = min(wl.batch_pages, g.n_pages)
        self.staging = torch.empty(self.n_batch * g.blk_bytes, dtype=torch.uint8, device="cuda")
        order = np.random.default_rng(wl.cfg).permutation(g.n_pages).astype(np.int32)
        nb = max(1, g.n_pages // self.n_batch)
        self.batches = [torch.from_numpy(order[k * self.n_batch:(k + 1) * self.n_batch].copy()).cuda() for k in range(nb)]
        self.k = 0
        self.copy_bytes = 4 * self.n_batch * g.blk_bytes
        self.gather_bytes = self.scatter_bytes = 2 * self.n_batch * g.blk_bytes
        self.n_gathered = self.n_scattered = self.n_batch
        self.preload()
        torch.cuda.synchronize()

    def run(self):
        a, wl, c = self.a, self.wl, self.counters
        pages = self.batches[self.k % len(self.batches)]
        self.k += 1
        a.aibx_block_hash(self.tokens, self.tok_off, self.blk_off, self.R, self.N, wl.block_size, wl.hash_seed,
                          self.hash)
        a.aibx_index_insert(self.ix, self.hash, self.block_values, self.N, c[0:3])
        a.aibx_prefix_match(self.ix, self.hash, self.blk_off, self.R, self.N, self.values, self.mlen)
        self._mark(0)
        a.aibx_kv_gather(self.desc, pages, None, self.n_batch, self.staging, wl.geom.blk_bytes, c[5:6])
        self._mark(1)
        self._mark(2)
        a.aibx_kv_scatter(self.desc, pages, None, self.n_batch, self.staging, wl.geom.blk_bytes, c[6:7])
        self._mark(3)
        a.aibx_index_evict(self.ix, self.all_keys, self.all_keys.numel(), None, c[3:5])

    def check(self):
        n_r = np.diff(self.wl.blk_off)
        assert np.array_equal(self.mlen.cpu().numpy(), n_r), "every block of the batch was indexed before the match"
        assert int(self.counters[5].item()) == 0 and int(self.counters[6].item()) == 0


class OffloadOnloadStep(StepBase):
    """Workload 2: hash, index every block, gather the cold half of the resident blocks (offload),
    re-point and evict index entries, match, scatter the staged blocks that lie on a matched prefix
    (onload), update the index, evict the batch's keys."""

    def __init__(self, torch, aibx, wl):
        from workloads.configs import ops_rng
        super().__init__(torch, aibx, wl)
        g = wl.geom
        h = self.host_hash
        dkeys, refcnt, rank = self._distinct()
        assert len(dkeys) <= g.n_pages
        dvalues = wl.page_perm[: len(dkeys)].astype(np.uint64)
        self.block_values = _dev_u64(torch, dvalues[rank])
        self._fillers(len(dkeys))
        cold = np.lexsort((dkeys, refcnt))[: len(dkeys) // 2]
        cold_keys, cold_pages = dkeys[cold], dvalues[cold].astype(np.int32)
        n_cold = self.n_cold = len(cold)
        self.staging = torch.empty(n_cold * g.blk_bytes, dtype=torch.uint8, device="cuda")
        self.cold_keys = _dev_u64(torch, cold_keys)
        self.cold_pages = torch.from_numpy(cold_pages.copy()).cuda()
        self.cold_slots = torch.arange(n_cold, dtype=torch.int32, device="cuda")
        self.cold_vals = _dev_u64(torch, STAGED | np.arange(n_cold, dtype=np.uint64))
        rng = ops_rng(wl.cfg, 2)
        dropped = cold_keys[rng.permutation(n_cold)[: n_cold // 10]]
        self.dropped = _dev_u64(torch, dropped)
        self.ev_out = torch.empty(len(dropped), dtype=torch.int64, device="cuda")
        self.all_keys = _dev_u64(torch, dkeys)
        # untimed planning pass: which staged blocks are on a matched prefix
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
        self.on_slots = torch.from_numpy(on_slots.copy()).cuda()
        self.on_pages = torch.from_numpy(new_pages.copy()).cuda()
        self.on_vals = _dev_u64(torch, new_pages.astype(np.uint64))
        self.plan_mlen = mlen.copy()
        self.copy_bytes = 2 * (self.n_cold + self.n_on) * g.blk_bytes
        self.gather_bytes = 2 * self.n_cold * g.blk_bytes
        self.scatter_bytes = 2 * self.n_on * g.blk_bytes
        self.n_gathered, self.n_scattered = self.n_cold, self.n_on
        self.preload()            # the planning pass left the batch's keys in the index
        torch.cuda.synchronize()

    def _front(self):
        a, wl, c = self.a, self.wl, self.counters
        a.aibx_block_hash(self.tokens, self.tok_off, self.blk_off, self.R, self.N, wl.block_size,
                          wl.hash_seed, self.hash)
        a.aibx_index_insert(self.ix, self.hash, self.block_values, self.N, c[0:3])
        self._mark(0)
        a.aibx_kv_gather(self.desc, self.cold_pages, self.cold_slots, self.n_cold, self.staging,
                         wl.geom.blk_bytes, c[5:6])
        self._mark(1)
        a.aibx_index_insert(self.ix, self.cold_keys, self.cold_vals, self.n_cold, c[0:3])
        a.aibx_index_evict(self.ix, self.dropped, self.dropped.numel(), self.ev_out, c[3:5])

    def run(self):
        a, wl = self.a, self.wl
        self._front()
        a.aibx_prefix_match(self.ix, self.hash, self.blk_off, self.R, self.N, self.values, self.mlen)
        self._mark(2)
        a.aibx_kv_scatter(self.desc, self.on_pages, self.on_slots, self.n_on, self.staging,
                          wl.geom.blk_bytes, self.counters[6:7])
        self._mark(3)
        a.aibx_index_insert(self.ix, self.on_keys, self.on_vals, self.n_on, self.counters[0:3])
        a.aibx_index_evict(self.ix, self.all_keys, self.all_keys.numel(), None, self.counters[3:5])

    def check(self):
        assert np.array_equal(self.mlen.cpu().numpy(), self.plan_mlen)


class StressStep(StepBase):
    """Workload 5: one round of the index mix (insert 4,096 keys, evict 4,096, probe about 16 k
    blocks) with a 4,096-page gather and a 4,096-page scatter in flight on two streams."""

    def __init__(self, torch, aibx, wl, q=4096):
        super().__init__(torch, aibx, wl)
        g = wl.geom
        dkeys, _, rank = self._distinct()
        self.q = q
        self._fillers(0)                                       # the table's load is all filler keys
        self.new_keys = _dev_u64(torch, dkeys[:q])
        self.new_vals = _dev_u64(torch, wl.page_perm[:q].astype(np.uint64))
        self.ev_out = torch.empty(q, dtype=torch.int64, device="cuda")
        r_probe = int(np.searchsorted(wl.blk_off, 4 * q, side="right")) - 1
        self.r_probe, self.n_probe = r_probe, int(wl.blk_off[r_probe])
        self.n_batch = min(wl.batch_pages, g.n_pages // 2)
        self.staging = torch.empty(2 * self.n_batch * g.blk_bytes, dtype=torch.uint8, device="cuda")
        order = np.random.default_rng(wl.cfg).permutation(g.n_pages).astype(np.int32)
        n = self.n_batch
        self.pa, self.pb = torch.from_numpy(order[:n].copy()).cuda(), torch.from_numpy(order[n:2 * n].copy()).cuda()
        self.sa = torch.arange(n, dtype=torch.int32, device="cuda")
        self.sb = torch.arange(n, 2 * n, dtype=torch.int32, device="cuda")
        self.s1, self.s2 = torch.cuda.Stream(), torch.cuda.Stream()
        self.copy_bytes = 4 * n * g.blk_bytes
        self.gather_bytes = self.scatter_bytes = 2 * n * g.blk_bytes
        self.n_gathered = self.n_scattered = n
        self.preload()
        torch.cuda.synchronize()

    def run(self):
        a, wl, c, t = self.a, self.wl, self.counters, self.t
        cur = t.cuda.current_stream()
        a.aibx_block_hash(self.tokens, self.tok_off, self.blk_off, self.R, self.N, wl.block_size, wl.hash_seed,
                          self.hash)
        a.aibx_index_insert(self.ix, self.new_keys, self.new_vals, self.q, c[0:3])
        a.aibx_index_evict(self.ix, self.new_keys, self.q, self.ev_out, c[3:5])
        a.aibx_prefix_match(self.ix, self.hash, self.blk_off, self.r_probe, self.n_probe, self.values, self.mlen)
        fork = t.cuda.Event()
        fork.record(cur)
        self.s1.wait_event(fork)
        self.s2.wait_event(fork)
        if self.events is not None:
            self.events[0].record(self.s1)
            self.events[2].record(self.s2)
        a.aibx_kv_gather(self.desc, self.pa, self.sa, self.n_batch, self.staging, wl.geom.blk_bytes, c[5:6], self.s1)
        a.aibx_kv_scatter(self.desc, self.pb, self.sb, self.n_batch, self.staging, wl.geom.blk_bytes, c[6:7], self.s2)
        if self.events is not None:
            self.events[1].record(self.s1)
            self.events[3].record(self.s2)
        j1, j2 = t.cuda.Event(), t.cuda.Event()
        j1.record(self.s1)
        j2.record(self.s2)
        cur.wait_event(j1)
        cur.wait_event(j2)


def make_step(torch, aibx, wl):
    if wl.cfg == 2:
        return OffloadOnloadStep(torch, aibx, wl)
    if wl.cfg == 5:
        return StressStep(torch, aibx, wl)
    return BatchStep(torch, aibx, wl)


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


# ---- scaled hash+match batches at chosen matched fractions -----------------------------------------
def hit_batch(torch, aibx, cfg, min_blocks, live_target, B):
    """A batch of >= min_blocks blocks whose distinct blocks fit the index (at most 0.9 x the live
    keys it is configured for): replicas 0..K-1 of the workload's request mix, and when those are
    fewer than min_blocks the same replicas again (conversations that come back: the multi-turn
    shape, every turn re-sending its prefix). Returns device tokens/offsets, hashes and counts."""
    from workloads import make_scaled_tokens
    tok, tok_off, blk_off = make_scaled_tokens(cfg, min_blocks)
    n_rep = max(1, len(tok_off) // _native_requests(cfg))
    rpr = (len(tok_off) - 1) // n_rep                                    # requests per replica
    d_tok = torch.from_numpy(tok).cuda()
    d_to, d_bo = torch.from_numpy(tok_off).cuda(), torch.from_numpy(blk_off).cuda()
    N, R = int(blk_off[-1]), len(blk_off) - 1
    h = torch.empty(N, dtype=torch.int64, device="cuda")
    aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h)
    cap = int(0.9 * live_target)

    def distinct(k):                                                     # distinct blocks of the first k replicas
        return int(torch.unique(h[: int(blk_off[k * rpr])]).numel())
    k = n_rep
    if distinct(n_rep) > cap:
        lo, hi = 1, n_rep                                                # largest k whose blocks fit
        while lo < hi:
            mid = (lo + hi + 1) // 2
            if distinct(mid) <= cap:
                lo = mid
            else:
                hi = mid - 1
        k = lo
    if k < n_rep:                                                        # the first k replicas, repeated
        r_k, t_k, b_k = k * rpr, int(tok_off[k * rpr]), int(blk_off[k * rpr])
        times = -(-min_blocks // b_k)
        tok = np.tile(tok[:t_k], times)
        lens, blks = np.tile(np.diff(tok_off[: r_k + 1]), times), np.tile(np.diff(blk_off[: r_k + 1]), times)
        tok_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        blk_off = np.concatenate([[0], np.cumsum(blks)]).astype(np.int64)
        d_tok = torch.from_numpy(tok).cuda()
        d_to, d_bo = torch.from_numpy(tok_off).cuda(), torch.from_numpy(blk_off).cuda()
        N, R = int(blk_off[-1]), len(blk_off) - 1
        h = torch.empty(N, dtype=torch.int64, device="cuda")
        aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h)
    n_distinct = int(torch.unique(h).numel())
    return {"tok": d_tok, "tok_off": d_to, "blk_off": d_bo, "hash": h, "N": N, "R": R, "replicas": k,
            "repeats": 1 if k == n_rep else times, "distinct": n_distinct, "tokens": int(tok_off[-1])}


def _native_requests(cfg):
    return {1: 16, 2: 64, 3: 256, 4: 128, 5: 1024}[cfg]


def hash_match_at_fractions(torch, aibx, wl, ix, fk, fv, fractions=(0.0, 0.5, 1.0), min_blocks=4 << 20):
    """The scaled batch hashed and matched against the workload's index (its configured size and
    load) holding none, the first half, or all of every request's blocks, the rest of the load
    being filler keys. Two launches (hash, match) and one (aibx_hash_match), every lookup kept."""
    B = wl.block_size
    hb = hit_batch(torch, aibx, wl.cfg, min_blocks, wl.n_live_target, B)
    N, R, h, d_bo = hb["N"], hb["R"], hb["hash"], hb["blk_off"]
    v = torch.empty(N, dtype=torch.int64, device="cuda")
    m = torch.empty(R, dtype=torch.int32, device="cuda")
    n_r = (d_bo[1:] - d_bo[:-1])
    req_of = torch.repeat_interleave(torch.arange(R, device="cuda"), n_r)
    pos = torch.arange(N, device="cuda") - d_bo[:-1][req_of]
    c = torch.zeros(3, dtype=torch.int64, device="cuda")
    contract = 4 * B + 8 + 8 + 64 + 8
    rows = []
    for f in fractions:
        aibx.aibx_index_clear(ix)
        c.zero_()
        if f > 0:
            keep = pos < torch.ceil(n_r.double() * f).long()[req_of]
            keys = h[keep].contiguous()
            aibx.aibx_index_insert(ix, keys, (keys >> 8) & ((1 << 56) - 1), keys.numel(), c)   # value: a function of the key
        n_real = int(c[0].item())
        n_fill = max(0, min(wl.n_live_target - n_real, fk.numel()))
        if n_fill:
            aibx.aibx_index_insert(ix, fk, fv, n_fill, c)
        assert int(c[2].item()) == 0
        args = (hb["tok"], hb["tok_off"], d_bo, R, N, B, 0)
        ms_h, _ = time_calls(torch, lambda: aibx.aibx_block_hash(*args, h), 10)
        ms_m, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(ix, h, d_bo, R, N, v, m), 10)
        ms_f, _ = time_calls(torch, lambda: aibx.aibx_hash_match(ix, *args, h, v, m), 10)
        ms_l, _ = time_calls(torch, lambda: aibx.aibx_hash_match(ix, *args, None, None, m), 10)
        hit = float((v != -1).float().mean().item())
        matched = float(m.double().sum().item()) / N
        real = 4 * B + 8 + 8 + 16 + 16 * hit + 8         # tokens, hash out and in, a pair's tags, slot on a hit, value out
        two, one = N / ((ms_h + ms_m) * 1e-3), N / (ms_f * 1e-3)
        rows.append({
            "index_holds": f, "matched_fraction": matched, "lookup_hit_fraction": hit, "keys_from_batch": n_real,
            "filler_keys": n_fill, "hash_ms": ms_h, "match_ms": ms_m, "one_launch_ms": ms_f,
            "lengths_only_one_launch_ms": ms_l,
            "blocks_per_s": two, "one_launch_blocks_per_s": one, "match_Gprobes_per_s": N / (ms_m * 1e-3) / 1e9,
            "roofline_frac": two * contract / 1e9 / HBM_PEAK_GBPS,
            "one_launch_roofline_frac": one * contract / 1e9 / HBM_PEAK_GBPS,
            "bytes_moved_per_block": real, "bytes_moved_frac": two * real / 1e9 / HBM_PEAK_GBPS,
            "one_launch_bytes_moved_frac": one * (real - 8) / 1e9 / HBM_PEAK_GBPS})   # no hash read-back
    return {"workload": f"config {wl.cfg} request mix: replicas 0..{hb['replicas'] - 1} x {hb['repeats']} = {R} requests / "
                        f"{N} blocks / {hb['tokens']} tokens, {hb['distinct']} distinct blocks",
            "requests": R, "blocks": N, "distinct_blocks": hb["distinct"], "index_slots": wl.n_slots,
            "load_factor": wl.load_factor, "roofline_bytes_per_block": contract,
            "roofline_blocks_per_s": HBM_PEAK_GBPS * 1e9 / contract, "by_index_contents": rows}


def random_read_calibration(torch, aibx, n_slots):
    """Independent random reads (one per lane and step) over tables of the sizes a lookup touches:
    8 bytes of a random 8-byte word of a tag array of n_slots bytes, and 16 bytes of a random
    128-byte line of a slot array of 16*n_slots bytes. G reads/s."""
    out = {}
    sink = torch.zeros(1, dtype=torch.int64, device="cuda")
    n = 1 << 24
    for name, nbytes, line, rd in (("tag_words", max(n_slots, 1024), 8, 8), ("slot_lines", 16 * n_slots, 128, 16)):
        table = torch.zeros(max(nbytes, 4096), dtype=torch.uint8, device="cuda")
        ms, _ = time_calls(torch, lambda: aibx.aibx_calib_random_reads(table, nbytes, line, rd, n, 1, sink), 5)
        out[name] = {"table_bytes": nbytes, "line_bytes": line, "read_bytes": rd, "Greads_per_s": n / (ms * 1e-3) / 1e9}
        del table
    return out


def measure_config(torch, aibx, cfg, step=None, with_hash_match=True):
    """Per-workload figures: one gather and one scatter batch at the workload's pool geometry
    (random distinct pages), both on two streams, native-size call latencies, the scaled hash+match
    batch at three matched fractions, and the random-read calibration for its table size."""
    from workloads import fill_pool_torch, filler_keys, make_workload
    wl = step.wl if step is not None else make_workload(cfg, "full")
    g = wl.geom
    out = {"config": cfg, "workload": f"configs[{cfg - 1}] {wl.name}", "layout": g.layout, "n_seg": g.n_seg,
           "seg_bytes": g.seg_bytes, "blk_bytes": g.blk_bytes, "pool_GiB": g.pool_bytes / 2**30,
           "plane_stride_MiB": g.seg_stride / 2**20}
    n = min(wl.batch_pages, g.n_pages // 2)
    if step is not None:
        pool = step.pool
        step.staging = None                                   # the step is done: its staging memory is reused
        torch.cuda.empty_cache()
    else:
        pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device="cuda")
        fill_pool_torch(pool, wl.kv_dtype, cfg)
    staging = torch.empty(2 * n * g.blk_bytes, dtype=torch.uint8, device="cuda")
    desc = aibx.make_pool_desc(pool, *g.as_tuple())
    perm = np.random.default_rng(cfg).permutation(g.n_pages).astype(np.int32)
    pa, pb = torch.from_numpy(perm[:n].copy()).cuda(), torch.from_numpy(perm[n:2 * n].copy()).cuda()
    sa = torch.arange(n, dtype=torch.int32, device="cuda")
    sb = torch.arange(n, 2 * n, dtype=torch.int32, device="cuda")
    traffic = 2 * n * g.blk_bytes
    ms, _ = time_calls(torch, lambda: aibx.aibx_kv_gather(desc, pa, sa, n, staging, g.blk_bytes), 7)
    out["gather"] = _roofline(traffic, ms, COPY_KERNEL["gather"], blocks=n)
    ms, _ = time_calls(torch, lambda: aibx.aibx_kv_scatter(desc, pa, sa, n, staging, g.blk_bytes), 7)
    out["scatter"] = _roofline(traffic, ms, COPY_KERNEL["scatter"], blocks=n)
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
    wall = sorted(walls)[len(walls) // 2]
    out["two_stream_gather_scatter"] = {"GBps": 2 * traffic / wall / 1e6, "frac": 2 * traffic / wall / 1e6 / HBM_PEAK_GBPS,
                                        "wall_ms": wall}
    if g.n_seg > 1:
        # the same blocks in a page-major pool (one contiguous segment per page) over the same memory
        pm = aibx.make_pool_desc(pool, 1, g.blk_bytes * g.n_pages, g.blk_bytes, g.blk_bytes, g.n_pages)
        ms, _ = time_calls(torch, lambda: aibx.aibx_kv_gather(pm, pa, sa, n, staging, g.blk_bytes), 5)
        ms2, _ = time_calls(torch, lambda: aibx.aibx_kv_scatter(pm, pa, sa, n, staging, g.blk_bytes), 5)
        out["page_major"] = {"gather_GBps": traffic / ms / 1e6, "scatter_GBps": traffic / ms2 / 1e6}
    del staging, pool
    if step is not None:
        step.pool = None
    torch.cuda.empty_cache()
    if not with_hash_match:
        return out
    # native size: what a router sees per call
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
    c = torch.zeros(5, dtype=torch.int64, device="cuda")
    aibx.aibx_index_insert(ix, h, ((h >> 8) & ((1 << 56) - 1)) | 0xFF, N, c[0:3])   # read as pod sets: all of 8 pods
    n_fill = max(0, wl.n_live_target - int(c[0].item()))
    fk, fv = filler_keys(cfg, max(wl.n_live_target, 1))
    fk, fv = _dev_u64(torch, fk), _dev_u64(torch, fv)
    if n_fill:
        aibx.aibx_index_insert(ix, fk, fv, n_fill, c[0:3])
    ms_h, _ = time_calls(torch, lambda: aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h), 20)
    ms_m, _ = time_calls(torch, lambda: aibx.aibx_prefix_match(ix, h, d_bo, R, N, v, m), 20)
    ms_f, _ = time_calls(torch, lambda: aibx.aibx_hash_match(ix, d_tok, d_to, d_bo, R, N, B, 0, None, v, m), 20)
    ms_l, _ = time_calls(torch, lambda: aibx.aibx_hash_match(ix, d_tok, d_to, d_bo, R, N, B, 0, None, None, m), 20)
    # the routing decision for the batch (8 pods, threshold 1/2): three launches, two, one
    load = torch.zeros(8, dtype=torch.int32, device="cuda")
    pod = torch.empty(R, dtype=torch.int32, device="cuda")
    hit = torch.empty(R, dtype=torch.int32, device="cuda")

    def three():
        aibx.aibx_block_hash(d_tok, d_to, d_bo, R, N, B, 0, h)
        aibx.aibx_prefix_match(ix, h, d_bo, R, N, v, m)
        aibx.aibx_route(v, d_bo, R, N, 8, load, 1, 2, pod, hit)

    def two():
        aibx.aibx_hash_match(ix, d_tok, d_to, d_bo, R, N, B, 0, None, v, m)
        aibx.aibx_route(v, d_bo, R, N, 8, load, 1, 2, pod, hit)
    ms_3, _ = time_calls(torch, three, 20)
    ms_2, _ = time_calls(torch, two, 20)
    want = (pod.clone(), hit.clone())
    ms_1, _ = time_calls(torch, lambda: aibx.aibx_hash_match_route(ix, d_tok, d_to, d_bo, R, N, B, 0, 8, load, 1, 2,
                                                                   pod, hit), 20)
    assert torch.equal(pod, want[0]) and torch.equal(hit, want[1])
    out["native"] = {"requests": R, "blocks": N, "hash_us": ms_h * 1e3, "match_us": ms_m * 1e3,
                     "hash_match_one_launch_us": ms_f * 1e3, "lengths_only_one_launch_us": ms_l * 1e3,
                     "tokens_to_pod_three_launches_us": ms_3 * 1e3, "tokens_to_pod_two_launches_us": ms_2 * 1e3,
                     "tokens_to_pod_one_launch_us": ms_1 * 1e3, "every_block_present": True}
    out["random_read_calibration"] = random_read_calibration(torch, aibx, wl.n_slots)
    out["hash_match"] = hash_match_at_fractions(torch, aibx, wl, ix, fk, fv)
    aibx.aibx_index_destroy(ix)
    del storage, fk, fv
    torch.cuda.empty_cache()
    return out


def copy_probe(torch, aibx, wl, spec, launches, pool_pages=None):
    """`launches` launches (after one warm-up) of one copy at the workload's pool geometry and batch
    size, random distinct pages (2 x n x blk_bytes of traffic per launch), then one plain elementwise
    kernel of known traffic for scaling a profiler's byte counters. pool_pages changes the number
    of pages per plane, i.e. the distance between the planes of a layer-major pool."""
    from workloads import Geometry, fill_pool_torch
    layout, op = spec.split(":")
    assert layout in ("layer", "page") and op in ("gather", "scatter"), spec
    g = wl.geom
    if pool_pages is not None:
        g = Geometry(g.n_seg, g.seg_bytes, int(pool_pages), g.layout)
    n = min(wl.batch_pages, g.n_pages // 2)
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device="cuda")
    fill_pool_torch(pool, wl.kv_dtype, wl.cfg)
    staging = torch.empty(n * g.blk_bytes, dtype=torch.uint8, device="cuda")
    staging.view(torch.int64).random_()
    if layout == "layer":
        desc = aibx.make_pool_desc(pool, *g.as_tuple())
    else:
        desc = aibx.make_pool_desc(pool, 1, g.blk_bytes * g.n_pages, g.blk_bytes, g.blk_bytes, g.n_pages)
    perm = np.random.default_rng(wl.cfg).permutation(g.n_pages).astype(np.int32)
    pages = torch.from_numpy(perm[:n].copy()).cuda()
    fn = aibx.aibx_kv_gather if op == "gather" else aibx.aibx_kv_scatter
    ms, best = time_calls(torch, lambda: fn(desc, pages, None, n, staging, g.blk_bytes), launches, warm=1)
    cal = staging.view(torch.int64)          # known traffic for scaling the profiler's byte counters
    cal.add_(1)
    torch.cuda.synchronize()
    traffic = 2 * n * g.blk_bytes
    return {"probe": spec, "config": wl.cfg, "pool_pages": g.n_pages, "plane_stride_MiB": g.seg_stride / 2**20,
            "n_seg": g.n_seg if layout == "layer" else 1,
            "seg_bytes": g.seg_bytes if layout == "layer" else g.blk_bytes, "blocks": n, "launches": launches + 1,
            "bytes_per_launch": traffic, "median_ms": ms, "GBps": traffic / ms / 1e6,
            "calibration": {"kernel": "torch elementwise add_ (int64)", "bytes_read": cal.numel() * 8,
                            "bytes_written": cal.numel() * 8}}


# ---- the oracle on the host ------------------------------------------------------------------------
def _host_info():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return model, os.cpu_count() or 1, usable


def cpu_baseline(wl, gpu_hash):
    """The oracle, unchanged, on a bounded sample of the headline workload: hash+match of the whole
    native batch, and gather+scatter of 512 blocks on a 1,024-page host mirror of the pool; on one
    thread, and on all usable cores (at most 16) by giving each thread its own requests (hash) or
    its own entries (copies) - the index stays serial. Also cross-checks the GPU's hashes."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    from workloads import Geometry
    model, n_cpu, usable = _host_info()
    threads = max(1, min(16, usable))
    B = wl.block_size

    def hash_range(r0, r1):
        to, bo = wl.tok_off[r0:r1 + 1], wl.blk_off[r0:r1 + 1]
        return oracle.block_hash(wl.tokens[to[0]:to[-1]], to - to[0], bo - bo[0], B, wl.hash_seed)
    def median_time(fn, reps=5):
        fn()                                                                  # warm-up
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            r = fn()
            ts.append(time.perf_counter() - t0)
        return sorted(ts)[len(ts) // 2], r
    t_hash, h = median_time(lambda: hash_range(0, wl.n_req))
    checked = bool(np.array_equal(h, gpu_hash))
    cuts = np.linspace(0, wl.n_req, threads + 1).astype(int)
    with ThreadPoolExecutor(threads) as ex:
        t_hash_mt, parts = median_time(lambda: list(ex.map(lambda k: hash_range(cuts[k], cuts[k + 1]), range(threads))))
    assert np.array_equal(np.concatenate(parts), h)
    ix = oracle.Index(wl.n_slots)
    ix.insert(h, np.arange(len(h), dtype=np.uint64))
    reps_m = 10
    t0 = time.perf_counter()
    for _ in range(reps_m):
        ix.match(h, wl.blk_off)
    t_match = (time.perf_counter() - t0) / reps_m
    g = Geometry(wl.geom.n_seg, wl.geom.seg_bytes, 1024)
    tile = np.random.default_rng(0).integers(0, 256, size=1 << 26, dtype=np.uint8)
    pool = np.tile(tile, -(-g.pool_bytes // len(tile)))[: g.pool_bytes]
    n = 512
    staging = np.zeros(n * g.blk_bytes, dtype=np.uint8)
    ids = np.random.default_rng(1).permutation(g.n_pages)[:n].astype(np.int32)
    slots = np.arange(n, dtype=np.int32)
    geom = g.as_tuple()

    def copy_range(k0, k1):
        oracle.kv_gather(pool, geom, ids[k0:k1], slots[k0:k1], staging, g.blk_bytes)
        oracle.kv_scatter(pool, geom, ids[k0:k1], slots[k0:k1], staging, g.blk_bytes)
    copy_range(0, n)                                                          # touch the pages once
    reps = 4
    t0 = time.perf_counter()
    for _ in range(reps):
        copy_range(0, n)
    t_copy = (time.perf_counter() - t0) / (2 * reps)
    ecuts = np.linspace(0, n, threads + 1).astype(int)
    with ThreadPoolExecutor(threads) as ex:
        t0 = time.perf_counter()
        for _ in range(reps):
            list(ex.map(lambda k: copy_range(ecuts[k], ecuts[k + 1]), range(threads)))
        t_copy_mt = (time.perf_counter() - t0) / (2 * reps)
    bytes_moved = 2 * n * g.blk_bytes
    return {
        "value": bytes_moved / t_copy_mt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": f"gather+scatter of {n} blocks of {g.blk_bytes} B on a {g.n_pages}-page host mirror "
                  f"({g.pool_bytes / 2**30:.1f} GiB), {reps} repetitions; hash+match of the native batch "
                  f"({wl.n_blocks} blocks, index serial)",
        "one_thread": {"value": bytes_moved / t_copy / 1e9, "unit": "GB/s", "cores": 1,
                       "hash_match_blocks_per_s": wl.n_blocks / (t_hash + t_match)},
        "hash_match_blocks_per_s": wl.n_blocks / (t_hash_mt + t_match),
        "cpu_model": model, "nproc": n_cpu, "usable_cpus": usable, "threads": threads,
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
    ap.add_argument("--config", type=int, default=3,
                    help="headline workload (3 = Llama-3-70B-shaped, the largest that fits one GPU)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="leave out the per_config array (the other four workloads are then not run)")
    ap.add_argument("--only-steps", action="store_true",
                    help="run the warm-up and the timed steps and nothing else (for profiler runs)")
    ap.add_argument("--copy-probe", metavar="LAYOUT:OP", default=None,
                    help="profiler aid: nothing but --steps launches of one copy at the workload's pool "
                         "geometry; LAYOUT layer|page, OP gather|scatter (e.g. layer:scatter)")
    ap.add_argument("--pool-pages", type=int, default=None,
                    help="with --copy-probe: pages per plane of the pool (sets the plane stride) instead of "
                         "the workload's own")
    ap.add_argument("--hash-match-probe", metavar="F", type=float, default=None,
                    help="profiler aid: nothing but the scaled hash+match batch with the index holding the "
                         "first fraction F of every request's blocks")
    ap.add_argument("--random-read-probe", metavar="MIB:BYTES", default=None,
                    help="profiler aid: nothing but --steps launches of 16 Mi independent random reads of BYTES "
                         "(8, 16, 64 or 128) from the start of random 128-byte lines of a table of MIB MiB")
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
    if args.random_read_probe is not None:
        mib, rd = (int(x) for x in args.random_read_probe.split(":"))
        table = torch.zeros(mib << 20, dtype=torch.uint8, device="cuda")
        sink = torch.zeros(1, dtype=torch.int64, device="cuda")
        n = 1 << 24
        ms, _ = time_calls(torch, lambda: aibx.aibx_calib_random_reads(table, mib << 20, 128, rd, n, 1, sink),
                           args.steps, warm=1)
        print(json.dumps({"table_MiB": mib, "line_bytes": 128, "read_bytes": rd, "reads": n, "ms": ms,
                          "Greads_per_s": n / (ms * 1e-3) / 1e9, "launches": args.steps + 1}))
        return
    wl = make_workload(args.config, "full")
    if args.copy_probe is not None:
        print(json.dumps(copy_probe(torch, aibx, wl, args.copy_probe, args.steps, args.pool_pages)))
        return
    if args.hash_match_probe is not None:
        from workloads import filler_keys
        storage = torch.empty(aibx.aibx_index_storage_bytes(wl.n_slots), dtype=torch.uint8, device="cuda")
        ix = aibx.aibx_index_create(storage, wl.n_slots)
        fk, fv = filler_keys(args.config, max(wl.n_live_target, 1))
        res = hash_match_at_fractions(torch, aibx, wl, ix, _dev_u64(torch, fk), _dev_u64(torch, fv),
                                      fractions=(args.hash_match_probe,))
        print(json.dumps(res))
        return
    step = make_step(torch, aibx, wl)
    for _ in range(args.warmup):
        step.run()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step.events = evs[k]
        step.run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step.events = None
    step.check()
    ms_per_step = dt * 1e3 / args.steps
    gather_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    scatter_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    g = wl.geom
    value = step.copy_bytes / (ms_per_step * 1e-3) / 1e9
    roof_g = _roofline(step.gather_bytes, gather_ms, COPY_KERNEL["gather"], blocks=step.n_gathered)
    roof_s = _roofline(step.scatter_bytes, scatter_ms, COPY_KERNEL["scatter"], blocks=step.n_scattered)
    if (MEASURED_TRAFFIC["kvcopy_sha1"] == _kvcopy_sha1() and MEASURED_TRAFFIC["config"] == args.config):
        roof_g["traffic"] = MEASURED_TRAFFIC["bytes_per_launch"]
        roof_s["traffic"] = MEASURED_TRAFFIC["scatter_bytes_per_launch"]
    out = {
        "metric": "kv_gather_scatter_hbm_GBps", "value": value, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] {wl.name}", "requests": wl.n_req,
                   "tokens": int(wl.tok_off[-1]), "blocks": wl.n_blocks, "block_size": wl.block_size,
                   "blk_bytes": g.blk_bytes, "n_seg": g.n_seg, "pool_pages": g.n_pages,
                   "pool_GiB": g.pool_bytes / 2**30, "index_slots": wl.n_slots, "load_factor": wl.load_factor,
                   "gathered_blocks": step.n_gathered, "scattered_blocks": step.n_scattered},
        "pct_of_peak": 100.0 * value / HBM_PEAK_GBPS,
        "roofline": roof_g, "roofline_scatter": roof_s,
    }
    if args.only_steps:
        if args.calibrate:
            cal = step.staging.view(torch.int64)
            cal.add_(1)
            torch.cuda.synchronize()
            out["calibration"] = {"kernel": "torch elementwise add_ (int64)", "bytes_read": cal.numel() * 8,
                                  "bytes_written": cal.numel() * 8}
        print(json.dumps(out))
        return
    # what a library device-to-device copy of a staging-sized volume reaches on this GPU, for context
    src = step.staging[: min(step.staging.numel(), 8 << 30)]
    dst = step.pool[: src.numel()]
    plain_ms, _ = time_calls(torch, lambda: dst.copy_(src), 5)
    out["roofline"]["plain_d2d_copy_GBps"] = 2 * src.numel() / (plain_ms * 1e-3) / 1e9
    del src, dst
    if args.calibrate:
        cal = step.staging.view(torch.int64)
        cal.add_(1)
        torch.cuda.synchronize()
        out["calibration"] = {"kernel": "torch elementwise add_ (int64)", "bytes_read": cal.numel() * 8,
                              "bytes_written": cal.numel() * 8}
        del cal
    gpu_hash = step.host_hash
    if not args.no_per_config:
        by_cfg = {args.config: measure_config(torch, aibx, args.config, step=step)}   # reuses the step's pool
        step = None
        torch.cuda.empty_cache()
        for cfg in (1, 2, 3, 4, 5):
            if cfg not in by_cfg:
                by_cfg[cfg] = measure_config(torch, aibx, cfg)
                torch.cuda.empty_cache()
        per = [by_cfg[cfg] for cfg in (1, 2, 3, 4, 5)]
        out["per_config"] = per
        mine = per[args.config - 1]
        out["hash_match"] = mine["hash_match"]
        out["hash_match_blocks_per_s"] = mine["hash_match"]["by_index_contents"][0]["blocks_per_s"]
    step = None
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, gpu_hash)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
