"""Backends for workloads.flows: the CPU oracle, and the HIP library through its Python binding."""
from __future__ import annotations

import numpy as np


class OracleBackend:
    name = "oracle"

    def __init__(self):
        import oracle
        self.o = oracle
        self.pool = self.staging = self.geom = None

    def block_hash(self, tokens, tok_off, blk_off, block_size, seed):
        return self.o.block_hash(tokens, tok_off, blk_off, block_size, seed)

    def index_create(self, n_slots):
        return self.o.Index(n_slots)

    def pool_create(self, geom, kv_dtype, cfg):
        from workloads import fill_pool_numpy
        self.geom = geom
        self.pool = fill_pool_numpy(geom, kv_dtype, cfg)

    def staging_create(self, n_blocks, stride):
        self.stride = int(stride)
        self.staging = np.zeros(int(n_blocks) * self.stride, dtype=np.uint8)

    def _check(self, page_ids, slot_ids):
        n = len(page_ids)
        slots = np.arange(n) if slot_ids is None else np.asarray(slot_ids)
        assert n == 0 or (int(slots.min()) >= 0 and (int(slots.max()) + 1) * self.stride <= len(self.staging))

    def gather(self, page_ids, slot_ids):
        self._check(page_ids, slot_ids)
        return self.o.kv_gather(self.pool, self.geom.as_tuple(), page_ids, slot_ids, self.staging,
                                self.stride)

    def scatter(self, page_ids, slot_ids):
        self._check(page_ids, slot_ids)
        return self.o.kv_scatter(self.pool, self.geom.as_tuple(), page_ids, slot_ids, self.staging,
                                 self.stride)

    def gather_scatter_pair(self, g_pages, g_slots, s_pages, s_slots):
        return (self.gather(g_pages, g_slots), self.scatter(s_pages, s_slots))

    def _planes(self):
        g = self.geom
        return self.pool.reshape(g.n_seg, g.n_pages, g.seg_bytes)

    def fill_pages(self, page_ids, byte):
        self._planes()[:, np.asarray(page_ids, dtype=np.int64), :] = byte

    def read_pages(self, page_ids):
        ids = np.asarray(page_ids, dtype=np.int64)
        return np.ascontiguousarray(self._planes()[:, ids, :].transpose(1, 0, 2)).reshape(len(ids), -1)

    def read_slots(self, slot_ids):
        ids = np.asarray(slot_ids, dtype=np.int64)
        st = self.staging.reshape(-1, self.stride)
        return st[ids, : self.geom.blk_bytes].copy()


class CompactOracleBackend(OracleBackend):
    """The oracle on a pool that is too large to mirror on the host: only the pages a flow names
    exist here, as rows of a compact pool of `capacity` pages with the same planes and segment
    size. A page gets its row the first time a call names it, filled with the page's original
    bytes by `fetch(page_ids) -> uint8[n, blk_bytes]` (transport of input data; none of the
    method's arithmetic). Page ids are translated to rows on the way into the oracle's copies:
    holes stay holes, ids outside the real pool stay outside the compact one."""
    name = "oracle-compact"

    def __init__(self, fetch, capacity):
        super().__init__()
        self.fetch, self.capacity = fetch, int(capacity)
        self.row_of = {}
        self.full_pages = 0

    def pool_create(self, geom, kv_dtype, cfg):
        from workloads import Geometry
        self.full_pages = geom.n_pages
        self.geom = Geometry(geom.n_seg, geom.seg_bytes, self.capacity, geom.layout)
        self.pool = np.zeros(self.geom.pool_bytes, dtype=np.uint8)

    def named_pages(self):
        return np.fromiter(self.row_of.keys(), dtype=np.int64, count=len(self.row_of))

    def _rows(self, page_ids):
        ids = np.asarray(page_ids, dtype=np.int64)
        real = (ids >= 0) & (ids < self.full_pages)
        new = [int(p) for p in np.unique(ids[real]) if int(p) not in self.row_of]
        if new:
            assert len(self.row_of) + len(new) <= self.capacity, "compact pool too small for this flow"
            planes = self._planes()
            for a in range(0, len(new), 512):
                part = new[a:a + 512]
                rows = np.arange(len(self.row_of), len(self.row_of) + len(part))
                blocks = self.fetch(np.asarray(part, dtype=np.int64))
                planes[:, rows, :] = blocks.reshape(len(part), self.geom.n_seg, self.geom.seg_bytes).transpose(1, 0, 2)
                for p, r in zip(part, rows):
                    self.row_of[p] = int(r)
        out = np.where(ids < 0, -1, self.capacity).astype(np.int32)   # holes; ids beyond the pool stay bad
        out[real] = [self.row_of[int(p)] for p in ids[real]]
        return out

    def gather(self, page_ids, slot_ids):
        return super().gather(self._rows(page_ids), slot_ids)

    def scatter(self, page_ids, slot_ids):
        return super().scatter(self._rows(page_ids), slot_ids)

    def fill_pages(self, page_ids, byte):
        super().fill_pages(self._rows(page_ids), byte)

    def read_pages(self, page_ids):
        return super().read_pages(self._rows(page_ids))


class HipIndex:
    """Index handle over the HIP library, with the same surface as oracle.Index."""

    def __init__(self, n_slots, stream=None):
        import torch
        import paper_2504_03648_amd as aibx
        self.t, self.a = torch, aibx
        self.n_slots = int(n_slots)
        nbytes = aibx.aibx_index_storage_bytes(self.n_slots)
        self.storage = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.h = aibx.aibx_index_create(self.storage, self.n_slots)
        self.c_ins = torch.zeros(3, dtype=torch.int64, device="cuda")
        self.c_ev = torch.zeros(2, dtype=torch.int64, device="cuda")

    def __del__(self):
        try:
            if getattr(self, "h", None) is not None:
                self.a.aibx_index_destroy(self.h)
                self.h = None
        except Exception:          # interpreter shutdown: the binding may already be gone
            pass

    def _dev(self, x, dtype=np.uint64):
        x = np.ascontiguousarray(x, dtype=dtype)
        if dtype == np.uint64:
            x = x.view(np.int64)
        return self.t.from_numpy(x.copy()).cuda()

    @staticmethod
    def _host_u64(t):
        return t.cpu().numpy().view(np.uint64)

    @property
    def counters_insert(self):
        return self._host_u64(self.c_ins)

    @property
    def counters_evict(self):
        return self._host_u64(self.c_ev)

    def clear(self):
        self.a.aibx_index_clear(self.h)

    def insert(self, keys, values):
        k, v = self._dev(keys), self._dev(values)
        assert k.shape == v.shape
        self.a.aibx_index_insert(self.h, k, v, k.numel(), self.c_ins)

    def evict(self, keys):
        k = self._dev(keys)
        out = self.t.empty_like(k)
        self.a.aibx_index_evict(self.h, k, k.numel(), out, self.c_ev)
        return self._host_u64(out)

    def count(self):
        n = self.t.empty(1, dtype=self.t.int64, device="cuda")
        self.a.aibx_index_count(self.h, n)
        return int(n.item())

    def dump(self):
        cap = self.count()
        k = self.t.empty(max(cap, 1), dtype=self.t.int64, device="cuda")
        v = self.t.empty_like(k)
        n = self.t.empty(1, dtype=self.t.int64, device="cuda")
        self.a.aibx_index_dump(self.h, k, v, cap, n)
        assert int(n.item()) == cap
        hk, hv = self._host_u64(k)[:cap], self._host_u64(v)[:cap]
        order = np.argsort(hk, kind="stable")
        return hk[order], hv[order]

    def stats(self):
        """(live keys, tombstones)"""
        out = self.t.empty(2, dtype=self.t.int64, device="cuda")
        self.a.aibx_index_stats(self.h, out)
        live, tombs = out.tolist()
        return live, tombs

    def rebuild_into(self, dst: "HipIndex"):
        c = self.t.zeros(3, dtype=self.t.int64, device="cuda")
        self.a.aibx_index_rebuild(self.h, dst.h, c)
        return self._host_u64(c)

    def touch(self, keys, epoch):
        k = self._dev(keys)
        self.a.aibx_index_touch(self.h, k, k.numel(), epoch)

    def age(self):
        self.a.aibx_index_age(self.h)

    def select_victims(self, protect_count, before_epoch):
        cap = max(self.count(), 1)
        k = self.t.empty(cap, dtype=self.t.int64, device="cuda")
        v = self.t.empty_like(k)
        n = self.t.empty(1, dtype=self.t.int64, device="cuda")
        self.a.aibx_index_select_victims(self.h, protect_count, before_epoch, k, v, cap, n)
        m = int(n.item())
        hk, hv = self._host_u64(k)[:m], self._host_u64(v)[:m]
        order = np.argsort(hk, kind="stable")
        return hk[order], hv[order]

    def match(self, hashes, blk_off):
        h = self._dev(hashes)
        bo = self._dev(blk_off, np.int64)
        n_req = bo.numel() - 1
        values = self.t.empty_like(h)
        mlen = self.t.full((max(n_req, 0),), -7, dtype=self.t.int32, device="cuda")
        self.a.aibx_prefix_match(self.h, h, bo, n_req, h.numel(), values, mlen)
        # the same call without per-block values (the kernel may then stop behind a first miss)
        mlen2 = self.t.full((max(n_req, 0),), -7, dtype=self.t.int32, device="cuda")
        self.a.aibx_prefix_match(self.h, h, bo, n_req, h.numel(), None, mlen2)
        assert self.t.equal(mlen, mlen2)
        return self._host_u64(values), mlen.cpu().numpy()


def hip_hash_match(ix, tokens, tok_off, blk_off, block_size, seed, want_hashes=True, want_values=True):
    """aibx_hash_match on host arrays: (hashes or None, values or None, match_len)."""
    t, a = ix.t, ix.a
    d_tok = t.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32).copy()).cuda()
    d_to = t.from_numpy(np.ascontiguousarray(tok_off, dtype=np.int64).copy()).cuda()
    d_bo = t.from_numpy(np.ascontiguousarray(blk_off, dtype=np.int64).copy()).cuda()
    n_req, n = len(tok_off) - 1, int(blk_off[-1])
    h = t.full((n,), -3, dtype=t.int64, device="cuda") if want_hashes else None
    v = t.full((n,), -5, dtype=t.int64, device="cuda") if want_values else None
    m = t.full((max(n_req, 0),), -7, dtype=t.int32, device="cuda")
    a.aibx_hash_match(ix.h, d_tok, d_to, d_bo, n_req, n, block_size, seed, h, v, m)
    u = lambda x: None if x is None else x.cpu().numpy().view(np.uint64)
    return u(h), u(v), m.cpu().numpy()


class HipBackend:
    """The HIP library through its Python binding; host arrays in, host arrays out."""
    name = "hip"

    GUARD = 4096          # canary bytes in front of and behind the pool and the staging buffer
    GUARD_BYTE = 0xC3

    def __init__(self, two_streams=True, device_fill=False):
        import torch
        import paper_2504_03648_amd as aibx
        self.t, self.a = torch, aibx
        self.two_streams = two_streams
        self.device_fill = device_fill      # pool bytes drawn on the GPU (full-size pools)
        self.pool = self.staging = self.geom = self.desc = None
        self._pool_buf = self._staging_buf = None

    def _guarded(self, nbytes):
        """A buffer of nbytes between two canary regions: (whole allocation, the inner view)."""
        G = self.GUARD
        buf = self.t.empty(nbytes + 2 * G, dtype=self.t.uint8, device="cuda")
        buf[:G] = self.GUARD_BYTE
        buf[G + nbytes:] = self.GUARD_BYTE
        return buf, buf[G:G + nbytes]

    def check_guards(self):
        """No call wrote in front of or behind the pool or the staging buffer."""
        G = self.GUARD
        for buf in (self._pool_buf, self._staging_buf):
            if buf is not None:
                assert bool((buf[:G] == self.GUARD_BYTE).all()) and bool((buf[-G:] == self.GUARD_BYTE).all()), \
                    "a copy wrote outside its buffer"

    def _dev(self, x, dtype):
        return self.t.from_numpy(np.ascontiguousarray(x, dtype=dtype).copy()).cuda()

    def block_hash(self, tokens, tok_off, blk_off, block_size, seed):
        t = self._dev(tokens, np.int32)
        to, bo = self._dev(tok_off, np.int64), self._dev(blk_off, np.int64)
        n_req = len(tok_off) - 1
        n_blocks = int(blk_off[-1]) if n_req >= 0 else 0
        out = self.t.full((n_blocks,), -1, dtype=self.t.int64, device="cuda")
        self.a.aibx_block_hash(t, to, bo, n_req, n_blocks, block_size, seed, out)
        return out.cpu().numpy().view(np.uint64)

    def index_create(self, n_slots):
        return HipIndex(n_slots)

    def pool_create(self, geom, kv_dtype, cfg, host_bytes=None):
        """Same bytes as the oracle backend's pool (generated on the host, uploaded)."""
        from workloads import fill_pool_numpy, fill_pool_torch
        if self.pool is not None and self.geom == geom:
            return                              # created ahead of the flow (full-size tests)
        self.geom = geom
        self._pool_buf, self.pool = self._guarded(geom.pool_bytes)
        if host_bytes is None and self.device_fill:
            fill_pool_torch(self.pool, kv_dtype, cfg)
        else:
            if host_bytes is None:
                host_bytes = fill_pool_numpy(geom, kv_dtype, cfg)
            self.pool.copy_(self.t.from_numpy(host_bytes))
        self.desc = self.a.make_pool_desc(self.pool, *geom.as_tuple())

    def staging_create(self, n_blocks, stride):
        self.stride = int(stride)
        self._staging_buf, self.staging = self._guarded(int(n_blocks) * self.stride)
        self.staging.zero_()

    def _ids(self, page_ids, slot_ids):
        p = self._dev(page_ids, np.int32)
        s = None if slot_ids is None else self._dev(slot_ids, np.int32)
        n = p.numel()
        if n:
            smax = n - 1 if slot_ids is None else int(np.max(slot_ids))
            smin = 0 if slot_ids is None else int(np.min(slot_ids))
            assert smin >= 0 and (smax + 1) * self.stride <= self.staging.numel()
        return p, s, n

    def gather(self, page_ids, slot_ids, stream=None):
        p, s, n = self._ids(page_ids, slot_ids)
        bad = self.t.zeros(1, dtype=self.t.int64, device="cuda")
        self.a.aibx_kv_gather(self.desc, p, s, n, self.staging, self.stride, bad, stream)
        return int(bad.item())

    def scatter(self, page_ids, slot_ids, stream=None):
        p, s, n = self._ids(page_ids, slot_ids)
        bad = self.t.zeros(1, dtype=self.t.int64, device="cuda")
        self.a.aibx_kv_scatter(self.desc, p, s, n, self.staging, self.stride, bad, stream)
        return int(bad.item())

    def gather_scatter_pair(self, g_pages, g_slots, s_pages, s_slots):
        """Gather and scatter enqueued on two streams so that they overlap on the GPU."""
        t = self.t
        if not self.two_streams:
            return (self.gather(g_pages, g_slots), self.scatter(s_pages, s_slots))
        gp, gs, gn = self._ids(g_pages, g_slots)
        sp, ss, sn = self._ids(s_pages, s_slots)
        bad = t.zeros(2, dtype=t.int64, device="cuda")
        t.cuda.synchronize()
        sa, sb = t.cuda.Stream(), t.cuda.Stream()
        self.a.aibx_kv_gather(self.desc, gp, gs, gn, self.staging, self.stride, bad[0:1], sa)
        self.a.aibx_kv_scatter(self.desc, sp, ss, sn, self.staging, self.stride, bad[1:2], sb)
        sa.synchronize()
        sb.synchronize()
        b = bad.cpu().numpy()
        return (int(b[0]), int(b[1]))

    def _planes(self):
        g = self.geom
        return self.pool.view(g.n_seg, g.n_pages, g.seg_bytes)

    def fill_pages(self, page_ids, byte):
        ids = self._dev(page_ids, np.int64)
        self._planes()[:, ids, :] = byte

    def read_pages(self, page_ids):
        ids = self._dev(page_ids, np.int64)
        return self._planes()[:, ids, :].permute(1, 0, 2).contiguous().view(len(page_ids), -1).cpu().numpy()

    def read_slots(self, slot_ids):
        ids = self._dev(slot_ids, np.int64)
        st = self.staging.view(-1, self.stride)
        return st[ids, : self.geom.blk_bytes].cpu().numpy()
