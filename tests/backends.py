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
        assert n == 0 or (slots.min() >= 0 and (slots.max() + 1) * self.stride <= len(self.staging))

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
