"""CPU oracle for the KV-cache hot path - TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy wrapper over ``aibx_oracle.cpp`` (plain single-threaded C++). Only the tests,
the smoke check and the benchmark's CPU-baseline leg may import this package; the product
package never does, and the two share no code. All arrays are host numpy arrays.

The operations follow the problem stated in the paper's Section 3.2.5 (Distributed KV Cache
Pool) and the prefix-cache-aware policy of Section 3.2.2; the concrete rules (hash, index
semantics, match rule, copy layout) are written out in ``aibx_oracle.cpp``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aibx_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

NO_VALUE = np.uint64(0xFFFFFFFFFFFFFFFF)


SANITIZE = os.environ.get("AIBX_ORACLE_SANITIZE", "") not in ("", "0")
if SANITIZE:                       # a second library, so that the plain one is never replaced by it
    _LIB = os.path.join(_HERE, "liboracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only). Returns the library path. With
    AIBX_ORACLE_SANITIZE=1 in the environment the build is instrumented with AddressSanitizer and
    UndefinedBehaviorSanitizer (any finding aborts the process); loading it into Python needs the
    ASan runtime preloaded, which tests/test_oracle_sanitized.py arranges for a child process."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O2"]
        if SANITIZE:
            flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                     "-fno-sanitize-recover=all"]
        subprocess.check_call(["g++", *flags, "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB + ".tmp", _SRC])
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


class _PoolDesc(C.Structure):
    _fields_ = [("base", C.c_void_p), ("n_seg", C.c_int32), ("seg_stride", C.c_uint64),
                ("page_stride", C.c_uint64), ("seg_bytes", C.c_uint64), ("n_pages", C.c_int64)]


class _PoolRunsDesc(C.Structure):
    _fields_ = [("base", C.c_void_p), ("n_seg", C.c_int32), ("n_run", C.c_int32), ("seg_stride", C.c_uint64),
                ("page_stride", C.c_uint64), ("run_stride", C.c_uint64), ("run_bytes", C.c_uint64),
                ("n_pages", C.c_int64)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        lib.orc_index_create.restype = C.c_void_p
        lib.orc_index_create.argtypes = [C.c_uint64]
        lib.orc_index_destroy.argtypes = [C.c_void_p]
        lib.orc_index_destroy.restype = None
        lib.orc_index_clear.argtypes = [C.c_void_p]
        lib.orc_index_clear.restype = None
        lib.orc_index_count.argtypes = [C.c_void_p]
        lib.orc_index_count.restype = C.c_uint64
        lib.orc_index_dump.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64]
        lib.orc_index_dump.restype = C.c_uint64
        lib.orc_block_hash.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                       C.c_int32, C.c_uint64, C.c_void_p]
        lib.orc_index_insert.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        lib.orc_index_evict.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.orc_prefix_match.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                         C.c_void_p, C.c_void_p]
        for f in (lib.orc_kv_gather, lib.orc_kv_scatter):
            f.argtypes = [C.POINTER(_PoolDesc), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                          C.c_uint64, C.c_void_p]
        for f in (lib.orc_kv_gather_fill, lib.orc_kv_scatter_fill):
            f.argtypes = [C.POINTER(_PoolDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                          C.c_uint64, C.c_void_p]
        for f in (lib.orc_kv_gather_runs, lib.orc_kv_scatter_runs):
            f.argtypes = [C.POINTER(_PoolRunsDesc), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                          C.c_uint64, C.c_void_p]
        lib.orc_index_touch.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_uint32]
        lib.orc_index_rebuild.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_index_age.argtypes = [C.c_void_p]
        lib.orc_index_age.restype = None
        lib.orc_index_select_victims.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p,
                                                 C.c_uint64]
        lib.orc_index_select_victims.restype = C.c_uint64
        lib.orc_route.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_uint64,
                                  C.c_uint64, C.c_void_p, C.c_void_p]
        for f in (lib.orc_finalise, lib.orc_avoid_reserved):
            f.argtypes = [C.c_uint64]
            f.restype = C.c_uint64
        lib.orc_token_term.argtypes = [C.c_int32, C.c_int64]
        lib.orc_token_term.restype = C.c_uint64
        _lib = lib
    return _lib


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def finalise(x: int) -> int:
    return int(_load().orc_finalise(C.c_uint64(x & 0xFFFFFFFFFFFFFFFF)))


def token_term(token: int, i: int) -> int:
    return int(_load().orc_token_term(int(token), int(i)))


def avoid_reserved(h: int) -> int:
    return int(_load().orc_avoid_reserved(C.c_uint64(h & 0xFFFFFFFFFFFFFFFF)))


def block_hash(tokens, tok_off, blk_off, block_size: int, seed: int = 0) -> np.ndarray:
    """Chained per-block prefix hashes, uint64[blk_off[-1]]."""
    tokens = _arr(tokens, np.int32)
    tok_off = _arr(tok_off, np.int64)
    blk_off = _arr(blk_off, np.int64)
    n_req = len(tok_off) - 1
    n_blocks = int(blk_off[-1]) if n_req >= 0 and len(blk_off) else 0
    out = np.empty(n_blocks, dtype=np.uint64)
    rc = _load().orc_block_hash(_ptr(tokens), _ptr(tok_off), _ptr(blk_off), n_req, n_blocks,
                                int(block_size), C.c_uint64(int(seed) & 0xFFFFFFFFFFFFFFFF),
                                _ptr(out))
    if rc != 0:
        raise ValueError(f"orc_block_hash: invalid arguments (rc={rc})")
    return out


class Index:
    """Abstract key->value map with a capacity (see aibx_oracle.cpp)."""

    def __init__(self, n_slots: int):
        self._lib = _load()
        self.n_slots = int(n_slots)
        self._h = self._lib.orc_index_create(self.n_slots)
        self.counters_insert = np.zeros(3, dtype=np.uint64)   # inserted, updated, full
        self.counters_evict = np.zeros(2, dtype=np.uint64)    # evicted, missing

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.orc_index_destroy(self._h)
            self._h = None

    def clear(self):
        self._lib.orc_index_clear(self._h)

    def insert(self, keys, values):
        keys = _arr(keys, np.uint64)
        values = _arr(values, np.uint64)
        assert keys.shape == values.shape
        rc = self._lib.orc_index_insert(self._h, _ptr(keys), _ptr(values), len(keys),
                                        _ptr(self.counters_insert))
        assert rc == 0

    def evict(self, keys) -> np.ndarray:
        keys = _arr(keys, np.uint64)
        out = np.empty(len(keys), dtype=np.uint64)
        rc = self._lib.orc_index_evict(self._h, _ptr(keys), len(keys), _ptr(out),
                                       _ptr(self.counters_evict))
        assert rc == 0
        return out

    def count(self) -> int:
        return int(self._lib.orc_index_count(self._h))

    def dump(self):
        """(keys, values) sorted by key."""
        n = self.count()
        k = np.empty(n, dtype=np.uint64)
        v = np.empty(n, dtype=np.uint64)
        m = self._lib.orc_index_dump(self._h, _ptr(k), _ptr(v), n)
        assert m == n
        return k, v

    def rebuild_into(self, dst: "Index") -> np.ndarray:
        """dst <- this index's keys, values and usage; returns {moved, 0, dropped}."""
        c = np.zeros(3, dtype=np.uint64)
        rc = self._lib.orc_index_rebuild(self._h, dst._h, _ptr(c))
        assert rc == 0
        return c

    def touch(self, keys, epoch: int):
        keys = _arr(keys, np.uint64)
        rc = self._lib.orc_index_touch(self._h, _ptr(keys), len(keys), int(epoch))
        assert rc == 0

    def age(self):
        self._lib.orc_index_age(self._h)

    def select_victims(self, protect_count: int, before_epoch: int):
        """(keys, values) of the victims, sorted by key."""
        cap = self.count()
        k = np.empty(cap, dtype=np.uint64)
        v = np.empty(cap, dtype=np.uint64)
        m = int(self._lib.orc_index_select_victims(self._h, int(protect_count), int(before_epoch),
                                                   _ptr(k), _ptr(v), cap))
        return k[:m].copy(), v[:m].copy()

    def match(self, hashes, blk_off):
        """(values uint64[N], match_len int32[R]) under the first-miss rule."""
        hashes = _arr(hashes, np.uint64)
        blk_off = _arr(blk_off, np.int64)
        n_req = len(blk_off) - 1
        values = np.empty(len(hashes), dtype=np.uint64)
        mlen = np.empty(max(n_req, 0), dtype=np.int32)
        rc = self._lib.orc_prefix_match(self._h, _ptr(hashes), _ptr(blk_off), n_req, len(hashes),
                                        _ptr(values), _ptr(mlen))
        assert rc == 0
        return values, mlen


def route(pod_sets, blk_off, n_pods: int, pod_load, thr_num: int, thr_den: int):
    """(pod int32[R], hit_len int32[R]): prefix-cache-aware choice with least-request fallback."""
    pod_sets = _arr(pod_sets, np.uint64)
    blk_off = _arr(blk_off, np.int64)
    pod_load = _arr(pod_load, np.int32)
    assert len(pod_load) == n_pods
    n_req = len(blk_off) - 1
    pod = np.empty(max(n_req, 0), dtype=np.int32)
    hit = np.empty(max(n_req, 0), dtype=np.int32)
    rc = _load().orc_route(_ptr(pod_sets), _ptr(blk_off), n_req, int(n_pods), _ptr(pod_load),
                           C.c_uint64(thr_num), C.c_uint64(thr_den), _ptr(pod), _ptr(hit))
    if rc != 0:
        raise ValueError(f"orc_route: invalid arguments (rc={rc})")
    return pod, hit


def _desc(pool: np.ndarray, n_seg, seg_stride, page_stride, seg_bytes, n_pages):
    assert pool.dtype == np.uint8 and pool.flags["C_CONTIGUOUS"]
    return _PoolDesc(pool.ctypes.data, int(n_seg), int(seg_stride), int(page_stride),
                     int(seg_bytes), int(n_pages))


def kv_gather(pool, geom, page_ids, slot_ids, staging, stride) -> int:
    """pool -> staging. ``geom`` = (n_seg, seg_stride, page_stride, seg_bytes, n_pages); pool and
    staging are uint8 arrays (staging is written in place). Returns the bad-page count."""
    return _copy(_load().orc_kv_gather, pool, geom, page_ids, slot_ids, staging, stride)


def kv_scatter(pool, geom, page_ids, slot_ids, staging, stride) -> int:
    """staging -> pool (pool is written in place). Returns the bad-page count."""
    return _copy(_load().orc_kv_scatter, pool, geom, page_ids, slot_ids, staging, stride)


def kv_gather_fill(pool, geom, page_ids, slot_ids, seg_fill, staging, stride) -> int:
    """pool -> staging, entry i moving only the first seg_fill[i] bytes of each of its segments
    (clamped to [0, seg_bytes], rounded down to a multiple of 16). Returns the bad-page count."""
    return _copy_fill(_load().orc_kv_gather_fill, pool, geom, page_ids, slot_ids, seg_fill, staging, stride)


def kv_scatter_fill(pool, geom, page_ids, slot_ids, seg_fill, staging, stride) -> int:
    return _copy_fill(_load().orc_kv_scatter_fill, pool, geom, page_ids, slot_ids, seg_fill, staging, stride)


def _copy_fill(fn, pool, geom, page_ids, slot_ids, seg_fill, staging, stride):
    page_ids = _arr(page_ids, np.int32)
    slot_ids = None if slot_ids is None else _arr(slot_ids, np.int32)
    seg_fill = None if seg_fill is None else _arr(seg_fill, np.int32)
    assert seg_fill is None or len(seg_fill) == len(page_ids)
    assert staging.dtype == np.uint8 and staging.flags["C_CONTIGUOUS"]
    d = _desc(pool, *geom)
    bad = np.zeros(1, dtype=np.uint64)
    rc = fn(C.byref(d), _ptr(page_ids), _ptr(slot_ids), _ptr(seg_fill), len(page_ids), _ptr(staging),
            int(stride), _ptr(bad))
    if rc != 0:
        raise ValueError(f"oracle copy: invalid arguments (rc={rc})")
    return int(bad[0])


def _copy(fn, pool, geom, page_ids, slot_ids, staging, stride):
    page_ids = _arr(page_ids, np.int32)
    slot_ids = None if slot_ids is None else _arr(slot_ids, np.int32)
    assert staging.dtype == np.uint8 and staging.flags["C_CONTIGUOUS"]
    d = _desc(pool, *geom)
    bad = np.zeros(1, dtype=np.uint64)
    rc = fn(C.byref(d), _ptr(page_ids), _ptr(slot_ids), len(page_ids), _ptr(staging),
            int(stride), _ptr(bad))
    if rc != 0:
        raise ValueError(f"oracle copy: invalid arguments (rc={rc})")
    return int(bad[0])


def _copy_runs(fn, pool, geom, page_ids, slot_ids, staging, stride):
    page_ids = _arr(page_ids, np.int32)
    slot_ids = None if slot_ids is None else _arr(slot_ids, np.int32)
    assert pool.dtype == np.uint8 and pool.flags["C_CONTIGUOUS"]
    assert staging.dtype == np.uint8 and staging.flags["C_CONTIGUOUS"]
    n_seg, n_run, seg_stride, page_stride, run_stride, run_bytes, n_pages = (int(x) for x in geom)
    d = _PoolRunsDesc(pool.ctypes.data, n_seg, n_run, seg_stride, page_stride, run_stride, run_bytes, n_pages)
    bad = np.zeros(1, dtype=np.uint64)
    rc = fn(C.byref(d), _ptr(page_ids), _ptr(slot_ids), len(page_ids), _ptr(staging), int(stride), _ptr(bad))
    if rc != 0:
        raise ValueError(f"oracle copy: invalid arguments (rc={rc})")
    return int(bad[0])


def kv_gather_runs(pool, geom, page_ids, slot_ids, staging, stride) -> int:
    """pool -> staging for a pool whose segments are runs: ``geom`` = (n_seg, n_run, seg_stride,
    page_stride, run_stride, run_bytes, n_pages). Returns the bad-page count."""
    return _copy_runs(_load().orc_kv_gather_runs, pool, geom, page_ids, slot_ids, staging, stride)


def kv_scatter_runs(pool, geom, page_ids, slot_ids, staging, stride) -> int:
    return _copy_runs(_load().orc_kv_scatter_runs, pool, geom, page_ids, slot_ids, staging, stride)
