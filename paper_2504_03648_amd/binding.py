"""ctypes binding of libaibx.so: the same entry points as include/aibx.h, taking torch tensors
(device memory) and torch streams. Argument marshalling only - every step runs in the library's
HIP kernels. There is no CPU fallback: if the library is missing or a call fails, this raises."""
from __future__ import annotations

import ctypes as C
import os

import torch  # loaded first so that libaibx resolves the same HIP runtime as torch

from .build import LIB_PATH, build_library

AIBX_OK = 0
AIBX_NO_VALUE = 0xFFFFFFFFFFFFFFFF
EXPORTS = [
    "aibx_version", "aibx_hash_version", "aibx_strerror", "aibx_last_hip_error",
    "aibx_block_hash", "aibx_index_storage_bytes", "aibx_index_create", "aibx_index_destroy",
    "aibx_index_clear", "aibx_index_insert", "aibx_index_evict", "aibx_index_count",
    "aibx_index_dump", "aibx_index_touch", "aibx_index_age", "aibx_index_select_victims",
    "aibx_index_stats", "aibx_index_rebuild",
    "aibx_prefix_match", "aibx_hash_match", "aibx_route", "aibx_hash_match_route", "aibx_kv_gather", "aibx_kv_scatter", "aibx_kv_gather_fill", "aibx_kv_scatter_fill", "aibx_kv_copy_launches", "aibx_kv_gather_runs", "aibx_kv_scatter_runs", "aibx_kv_offload", "aibx_kv_onload",
    "aibx_calib_random_reads",
]


class AibxError(RuntimeError):
    def __init__(self, fn: str, status: int):
        lib = load()
        msg = lib.aibx_strerror(status).decode()
        if status == -4:
            msg += ": " + lib.aibx_last_hip_error().decode()
        super().__init__(f"{fn} failed with status {status} ({msg})")
        self.status = status


class PoolRunsDesc(C.Structure):
    """aibx_pool_runs_desc"""
    _fields_ = [("base", C.c_void_p), ("n_seg", C.c_int32), ("n_run", C.c_int32), ("seg_stride", C.c_uint64),
                ("page_stride", C.c_uint64), ("run_stride", C.c_uint64), ("run_bytes", C.c_uint64),
                ("n_pages", C.c_int64)]


class PoolDesc(C.Structure):
    """aibx_pool_desc"""
    _fields_ = [("base", C.c_void_p), ("n_seg", C.c_int32), ("seg_stride", C.c_uint64),
                ("page_stride", C.c_uint64), ("seg_bytes", C.c_uint64), ("n_pages", C.c_int64)]


_lib = None


def load(build_if_missing: bool = True):
    """Loads libaibx.so (building it first only if no built library is there)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise RuntimeError(f"{LIB_PATH} is missing: run __graft_entry__.build() first")
        build_library()
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    lib.aibx_version.restype = C.c_int
    lib.aibx_hash_version.restype = C.c_int
    lib.aibx_strerror.restype = C.c_char_p
    lib.aibx_strerror.argtypes = [C.c_int]
    lib.aibx_last_hip_error.restype = C.c_char_p
    lib.aibx_block_hash.argtypes = [vp, vp, vp, i32, i64, i32, u64, vp, vp]
    lib.aibx_index_storage_bytes.argtypes = [u64, C.POINTER(C.c_size_t)]
    lib.aibx_index_create.argtypes = [vp, C.c_size_t, u64, vp, C.POINTER(vp)]
    lib.aibx_index_destroy.argtypes = [vp]
    lib.aibx_index_clear.argtypes = [vp, vp]
    lib.aibx_index_insert.argtypes = [vp, vp, vp, i64, vp, vp]
    lib.aibx_index_evict.argtypes = [vp, vp, i64, vp, vp, vp]
    lib.aibx_index_count.argtypes = [vp, vp, vp]
    lib.aibx_index_dump.argtypes = [vp, vp, vp, u64, vp, vp]
    lib.aibx_index_stats.argtypes = [vp, vp, vp]
    lib.aibx_index_rebuild.argtypes = [vp, vp, vp, vp]
    lib.aibx_prefix_match.argtypes = [vp, vp, vp, i32, i64, vp, vp, vp]
    lib.aibx_index_touch.argtypes = [vp, vp, i64, C.c_uint32, vp]
    lib.aibx_index_age.argtypes = [vp, vp]
    lib.aibx_index_select_victims.argtypes = [vp, C.c_uint32, C.c_uint32, vp, vp, u64, vp, vp]
    lib.aibx_route.argtypes = [vp, vp, i32, i64, i32, vp, u64, u64, vp, vp, vp]
    lib.aibx_hash_match.argtypes = [vp, vp, vp, vp, i32, i64, i32, u64, vp, vp, vp, vp]
    lib.aibx_hash_match_route.argtypes = [vp, vp, vp, vp, i32, i64, i32, u64, i32, vp, u64, u64, vp, vp, vp]
    for f in (lib.aibx_kv_gather, lib.aibx_kv_scatter):
        f.argtypes = [C.POINTER(PoolDesc), vp, vp, i64, vp, u64, vp, vp]
    for f in (lib.aibx_kv_gather_fill, lib.aibx_kv_scatter_fill):
        f.argtypes = [C.POINTER(PoolDesc), vp, vp, vp, i64, vp, u64, vp, vp]
    lib.aibx_kv_copy_launches.argtypes = [C.POINTER(PoolDesc), i64, vp, vp, vp, i32]
    for f in (lib.aibx_kv_gather_runs, lib.aibx_kv_scatter_runs):
        f.argtypes = [C.POINTER(PoolRunsDesc), vp, vp, i64, vp, u64, vp, vp]
    for f in (lib.aibx_kv_offload, lib.aibx_kv_onload):
        f.argtypes = [C.POINTER(PoolDesc), vp, i64, vp, u64, vp, vp]
    lib.aibx_calib_random_reads.argtypes = [vp, u64, C.c_uint32, C.c_uint32, i64, u64, vp, vp]
    for name in EXPORTS[4:]:
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _p(t, dtype=None):
    """Device pointer of a tensor (None -> NULL)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError("expected a torch.Tensor or None")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("aibx takes contiguous GPU tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _s(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(fn, status):
    if status != AIBX_OK:
        raise AibxError(fn, status)


# torch has no uint64 arithmetic we need; 64-bit keys and values travel as int64 bit patterns.
U64 = torch.int64


def aibx_version() -> int:
    return load().aibx_version()


def aibx_hash_version() -> int:
    return load().aibx_hash_version()


def aibx_block_hash(d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed,
                    d_hash_out, stream=None):
    _check("aibx_block_hash", load().aibx_block_hash(
        _p(d_tokens, torch.int32), _p(d_tok_off, torch.int64), _p(d_blk_off, torch.int64),
        int(n_req), int(n_blocks_total), int(block_size), C.c_uint64(int(seed) & AIBX_NO_VALUE),
        _p(d_hash_out, U64), _s(stream)))


def aibx_index_storage_bytes(n_slots: int) -> int:
    out = C.c_size_t(0)
    _check("aibx_index_storage_bytes", load().aibx_index_storage_bytes(int(n_slots), C.byref(out)))
    return out.value


def aibx_index_create(d_storage, n_slots: int, stream=None) -> C.c_void_p:
    h = C.c_void_p()
    _check("aibx_index_create", load().aibx_index_create(
        _p(d_storage), d_storage.numel() * d_storage.element_size(), int(n_slots), _s(stream),
        C.byref(h)))
    return h


def aibx_index_destroy(index):
    _check("aibx_index_destroy", load().aibx_index_destroy(index))


def aibx_index_clear(index, stream=None):
    _check("aibx_index_clear", load().aibx_index_clear(index, _s(stream)))


def aibx_index_insert(index, d_keys, d_values, n, d_counters3=None, stream=None):
    _check("aibx_index_insert", load().aibx_index_insert(
        index, _p(d_keys, U64), _p(d_values, U64), int(n), _p(d_counters3, U64), _s(stream)))


def aibx_index_evict(index, d_keys, n, d_values_out=None, d_counters2=None, stream=None):
    _check("aibx_index_evict", load().aibx_index_evict(
        index, _p(d_keys, U64), int(n), _p(d_values_out, U64), _p(d_counters2, U64), _s(stream)))


def aibx_index_count(index, d_live_out, stream=None):
    _check("aibx_index_count", load().aibx_index_count(index, _p(d_live_out, U64), _s(stream)))


def aibx_index_stats(index, d_out2, stream=None):
    _check("aibx_index_stats", load().aibx_index_stats(index, _p(d_out2, U64), _s(stream)))


def aibx_index_rebuild(src, dst, d_counters3=None, stream=None):
    _check("aibx_index_rebuild", load().aibx_index_rebuild(src, dst, _p(d_counters3, U64), _s(stream)))


def aibx_index_dump(index, d_keys_out, d_values_out, capacity, d_n_out, stream=None):
    _check("aibx_index_dump", load().aibx_index_dump(
        index, _p(d_keys_out, U64), _p(d_values_out, U64), int(capacity), _p(d_n_out, U64),
        _s(stream)))


def aibx_index_touch(index, d_keys, n, epoch, stream=None):
    _check("aibx_index_touch", load().aibx_index_touch(index, _p(d_keys, U64), int(n), int(epoch), _s(stream)))


def aibx_index_age(index, stream=None):
    _check("aibx_index_age", load().aibx_index_age(index, _s(stream)))


def aibx_index_select_victims(index, protect_count, before_epoch, d_keys_out, d_values_out, capacity,
                              d_n_out, stream=None):
    _check("aibx_index_select_victims", load().aibx_index_select_victims(
        index, int(protect_count), int(before_epoch), _p(d_keys_out, U64), _p(d_values_out, U64),
        int(capacity), _p(d_n_out, U64), _s(stream)))


def aibx_prefix_match(index, d_hashes, d_blk_off, n_req, n_blocks_total, d_values_out,
                      d_match_len, stream=None):
    _check("aibx_prefix_match", load().aibx_prefix_match(
        index, _p(d_hashes, U64), _p(d_blk_off, torch.int64), int(n_req), int(n_blocks_total),
        _p(d_values_out, U64), _p(d_match_len, torch.int32), _s(stream)))


def aibx_hash_match(index, d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed,
                    d_hash_out, d_values_out, d_match_len, stream=None):
    _check("aibx_hash_match", load().aibx_hash_match(
        index, _p(d_tokens, torch.int32), _p(d_tok_off, torch.int64), _p(d_blk_off, torch.int64),
        int(n_req), int(n_blocks_total), int(block_size), C.c_uint64(int(seed) & AIBX_NO_VALUE),
        _p(d_hash_out, U64), _p(d_values_out, U64), _p(d_match_len, torch.int32), _s(stream)))


def aibx_route(d_pod_sets, d_blk_off, n_req, n_blocks_total, n_pods, d_pod_load, threshold_num,
               threshold_den, d_pod_out, d_hit_len_out, stream=None):
    _check("aibx_route", load().aibx_route(
        _p(d_pod_sets, U64), _p(d_blk_off, torch.int64), int(n_req), int(n_blocks_total), int(n_pods),
        _p(d_pod_load, torch.int32), int(threshold_num), int(threshold_den),
        _p(d_pod_out, torch.int32), _p(d_hit_len_out, torch.int32), _s(stream)))


def aibx_hash_match_route(index, d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed, n_pods,
                          d_pod_load, threshold_num, threshold_den, d_pod_out, d_hit_len_out, stream=None):
    _check("aibx_hash_match_route", load().aibx_hash_match_route(
        index, _p(d_tokens, torch.int32), _p(d_tok_off, torch.int64), _p(d_blk_off, torch.int64), int(n_req),
        int(n_blocks_total), int(block_size), int(seed) & 0xFFFFFFFFFFFFFFFF, int(n_pods),
        _p(d_pod_load, torch.int32), int(threshold_num), int(threshold_den), _p(d_pod_out, torch.int32),
        _p(d_hit_len_out, torch.int32), _s(stream)))


def make_pool_desc(d_pool, n_seg, seg_stride, page_stride, seg_bytes, n_pages) -> PoolDesc:
    return PoolDesc(d_pool.data_ptr(), int(n_seg), int(seg_stride), int(page_stride),
                    int(seg_bytes), int(n_pages))


def aibx_kv_gather(pool: PoolDesc, d_page_ids, d_slot_ids, n, d_staging, staging_block_stride,
                   d_bad_page_counter=None, stream=None):
    _check("aibx_kv_gather", load().aibx_kv_gather(
        C.byref(pool), _p(d_page_ids, torch.int32), _p(d_slot_ids, torch.int32), int(n),
        _p(d_staging), int(staging_block_stride), _p(d_bad_page_counter, U64), _s(stream)))


def aibx_kv_scatter(pool: PoolDesc, d_page_ids, d_slot_ids, n, d_staging, staging_block_stride,
                    d_bad_page_counter=None, stream=None):
    _check("aibx_kv_scatter", load().aibx_kv_scatter(
        C.byref(pool), _p(d_page_ids, torch.int32), _p(d_slot_ids, torch.int32), int(n),
        _p(d_staging), int(staging_block_stride), _p(d_bad_page_counter, U64), _s(stream)))


def aibx_kv_gather_fill(pool: PoolDesc, d_page_ids, d_slot_ids, d_seg_fill, n, d_staging, staging_block_stride,
                        d_bad_page_counter=None, stream=None):
    _check("aibx_kv_gather_fill", load().aibx_kv_gather_fill(
        C.byref(pool), _p(d_page_ids, torch.int32), _p(d_slot_ids, torch.int32), _p(d_seg_fill, torch.int32), int(n),
        _p(d_staging), int(staging_block_stride), _p(d_bad_page_counter, U64), _s(stream)))


def aibx_kv_scatter_fill(pool: PoolDesc, d_page_ids, d_slot_ids, d_seg_fill, n, d_staging, staging_block_stride,
                         d_bad_page_counter=None, stream=None):
    _check("aibx_kv_scatter_fill", load().aibx_kv_scatter_fill(
        C.byref(pool), _p(d_page_ids, torch.int32), _p(d_slot_ids, torch.int32), _p(d_seg_fill, torch.int32), int(n),
        _p(d_staging), int(staging_block_stride), _p(d_bad_page_counter, U64), _s(stream)))


def aibx_kv_copy_launches(pool: PoolDesc, n: int, capacity: int = 64):
    """[(first_entry, n_entries, workgroups)] of the launches a gather/scatter of n entries makes."""
    first, cnt, grid = (C.c_int64 * capacity)(), (C.c_int64 * capacity)(), (C.c_uint32 * capacity)()
    k = load().aibx_kv_copy_launches(C.byref(pool), int(n), first, cnt, grid, capacity)
    if k < 0:
        raise AibxError("aibx_kv_copy_launches", k)
    return [(first[i], cnt[i], grid[i]) for i in range(min(k, capacity))], k


def make_pool_runs_desc(pool_tensor, n_seg, n_run, seg_stride, page_stride, run_stride, run_bytes, n_pages):
    return PoolRunsDesc(pool_tensor.data_ptr(), int(n_seg), int(n_run), int(seg_stride), int(page_stride),
                        int(run_stride), int(run_bytes), int(n_pages))


def aibx_kv_gather_runs(pool: PoolRunsDesc, d_page_ids, d_slot_ids, n, d_staging, staging_block_stride,
                        d_bad_page_counter=None, stream=None):
    _check("aibx_kv_gather_runs", load().aibx_kv_gather_runs(
        C.byref(pool), _p(d_page_ids, torch.int32), _p(d_slot_ids, torch.int32), int(n),
        _p(d_staging), int(staging_block_stride), _p(d_bad_page_counter, U64), _s(stream)))


def aibx_kv_scatter_runs(pool: PoolRunsDesc, d_page_ids, d_slot_ids, n, d_staging, staging_block_stride,
                         d_bad_page_counter=None, stream=None):
    _check("aibx_kv_scatter_runs", load().aibx_kv_scatter_runs(
        C.byref(pool), _p(d_page_ids, torch.int32), _p(d_slot_ids, torch.int32), int(n),
        _p(d_staging), int(staging_block_stride), _p(d_bad_page_counter, U64), _s(stream)))


def _host_ptr(t):
    """Address of a host tensor; the library itself refuses memory that is not pinned."""
    if not isinstance(t, torch.Tensor) or t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous host tensor")
    return C.c_void_p(t.data_ptr())


def aibx_kv_offload(pool: PoolDesc, d_page_ids, n, h_dst, host_block_stride, d_bad_page_counter=None, stream=None):
    _check("aibx_kv_offload", load().aibx_kv_offload(
        C.byref(pool), _p(d_page_ids, torch.int32), int(n), _host_ptr(h_dst), int(host_block_stride),
        _p(d_bad_page_counter, U64), _s(stream)))


def aibx_kv_onload(pool: PoolDesc, d_page_ids, n, h_src, host_block_stride, d_bad_page_counter=None, stream=None):
    _check("aibx_kv_onload", load().aibx_kv_onload(
        C.byref(pool), _p(d_page_ids, torch.int32), int(n), _host_ptr(h_src), int(host_block_stride),
        _p(d_bad_page_counter, U64), _s(stream)))


def aibx_calib_random_reads(d_table, table_bytes, line_bytes, read_bytes, n_reads, seed, d_sink, stream=None):
    _check("aibx_calib_random_reads", load().aibx_calib_random_reads(
        _p(d_table), int(table_bytes), int(line_bytes), int(read_bytes), int(n_reads), int(seed),
        _p(d_sink, U64), _s(stream)))
