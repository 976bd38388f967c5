"""aibx: MI355X-native hot path of a distributed KV cache with prefix-aware routing
(block hashing, prefix match against a GPU-resident index, index insert/evict, paged-KV
gather/scatter). See include/aibx.h for the C ABI; `binding` mirrors it one to one."""
from . import binding
from .binding import (AibxError, PoolDesc, PoolRunsDesc, make_pool_runs_desc, aibx_kv_gather_runs,
                      aibx_kv_scatter_runs, AIBX_NO_VALUE, aibx_version, aibx_hash_version,
                      aibx_block_hash, aibx_index_storage_bytes, aibx_index_create,
                      aibx_index_destroy, aibx_index_clear, aibx_index_insert, aibx_index_evict,
                      aibx_index_count, aibx_index_dump, aibx_index_touch, aibx_index_age,
                      aibx_index_select_victims, aibx_index_stats, aibx_index_rebuild, aibx_prefix_match,
                      aibx_hash_match, aibx_route, aibx_hash_match_route,
                      make_pool_desc,
                      aibx_kv_gather, aibx_kv_scatter, aibx_kv_offload, aibx_kv_onload,
                      aibx_kv_copy_launches, aibx_calib_random_reads, aibx_kv_gather_fill, aibx_kv_scatter_fill)
