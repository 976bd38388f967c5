// Paged-KV gather / scatter with a layout conversion (Section 3.2.5 of the paper: KV reuse across
// engines; here for engines whose pages are laid out differently). A segment of the staging block
// is contiguous, in the pool it is n_run runs of run_bytes at a stride - a token-major page
// [token][layer][bytes] seen from a layer-major staging block.
//
// Same shape as the plain copy kernel: one workgroup per 4 KiB tile of a staging segment, one
// 16-byte vector per lane, XCD x streams the x-th eighth of the staging bytes. The only addition is
// the lane's run index (one 32-bit division by run_bytes): a run is a multiple of 16 bytes, so a
// vector never straddles two runs. The contiguous side keeps full 4 KiB tiles; the pool side moves
// in pieces of run_bytes.
#include "common.h"

namespace aibx {
namespace {

struct RunCopyArgs {
  unsigned char* pool;
  unsigned char* staging;
  u64* bad_page;  // nullable
  u64 seg_stride, page_stride, run_stride, staging_stride;
  u32 run_bytes, seg_bytes;  // seg_bytes = n_run * run_bytes < 2^31
  int64_t n_pages;
  int64_t first_entry;
  u32 chunks_per_seg;
  u32 tiles_per_block;
  u32 total_tiles;
  u32 tiles_per_xcd;
};

typedef __attribute__((ext_vector_type(4))) u32 vec16;
constexpr int kRunThreads = 256;

template <bool kGather>
__global__ __launch_bounds__(kRunThreads) void kv_copy_runs_kernel(RunCopyArgs a,
                                                                    const int32_t* __restrict__ page_ids,
                                                                    const int32_t* __restrict__ slot_ids) {
  const u32 tile = (blockIdx.x & 7u) * a.tiles_per_xcd + (blockIdx.x >> 3);
  if (tile >= a.total_tiles) return;
  const u32 e = tile / a.tiles_per_block;
  const u32 tile_in_block = tile - e * a.tiles_per_block;
  const int64_t i = a.first_entry + e;
  const int64_t p = page_ids[i];
  const int64_t q = slot_ids ? (int64_t)slot_ids[i] : i;
  if (p < 0) return;  // hole
  if (p >= a.n_pages) {
    if (tile_in_block == 0 && threadIdx.x == 0 && a.bad_page) atomicAdd((unsigned long long*)a.bad_page, 1ull);
    return;
  }
  const u32 s = tile_in_block / a.chunks_per_seg;
  const u32 c = tile_in_block - s * a.chunks_per_seg;
  const u32 off = (c * kRunThreads + threadIdx.x) * 16;  // byte offset inside the staging segment
  if (off >= a.seg_bytes) return;                        // ragged last chunk of a segment
  const u32 t = off / a.run_bytes;                       // run, and offset inside it
  const u32 w = off - t * a.run_bytes;
  vec16* in_pool = reinterpret_cast<vec16*>(a.pool + (u64)p * a.page_stride + (u64)s * a.seg_stride +
                                            (u64)t * a.run_stride + w);
  vec16* in_stage = reinterpret_cast<vec16*>(a.staging + (u64)q * a.staging_stride + (u64)s * a.seg_bytes + off);
  if (kGather) {
    const vec16 v = __builtin_nontemporal_load(in_pool);
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(in_stage), "v"(v) : "memory");
  } else {
    const vec16 v = __builtin_nontemporal_load(in_stage);
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" ::"v"(in_pool), "v"(v) : "memory");
  }
}

template <bool kGather>
int launch_copy_runs(const aibx_pool_runs_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                     int64_t n, void* d_staging, u64 stride, u64* d_bad, void* stream) {
  if (n < 0) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!pool || !pool->base || !d_page_ids || !d_staging) return AIBX_ERR_INVALID_ARG;
  if (pool->n_seg < 1 || pool->n_run < 1 || pool->run_bytes == 0 || pool->n_pages < 0) return AIBX_ERR_INVALID_ARG;
  const u64 seg_bytes = (u64)pool->n_run * pool->run_bytes;
  if (seg_bytes / pool->run_bytes != (u64)pool->n_run || seg_bytes >= (1ull << 31)) return AIBX_ERR_UNSUPPORTED;
  const u64 blk_bytes = (u64)pool->n_seg * seg_bytes;
  if (stride < blk_bytes) return AIBX_ERR_INVALID_ARG;
  if (pool->n_run > 1 && pool->run_stride < pool->run_bytes) return AIBX_ERR_INVALID_ARG;
  if (!aligned(pool->base, 16) || !aligned(d_staging, 16) || pool->run_bytes % 16 || pool->seg_stride % 16 ||
      pool->page_stride % 16 || pool->run_stride % 16 || stride % 16)
    return AIBX_ERR_ALIGN;
  if (!aligned(d_page_ids, 4) || !aligned(d_slot_ids, 4) || !aligned(d_bad, 8)) return AIBX_ERR_ALIGN;

  const u64 tile_bytes = (u64)kRunThreads * 16;
  const u64 cps = (seg_bytes + tile_bytes - 1) / tile_bytes;
  const u64 tpb = cps * (u64)pool->n_seg;
  const int64_t max_entries = max_entries_per_launch(tpb, kRunThreads);
  if (max_entries < 1) return AIBX_ERR_UNSUPPORTED;  // one block alone exceeds a launch

  RunCopyArgs a;
  a.pool = static_cast<unsigned char*>(pool->base);
  a.staging = static_cast<unsigned char*>(d_staging);
  a.bad_page = d_bad;
  a.seg_stride = pool->seg_stride;
  a.page_stride = pool->page_stride;
  a.run_stride = pool->run_stride;
  a.staging_stride = stride;
  a.run_bytes = (u32)pool->run_bytes;
  a.seg_bytes = (u32)seg_bytes;
  a.n_pages = pool->n_pages;
  a.chunks_per_seg = (u32)cps;
  a.tiles_per_block = (u32)tpb;
  hipStream_t st = as_stream(stream);
  for (int64_t first = 0; first < n; first += max_entries) {
    const int64_t n_here = (n - first) < max_entries ? (n - first) : max_entries;
    a.first_entry = first;
    a.total_tiles = (u32)((u64)n_here * tpb);
    a.tiles_per_xcd = (a.total_tiles + 7) / 8;
    kv_copy_runs_kernel<kGather><<<dim3(a.tiles_per_xcd * 8), kRunThreads, 0, st>>>(a, d_page_ids, d_slot_ids);
    const int rc = launch_status();
    if (rc != AIBX_OK) return rc;
  }
  return AIBX_OK;
}

}  // namespace
}  // namespace aibx

extern "C" {

int aibx_kv_gather_runs(const aibx_pool_runs_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                        int64_t n, void* d_staging, uint64_t staging_block_stride, uint64_t* d_bad_page_counter,
                        void* stream) {
  return aibx::launch_copy_runs<true>(pool, d_page_ids, d_slot_ids, n, d_staging, staging_block_stride,
                                      d_bad_page_counter, stream);
}

int aibx_kv_scatter_runs(const aibx_pool_runs_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                         int64_t n, const void* d_staging, uint64_t staging_block_stride,
                         uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_copy_runs<false>(pool, d_page_ids, d_slot_ids, n, const_cast<void*>(d_staging),
                                       staging_block_stride, d_bad_page_counter, stream);
}

}  // extern "C"
