// Paged-KV gather / scatter (Section 3.2.5 of the paper: moving KV blocks between the engine's
// paged memory and the cache's contiguous buffers). Pure byte streaming, HBM-bound.
//
// Work decomposition: a tile is (entry i, segment s, chunk c) - kChunkVecs*16*256 contiguous
// bytes of one segment. blockIdx.x walks (s, c) of one block, so neighbouring workgroups stream
// neighbouring staging bytes; blockIdx.y walks the entries. Every lane moves 16 bytes per access
// and keeps all its loads of a tile in flight before the first store.
#include "common.h"

namespace aibx {
namespace {

constexpr int kCopyThreads = 256;

struct CopyArgs {
  unsigned char* pool;
  unsigned char* staging;
  const int32_t* page_ids;
  const int32_t* slot_ids;   // nullable
  u64* bad_page;             // nullable
  u64 seg_stride, page_stride, seg_bytes, staging_stride;
  int64_t n, n_pages;
  u32 chunks_per_seg;
};

typedef __attribute__((ext_vector_type(4))) u32 vec16;

template <bool kGather, int kVecs>
__global__ __launch_bounds__(kCopyThreads) void kv_copy_kernel(CopyArgs a) {
  constexpr u64 kChunkBytes = (u64)kVecs * 16 * kCopyThreads;
  const u32 s = blockIdx.x / a.chunks_per_seg;
  const u32 c = blockIdx.x - s * a.chunks_per_seg;
  const u64 off0 = (u64)c * kChunkBytes + (u64)threadIdx.x * 16;
  for (int64_t i = blockIdx.y; i < a.n; i += gridDim.y) {
    const int64_t p = a.page_ids[i];
    if (p < 0) continue;
    if (p >= a.n_pages) {
      if (blockIdx.x == 0 && threadIdx.x == 0 && a.bad_page) atomicAdd((unsigned long long*)a.bad_page, 1ull);
      continue;
    }
    const int64_t q = a.slot_ids ? (int64_t)a.slot_ids[i] : i;
    unsigned char* in_pool = a.pool + (u64)s * a.seg_stride + (u64)p * a.page_stride;
    unsigned char* in_stage = a.staging + (u64)q * a.staging_stride + (u64)s * a.seg_bytes;
    const unsigned char* src = kGather ? in_pool : in_stage;
    unsigned char* dst = kGather ? in_stage : in_pool;
    vec16 v[kVecs];
#pragma unroll
    for (int k = 0; k < kVecs; ++k) {
      const u64 off = off0 + (u64)k * 16 * kCopyThreads;
      if (off < a.seg_bytes) v[k] = __builtin_nontemporal_load(reinterpret_cast<const vec16*>(src + off));
    }
#pragma unroll
    for (int k = 0; k < kVecs; ++k) {
      const u64 off = off0 + (u64)k * 16 * kCopyThreads;
      if (off < a.seg_bytes) __builtin_nontemporal_store(v[k], reinterpret_cast<vec16*>(dst + off));
    }
  }
}

template <bool kGather>
int launch_copy(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                int64_t n, void* d_staging, u64 stride, u64* d_bad, void* stream) {
  if (n < 0) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!pool || !pool->base || !d_page_ids || !d_staging) return AIBX_ERR_INVALID_ARG;
  if (pool->n_seg < 1 || pool->seg_bytes == 0 || pool->n_pages < 0) return AIBX_ERR_INVALID_ARG;
  if (pool->page_stride < pool->seg_bytes) return AIBX_ERR_INVALID_ARG;
  const u64 blk_bytes = (u64)pool->n_seg * pool->seg_bytes;
  if (blk_bytes / pool->seg_bytes != (u64)pool->n_seg || stride < blk_bytes) return AIBX_ERR_INVALID_ARG;
  if (!aligned(pool->base, 16) || !aligned(d_staging, 16) || pool->seg_bytes % 16 || pool->seg_stride % 16 ||
      pool->page_stride % 16 || stride % 16)
    return AIBX_ERR_ALIGN;
  if (!aligned(d_page_ids, 4) || !aligned(d_slot_ids, 4) || !aligned(d_bad, 8)) return AIBX_ERR_ALIGN;

  // Chunk size: 16 KiB per workgroup unless the segment divides better into 8 or 4 KiB pieces.
  int vecs = 4;
  if (pool->seg_bytes % (4 * 4096) != 0) {
    if (pool->seg_bytes % (2 * 4096) == 0) vecs = 2;
    else if (pool->seg_bytes < 2 * 4096) vecs = 1;
  }
  const u64 chunk = (u64)vecs * 16 * kCopyThreads;
  const u64 cps = (pool->seg_bytes + chunk - 1) / chunk;
  const u64 gx = cps * (u64)pool->n_seg;
  if (gx > 0x7FFFFFFFull) return AIBX_ERR_UNSUPPORTED;

  CopyArgs a;
  a.pool = static_cast<unsigned char*>(pool->base);
  a.staging = static_cast<unsigned char*>(d_staging);
  a.page_ids = d_page_ids;
  a.slot_ids = d_slot_ids;
  a.bad_page = d_bad;
  a.seg_stride = pool->seg_stride;
  a.page_stride = pool->page_stride;
  a.seg_bytes = pool->seg_bytes;
  a.staging_stride = stride;
  a.n = n;
  a.n_pages = pool->n_pages;
  a.chunks_per_seg = (u32)cps;
  dim3 grid((u32)gx, (u32)(n < 65535 ? n : 65535));
  hipStream_t st = as_stream(stream);
  switch (vecs) {
    case 1: kv_copy_kernel<kGather, 1><<<grid, kCopyThreads, 0, st>>>(a); break;
    case 2: kv_copy_kernel<kGather, 2><<<grid, kCopyThreads, 0, st>>>(a); break;
    default: kv_copy_kernel<kGather, 4><<<grid, kCopyThreads, 0, st>>>(a); break;
  }
  return launch_status();
}

}  // namespace
}  // namespace aibx

extern "C" {

int aibx_kv_gather(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                   int64_t n, void* d_staging, uint64_t staging_block_stride,
                   uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_copy<true>(pool, d_page_ids, d_slot_ids, n, d_staging, staging_block_stride,
                                 d_bad_page_counter, stream);
}

int aibx_kv_scatter(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                    int64_t n, const void* d_staging, uint64_t staging_block_stride,
                    uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_copy<false>(pool, d_page_ids, d_slot_ids, n, const_cast<void*>(d_staging),
                                  staging_block_stride, d_bad_page_counter, stream);
}

}  // extern "C"
