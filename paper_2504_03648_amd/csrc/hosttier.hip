// Host-tier leg of offload / onload (Section 3.2.5 of the paper: the cache pool lives in DRAM and
// exchanges KV with the colocated engine through host memory).
//
// One kernel moves pages straight between the paged pool in HBM and pinned host memory, which the
// GPU addresses directly: no staging buffer, no second stream, no events. The link to the host is
// slower than HBM by two orders of magnitude, so the kernel is sized for the link, not for the
// chip: a fixed, small grid whose workgroups walk the tiles in order. Two things decide how it
// behaves beside other kernels, both measured on MI355X with an HBM-bound copy running on a
// second stream (6.5 TB/s alone):
//  - Stores to host memory are written through at system scope. Plain (or non-temporal) stores
//    reach the same link rate, but the copy on the other stream then stalls for milliseconds at a
//    time (single launches at 0.2-1.3 TB/s); with system-scope stores it never dropped below 6.1.
//  - 32 workgroups. The link is full from about 24-32 workgroups on (55.8 GB/s towards the host,
//    54.6-57.2 GB/s from it; one large library copy of pinned memory: 57.1 / 57.6), and every
//    further workgroup only adds requests that wait for the link inside the memory system: at 32
//    the copy beside it keeps 96 % of its rate, at 48 it loses 7-28 %, at 128 most of it.
// A pipeline of gather launches and chunked library copies on two streams reached the same rate at
// best, and half of it in runs where the runtime's chunk copies slowed down.
#include "common.h"

namespace aibx {
namespace {

struct HostCopyArgs {
  unsigned char* pool;
  unsigned char* host;  // the GPU's view of the pinned host buffer
  u64* bad_page;        // nullable
  u64 seg_stride, page_stride, seg_bytes, host_stride;
  int64_t n_pages;
  u64 total_tiles;      // n * tiles_per_block
  u32 chunks_per_seg;
  u32 tiles_per_block;  // chunks_per_seg * n_seg
};

constexpr int kHostThreads = 256;          // one 16-byte vector per lane: 4 KiB tiles
constexpr unsigned kHostWorkgroups = 32;   // fills the link and leaves the memory system to others, see above

typedef __attribute__((ext_vector_type(4))) u32 vec16;

// Tile t = (entry i, segment s, chunk c) in that order, so neighbouring workgroups write
// neighbouring 4 KiB pieces of a host block. kToHost: pool -> host (offload), else host -> pool.
template <bool kToHost>
__global__ __launch_bounds__(kHostThreads) void kv_host_copy_kernel(HostCopyArgs a,
                                                                     const int32_t* __restrict__ page_ids) {
  for (u64 t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const u64 i = t / a.tiles_per_block;
    const u32 tile_in_block = (u32)(t - i * a.tiles_per_block);
    const int64_t p = page_ids[i];
    if (p < 0) continue;  // hole
    if (p >= a.n_pages) {
      if (tile_in_block == 0 && threadIdx.x == 0 && a.bad_page) atomicAdd((unsigned long long*)a.bad_page, 1ull);
      continue;
    }
    const u32 s = tile_in_block / a.chunks_per_seg;
    const u32 c = tile_in_block - s * a.chunks_per_seg;
    const u64 off = ((u64)c * kHostThreads + threadIdx.x) * 16;
    if (off >= a.seg_bytes) continue;  // ragged last chunk of a segment
    vec16* in_pool = reinterpret_cast<vec16*>(a.pool + (u64)s * a.seg_stride + (u64)p * a.page_stride + off);
    vec16* in_host = reinterpret_cast<vec16*>(a.host + i * a.host_stride + (u64)s * a.seg_bytes + off);
    if (kToHost) {
      const vec16 v = *in_pool;
      asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(in_host), "v"(v) : "memory");
    } else {
      *in_pool = *in_host;
    }
  }
}

template <bool kToHost>
int launch_host_copy(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, void* h_buf, u64 host_stride,
                     u64* d_bad, void* stream) {
  if (n < 0) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!pool || !pool->base || !d_page_ids || !h_buf) return AIBX_ERR_INVALID_ARG;
  if (pool->n_seg < 1 || pool->seg_bytes == 0 || pool->n_pages < 0) return AIBX_ERR_INVALID_ARG;
  if (pool->page_stride < pool->seg_bytes) return AIBX_ERR_INVALID_ARG;
  const u64 blk_bytes = (u64)pool->n_seg * pool->seg_bytes;
  if (blk_bytes / pool->seg_bytes != (u64)pool->n_seg || host_stride < blk_bytes) return AIBX_ERR_INVALID_ARG;
  if (!aligned(pool->base, 16) || !aligned(h_buf, 16) || pool->seg_bytes % 16 || pool->seg_stride % 16 ||
      pool->page_stride % 16 || host_stride % 16)
    return AIBX_ERR_ALIGN;
  if (!aligned(d_page_ids, 4) || !aligned(d_bad, 8)) return AIBX_ERR_ALIGN;
  if ((u64)(n - 1) > (~0ull - blk_bytes) / host_stride) return AIBX_ERR_INVALID_ARG;
  const u64 extent = (u64)(n - 1) * host_stride + blk_bytes;  // bytes of the host buffer the call may touch

  // The kernel dereferences the host buffer, so it has to be pinned memory the GPU can address,
  // and long enough: anything else is refused here rather than left to fault on the GPU.
  void* dev_view = nullptr;
  if (hipHostGetDevicePointer(&dev_view, h_buf, 0) != hipSuccess || !dev_view) {
    (void)hipGetLastError();
    return AIBX_ERR_INVALID_ARG;  // not pinned host memory
  }
  hipDeviceptr_t range_base = nullptr;
  size_t range_bytes = 0;
  if (hipMemGetAddressRange(&range_base, &range_bytes, dev_view) != hipSuccess) {
    (void)hipGetLastError();
    return AIBX_ERR_INVALID_ARG;
  }
  const u64 lead = (u64)(static_cast<unsigned char*>(dev_view) - static_cast<unsigned char*>(range_base));
  if (lead > range_bytes || extent > range_bytes - lead) return AIBX_ERR_INVALID_ARG;  // buffer too short

  const u64 tile_bytes = (u64)kHostThreads * 16;
  const u64 cps = (pool->seg_bytes + tile_bytes - 1) / tile_bytes;
  const u64 tpb = cps * (u64)pool->n_seg;
  if (tpb > 0x7FFFFFF0ull) return AIBX_ERR_UNSUPPORTED;

  HostCopyArgs a;
  a.pool = static_cast<unsigned char*>(pool->base);
  a.host = static_cast<unsigned char*>(dev_view);
  a.bad_page = d_bad;
  a.seg_stride = pool->seg_stride;
  a.page_stride = pool->page_stride;
  a.seg_bytes = pool->seg_bytes;
  a.host_stride = host_stride;
  a.n_pages = pool->n_pages;
  a.total_tiles = (u64)n * tpb;
  a.chunks_per_seg = (u32)cps;
  a.tiles_per_block = (u32)tpb;
  const unsigned grid = a.total_tiles < kHostWorkgroups ? (unsigned)a.total_tiles : kHostWorkgroups;
  kv_host_copy_kernel<kToHost><<<dim3(grid), kHostThreads, 0, as_stream(stream)>>>(a, d_page_ids);
  return launch_status();
}

}  // namespace
}  // namespace aibx

extern "C" {

int aibx_kv_offload(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, void* h_dst,
                    uint64_t host_block_stride, uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_host_copy<true>(pool, d_page_ids, n, h_dst, host_block_stride, d_bad_page_counter, stream);
}

int aibx_kv_onload(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, const void* h_src,
                   uint64_t host_block_stride, uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_host_copy<false>(pool, d_page_ids, n, const_cast<void*>(h_src), host_block_stride,
                                       d_bad_page_counter, stream);
}

}  // extern "C"
