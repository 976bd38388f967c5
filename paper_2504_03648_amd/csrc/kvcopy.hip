// Paged-KV gather / scatter (Section 3.2.5 of the paper: moving KV blocks between the engine's
// paged memory and the cache's contiguous buffers). Pure byte streaming, HBM-bound.
//
// Shape of the kernel, chosen by measurement on MI355X (each point was worth 2-15 %):
//  - A tile is (entry i, segment s, chunk c): threads*16 contiguous bytes of one segment. One
//    workgroup moves exactly one tile and every lane exactly one 16-byte vector: many small
//    workgroups at full occupancy stream faster here than fewer workgroups that loop or that keep
//    several vectors per lane in flight.
//  - Loads carry the non-temporal hint; stores to the contiguous staging buffer are written
//    through at system scope, stores into the paged pool are written through with the
//    non-temporal hint as well (+0.7-2 % over the hint alone on every geometry; for the staging
//    stores the flavours are within 0.5 % of each other).
//  - Tile -> workgroup mapping. Workgroup ids are dealt round-robin over the 8 XCDs, so with the
//    "XCD-contiguous" map used here XCD x streams the x-th eighth of the tile sequence: each XCD
//    (own L2, own translation cache) works on one contiguous stretch of staging and sees whole
//    segments. Against the plain map (tile = workgroup id) this is worth 2-10 % depending on the
//    pool geometry, and it never lost in the sweeps.
#include "common.h"

namespace aibx {
namespace {

struct CopyArgs {
  unsigned char* pool;
  unsigned char* staging;
  u64* bad_page;             // nullable
  const int32_t* seg_fill;   // nullable: bytes of each segment that entry i moves (partly filled blocks)
  u64 seg_stride, page_stride, seg_bytes, staging_stride;
  int64_t n, n_pages;
  int64_t first_entry;       // entries [first_entry, first_entry + n_here) belong to this launch
  u32 chunks_per_seg;
  u32 tiles_per_block;       // chunks_per_seg * n_seg
  u32 total_tiles;           // XCD-contiguous map only
  u32 tiles_per_xcd;         // XCD-contiguous map only
};

typedef __attribute__((ext_vector_type(4))) u32 vec16;

// The asm statements below carry no "memory" clobber on purpose: they are volatile (kept, and kept
// in order), the data dependence orders each store after its load, and without the clobber the
// compiler may fetch the page and slot ids with scalar loads issued together, which shortens the
// dependent latency in front of every tile. The load and the wait for it are ONE statement, so
// the register it returns is complete wherever the compiler copies, spills or stores it.
__device__ __forceinline__ vec16 load_stream(const void* p) {
  vec16 v;
  asm volatile("global_load_dwordx4 %0, %1, off nt\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p));
  return v;
}
__device__ __forceinline__ void store_stream(void* p, vec16 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" ::"v"(p), "v"(v));
}
__device__ __forceinline__ void store_through(void* p, vec16 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v));
}

template <bool kGather, bool kFill>
__device__ __forceinline__ void copy_tile(const CopyArgs& a, const int32_t* __restrict__ page_ids,
                                          const int32_t* __restrict__ slot_ids, int64_t i, u32 tile_in_block,
                                          u32 threads) {
  const int64_t p = page_ids[i];
  const int64_t q = slot_ids ? (int64_t)slot_ids[i] : i;  // fetched together with the page id
  u64 limit = a.seg_bytes;  // bytes of a segment that this entry moves
  if constexpr (kFill) {    // clamped to the segment, rounded down to whole 16-byte vectors
    const int64_t f = a.seg_fill[i];
    limit = f <= 0 ? 0ull : (((u64)f < a.seg_bytes ? (u64)f : a.seg_bytes) & ~15ull);
  }
  if (p < 0) return;  // hole
  if (p >= a.n_pages) {
    if (tile_in_block == 0 && threadIdx.x == 0 && a.bad_page) atomicAdd((unsigned long long*)a.bad_page, 1ull);
    return;
  }
  const u32 s = tile_in_block / a.chunks_per_seg;
  const u32 c = tile_in_block - s * a.chunks_per_seg;
  const u64 off = ((u64)c * threads + threadIdx.x) * 16;
  if (off >= limit) return;  // ragged last chunk of a segment, or behind the tokens the block holds
  unsigned char* in_pool = a.pool + (u64)s * a.seg_stride + (u64)p * a.page_stride + off;
  unsigned char* in_stage = a.staging + (u64)q * a.staging_stride + (u64)s * a.seg_bytes + off;
  if (kGather) {
    store_through(in_stage, load_stream(in_pool));
  } else {
    store_stream(in_pool, load_stream(in_stage));
  }
}

// XCD x (= workgroup id mod 8) takes tiles [x*tiles_per_xcd, (x+1)*tiles_per_xcd)
template <bool kGather, int kThreads, bool kFill = false>
__global__ __launch_bounds__(kThreads) void kv_copy_xcd_kernel(CopyArgs a, const int32_t* __restrict__ page_ids,
                                                               const int32_t* __restrict__ slot_ids) {
  const u32 t = (blockIdx.x & 7u) * a.tiles_per_xcd + (blockIdx.x >> 3);
  if (t >= a.total_tiles) return;
  const u32 i = t / a.tiles_per_block;
  copy_tile<kGather, kFill>(a, page_ids, slot_ids, a.first_entry + i, t - i * a.tiles_per_block, kThreads);
}

constexpr u32 kCopyThreads = 256;  // 4 KiB tiles

// Tiles per entry and entries per launch of a pool geometry (false: one block exceeds a launch).
struct CopyShape {
  u64 chunks_per_seg, tiles_per_block;
  int64_t max_entries;
};
bool copy_shape(const aibx_pool_desc* pool, CopyShape& s) {
  const u64 tile_bytes = (u64)kCopyThreads * 16;
  s.chunks_per_seg = (pool->seg_bytes + tile_bytes - 1) / tile_bytes;
  s.tiles_per_block = s.chunks_per_seg * (u64)pool->n_seg;
  s.max_entries = max_entries_per_launch(s.tiles_per_block, kCopyThreads);
  return s.max_entries >= 1;
}
// workgroups of a launch that moves n_here entries: its tiles rounded up to whole rounds of 8
u32 copy_grid(const CopyShape& s, int64_t n_here) { return (u32)((((u64)n_here * s.tiles_per_block + 7) / 8) * 8); }

template <bool kGather>
int launch_copy(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                const int32_t* d_seg_fill, int64_t n, void* d_staging, u64 stride, u64* d_bad, void* stream) {
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
  if (!aligned(d_page_ids, 4) || !aligned(d_slot_ids, 4) || !aligned(d_seg_fill, 4) || !aligned(d_bad, 8))
    return AIBX_ERR_ALIGN;

  CopyShape shape;
  if (!copy_shape(pool, shape)) return AIBX_ERR_UNSUPPORTED;

  CopyArgs a;
  a.pool = static_cast<unsigned char*>(pool->base);
  a.staging = static_cast<unsigned char*>(d_staging);
  a.bad_page = d_bad;
  a.seg_fill = d_seg_fill;
  a.seg_stride = pool->seg_stride;
  a.page_stride = pool->page_stride;
  a.seg_bytes = pool->seg_bytes;
  a.staging_stride = stride;
  a.n = n;
  a.n_pages = pool->n_pages;
  a.first_entry = 0;
  a.chunks_per_seg = (u32)shape.chunks_per_seg;
  a.tiles_per_block = (u32)shape.tiles_per_block;
  a.total_tiles = a.tiles_per_xcd = 0;
  hipStream_t st = as_stream(stream);
  // as many launches as the grid limit asks for (one, below 64 GiB per call)
  for (int64_t first = 0; first < n; first += shape.max_entries) {
    const int64_t n_here = (n - first) < shape.max_entries ? (n - first) : shape.max_entries;
    const u32 grid = copy_grid(shape, n_here);
    a.first_entry = first;
    a.total_tiles = (u32)((u64)n_here * shape.tiles_per_block);
    a.tiles_per_xcd = grid / 8;
    if (d_seg_fill)
      kv_copy_xcd_kernel<kGather, kCopyThreads, true><<<dim3(grid), kCopyThreads, 0, st>>>(a, d_page_ids, d_slot_ids);
    else
      kv_copy_xcd_kernel<kGather, kCopyThreads><<<dim3(grid), kCopyThreads, 0, st>>>(a, d_page_ids, d_slot_ids);
    const int rc = launch_status();
    if (rc != AIBX_OK) return rc;
  }
  return AIBX_OK;
}

}  // namespace
}  // namespace aibx

extern "C" {

int aibx_kv_copy_launches(const aibx_pool_desc* pool, int64_t n, int64_t* first_entry_out,
                          int64_t* n_entries_out, uint32_t* workgroups_out, int32_t capacity) {
  using namespace aibx;
  if (!pool || n < 0 || capacity < 0 || pool->n_seg < 1 || pool->seg_bytes == 0) return AIBX_ERR_INVALID_ARG;
  if (capacity && (!first_entry_out || !n_entries_out || !workgroups_out)) return AIBX_ERR_INVALID_ARG;
  CopyShape shape;
  if (!copy_shape(pool, shape)) return AIBX_ERR_UNSUPPORTED;
  int k = 0;
  for (int64_t first = 0; first < n; first += shape.max_entries, ++k) {
    if (k >= capacity) continue;
    const int64_t n_here = (n - first) < shape.max_entries ? (n - first) : shape.max_entries;
    first_entry_out[k] = first;
    n_entries_out[k] = n_here;
    workgroups_out[k] = copy_grid(shape, n_here);
  }
  return k;
}

int aibx_kv_gather(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                   int64_t n, void* d_staging, uint64_t staging_block_stride,
                   uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_copy<true>(pool, d_page_ids, d_slot_ids, nullptr, n, d_staging, staging_block_stride,
                                 d_bad_page_counter, stream);
}

int aibx_kv_scatter(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                    int64_t n, const void* d_staging, uint64_t staging_block_stride,
                    uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_copy<false>(pool, d_page_ids, d_slot_ids, nullptr, n, const_cast<void*>(d_staging),
                                  staging_block_stride, d_bad_page_counter, stream);
}

int aibx_kv_gather_fill(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                        const int32_t* d_seg_fill, int64_t n, void* d_staging, uint64_t staging_block_stride,
                        uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_copy<true>(pool, d_page_ids, d_slot_ids, d_seg_fill, n, d_staging, staging_block_stride,
                                 d_bad_page_counter, stream);
}

int aibx_kv_scatter_fill(const aibx_pool_desc* pool, const int32_t* d_page_ids, const int32_t* d_slot_ids,
                         const int32_t* d_seg_fill, int64_t n, const void* d_staging,
                         uint64_t staging_block_stride, uint64_t* d_bad_page_counter, void* stream) {
  return aibx::launch_copy<false>(pool, d_page_ids, d_slot_ids, d_seg_fill, n, const_cast<void*>(d_staging),
                                  staging_block_stride, d_bad_page_counter, stream);
}

}  // extern "C"
