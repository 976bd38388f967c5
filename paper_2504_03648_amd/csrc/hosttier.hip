// Host-tier leg of offload / onload (Section 3.2.5 of the paper: the cache pool lives in DRAM and
// exchanges KV with the colocated engine through host memory). The paged pool is gathered into a
// two-part staging buffer in HBM chunk by chunk, and each chunk travels to pinned host memory on a
// second stream while the next chunk is being gathered (and the reverse for onload), so the PCIe
// transfer - the slow leg by two orders of magnitude - never waits for the copy kernels.
// Host code only: the device work is aibx_kv_gather / aibx_kv_scatter and the runtime's copies.
#include <vector>

#include "common.h"

namespace aibx {
namespace {

struct Events {
  std::vector<hipEvent_t> ev;
  ~Events() {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);  // pending work keeps its own reference
  }
  int make(hipEvent_t* out) {
    hipError_t e = hipEventCreateWithFlags(out, hipEventDisableTiming);
    if (e != hipSuccess) return hip_failed(e);
    ev.push_back(*out);
    return AIBX_OK;
  }
};

#define AIBX_HIP(call)                            \
  do {                                            \
    hipError_t e_ = (call);                       \
    if (e_ != hipSuccess) return hip_failed(e_);  \
  } while (0)

// One chunk between staging and host: a linear copy when both sides are densely packed, a pitched
// copy otherwise.
hipError_t copy_chunk(void* dst, u64 dst_stride, const void* src, u64 src_stride, u64 blk_bytes, int64_t m,
                      hipMemcpyKind kind, hipStream_t st) {
  if (dst_stride == blk_bytes && src_stride == blk_bytes) return hipMemcpyAsync(dst, src, blk_bytes * (u64)m, kind, st);
  return hipMemcpy2DAsync(dst, dst_stride, src, src_stride, blk_bytes, (size_t)m, kind, st);
}

int check_tier_args(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, void* d_staging,
                    int64_t chunk_blocks, u64 staging_stride, void* h_buf, u64 host_stride, void* s_copy,
                    void* s_xfer) {
  if (n < 0 || chunk_blocks < 1) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!pool || !d_page_ids || !d_staging || !h_buf) return AIBX_ERR_INVALID_ARG;
  if (pool->n_seg < 1 || pool->seg_bytes == 0) return AIBX_ERR_INVALID_ARG;
  const u64 blk_bytes = (u64)pool->n_seg * pool->seg_bytes;
  if (staging_stride < blk_bytes || host_stride < blk_bytes) return AIBX_ERR_INVALID_ARG;
  if (s_copy == s_xfer) return AIBX_ERR_INVALID_ARG;  // the overlap needs two streams
  if (!aligned(h_buf, 16) || host_stride % 16) return AIBX_ERR_ALIGN;
  return 1;  // proceed
}

}  // namespace
}  // namespace aibx

using namespace aibx;

extern "C" {

int aibx_kv_offload(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, void* d_staging,
                    int64_t chunk_blocks, uint64_t staging_block_stride, void* h_dst,
                    uint64_t host_block_stride, uint64_t* d_bad_page_counter, void* stream_copy,
                    void* stream_xfer) {
  const int pre = check_tier_args(pool, d_page_ids, n, d_staging, chunk_blocks, staging_block_stride, h_dst,
                                  host_block_stride, stream_copy, stream_xfer);
  if (pre != 1) return pre;
  const u64 blk_bytes = (u64)pool->n_seg * pool->seg_bytes;
  hipStream_t sc = as_stream(stream_copy), sx = as_stream(stream_xfer);
  Events events;
  hipEvent_t sent[2] = {nullptr, nullptr};  // transfer that last read staging half 0 / 1
  int64_t k = 0;
  for (int64_t first = 0; first < n; first += chunk_blocks, ++k) {
    const int64_t m = (n - first) < chunk_blocks ? (n - first) : chunk_blocks;
    const int half = (int)(k & 1);
    unsigned char* stage = static_cast<unsigned char*>(d_staging) + (u64)half * (u64)chunk_blocks * staging_block_stride;
    if (sent[half]) AIBX_HIP(hipStreamWaitEvent(sc, sent[half], 0));  // the half is free again
    const int rc = aibx_kv_gather(pool, d_page_ids + first, nullptr, m, stage, staging_block_stride,
                                  d_bad_page_counter, sc);
    if (rc != AIBX_OK) return rc;
    hipEvent_t gathered;
    int erc = events.make(&gathered);
    if (erc != AIBX_OK) return erc;
    AIBX_HIP(hipEventRecord(gathered, sc));
    AIBX_HIP(hipStreamWaitEvent(sx, gathered, 0));
    AIBX_HIP(copy_chunk(static_cast<unsigned char*>(h_dst) + (u64)first * host_block_stride, host_block_stride,
                        stage, staging_block_stride, blk_bytes, m, hipMemcpyDeviceToHost, sx));
    erc = events.make(&sent[half]);
    if (erc != AIBX_OK) return erc;
    AIBX_HIP(hipEventRecord(sent[half], sx));
  }
  for (int h = 0; h < 2; ++h)  // waiting on the copy stream now covers the transfers too
    if (sent[h]) AIBX_HIP(hipStreamWaitEvent(sc, sent[h], 0));
  return AIBX_OK;
}

int aibx_kv_onload(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, void* d_staging,
                   int64_t chunk_blocks, uint64_t staging_block_stride, const void* h_src,
                   uint64_t host_block_stride, uint64_t* d_bad_page_counter, void* stream_copy,
                   void* stream_xfer) {
  const int pre = check_tier_args(pool, d_page_ids, n, d_staging, chunk_blocks, staging_block_stride,
                                  const_cast<void*>(h_src), host_block_stride, stream_copy, stream_xfer);
  if (pre != 1) return pre;
  const u64 blk_bytes = (u64)pool->n_seg * pool->seg_bytes;
  hipStream_t sc = as_stream(stream_copy), sx = as_stream(stream_xfer);
  Events events;
  hipEvent_t scattered[2] = {nullptr, nullptr};  // scatter that last read staging half 0 / 1
  hipEvent_t start;
  int erc = events.make(&start);
  if (erc != AIBX_OK) return erc;
  AIBX_HIP(hipEventRecord(start, sc));  // the transfers start after what is already queued on the copy stream
  AIBX_HIP(hipStreamWaitEvent(sx, start, 0));
  int64_t k = 0;
  for (int64_t first = 0; first < n; first += chunk_blocks, ++k) {
    const int64_t m = (n - first) < chunk_blocks ? (n - first) : chunk_blocks;
    const int half = (int)(k & 1);
    unsigned char* stage = static_cast<unsigned char*>(d_staging) + (u64)half * (u64)chunk_blocks * staging_block_stride;
    if (scattered[half]) AIBX_HIP(hipStreamWaitEvent(sx, scattered[half], 0));
    AIBX_HIP(copy_chunk(stage, staging_block_stride,
                        static_cast<const unsigned char*>(h_src) + (u64)first * host_block_stride, host_block_stride,
                        blk_bytes, m, hipMemcpyHostToDevice, sx));
    hipEvent_t loaded;
    erc = events.make(&loaded);
    if (erc != AIBX_OK) return erc;
    AIBX_HIP(hipEventRecord(loaded, sx));
    AIBX_HIP(hipStreamWaitEvent(sc, loaded, 0));
    const int rc = aibx_kv_scatter(pool, d_page_ids + first, nullptr, m, stage, staging_block_stride,
                                   d_bad_page_counter, sc);
    if (rc != AIBX_OK) return rc;
    erc = events.make(&scattered[half]);
    if (erc != AIBX_OK) return erc;
    AIBX_HIP(hipEventRecord(scattered[half], sc));
  }
  return AIBX_OK;
}

}  // extern "C"
