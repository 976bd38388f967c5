// Measurement aid, not part of the hot path: independent random reads over a table, one read per
// lane and step - the access pattern of the index lookups with everything else taken away. The
// benchmark reports the lookup rates beside what this kernel reaches on a table of the same size.
#include "common.h"

namespace aibx {
namespace {

constexpr int kCalibThreads = 256;

__device__ __forceinline__ u64 scramble(u64 x) {
  x *= 0x9E3779B97F4A7C15ull;
  x ^= x >> 29;
  x *= 0xBB67AE8584CAA73Bull;
  x ^= x >> 32;
  return x;
}

// kWords 64-bit words are read from the start of a random line of line_words words.
template <int kWords>
__global__ __launch_bounds__(kCalibThreads) void random_read_kernel(const u64* __restrict__ table, u64 line_mask,
                                                                   u32 lg_line_words, int64_t n_reads, u64 seed,
                                                                   u64* __restrict__ sink) {
  u64 acc = 0;
  for (int64_t i = (int64_t)blockIdx.x * kCalibThreads + threadIdx.x; i < n_reads;
       i += (int64_t)gridDim.x * kCalibThreads) {
    const u64 line = scramble(seed + (u64)i) & line_mask;
    const u64* p = table + (line << lg_line_words);
#pragma unroll
    for (int w = 0; w < kWords; ++w) acc ^= p[w];
  }
  if (acc == 0x0123456789ABCDEFull) sink[0] = acc;  // keeps the loads alive; practically never taken
}

}  // namespace
}  // namespace aibx

extern "C" int aibx_calib_random_reads(const void* d_table, uint64_t table_bytes, uint32_t line_bytes,
                                       uint32_t read_bytes, int64_t n_reads, uint64_t seed, uint64_t* d_sink,
                                       void* stream) {
  using namespace aibx;
  if (!d_table || !d_sink || n_reads < 0) return AIBX_ERR_INVALID_ARG;
  if (line_bytes < 8 || (line_bytes & (line_bytes - 1)) || line_bytes > 4096) return AIBX_ERR_INVALID_ARG;
  if (table_bytes < line_bytes || (table_bytes & (table_bytes - 1))) return AIBX_ERR_INVALID_ARG;
  if (read_bytes > line_bytes || (read_bytes != 8 && read_bytes != 16 && read_bytes != 64 && read_bytes != 128))
    return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_table, 128) || !aligned(d_sink, 8)) return AIBX_ERR_ALIGN;
  if (n_reads == 0) return AIBX_OK;
  int lg = 0;
  while ((8u << lg) < line_bytes) ++lg;
  const u64 line_mask = table_bytes / line_bytes - 1;
  const u64 want = ((u64)n_reads + kCalibThreads - 1) / kCalibThreads;
  const u32 grid = (u32)(want > 8192 ? 8192 : want);
  const u64* t = static_cast<const u64*>(d_table);
  hipStream_t st = as_stream(stream);
  switch (read_bytes) {
    case 8: random_read_kernel<1><<<grid, kCalibThreads, 0, st>>>(t, line_mask, lg, n_reads, seed, d_sink); break;
    case 16: random_read_kernel<2><<<grid, kCalibThreads, 0, st>>>(t, line_mask, lg, n_reads, seed, d_sink); break;
    case 64: random_read_kernel<8><<<grid, kCalibThreads, 0, st>>>(t, line_mask, lg, n_reads, seed, d_sink); break;
    default: random_read_kernel<16><<<grid, kCalibThreads, 0, st>>>(t, line_mask, lg, n_reads, seed, d_sink); break;
  }
  return launch_status();
}
