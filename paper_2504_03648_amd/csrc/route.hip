// Prefix-cache-aware routing decision (Section 3.2.2 of the paper: route to an instance that
// already holds a reusable prefix of the request's KV cache when the hit is large enough; the
// fallback here is the least-request policy of the same list). Semantics are stated in aibx.h.
//
// One wavefront per request. A block's index value is the set of pods holding it (bit p = pod p).
// The set of pods that hold ALL of blocks 0..j is the running AND of those sets; it only shrinks,
// so the longest prefix any pod holds ends where the running AND becomes empty, and the pods that
// hold that longest prefix are the last non-empty running AND. No per-pod loop is needed: the
// wavefront scans 64 blocks per trip with a cross-lane AND scan (DPP row shifts and three scalar
// reads, no LDS) and stops at the first empty set.
#include "common.h"
#include "wave_ops.h"

namespace aibx {
namespace {

constexpr u64 kNoValue = AIBX_NO_VALUE;


__global__ __launch_bounds__(kWave) void route_kernel(const u64* __restrict__ pod_sets,
                                                      const int64_t* __restrict__ blk_off, int n_pods,
                                                      const int32_t* __restrict__ pod_load, u64 thr_num,
                                                      u64 thr_den, int32_t* __restrict__ pod_out,
                                                      int32_t* __restrict__ hit_len_out) {
  const int r = blockIdx.x;
  const int lane = threadIdx.x;
  const int64_t b0 = blk_off[r];
  const int64_t n_r = blk_off[r + 1] - b0;
  const u64 all_pods = (1ull << n_pods) - 1ull;  // n_pods <= 63

  // least-request pod over all pods (the fallback), ties to the lower id: min of (load, id)
  const u64 my_rank = lane < n_pods ? ((u64)(u32)pod_load[lane] << 8) | (u64)lane : ~0ull;
  const int fallback_pod = (int)(wave_min64(my_rank) & 0xFF);

  u64 alive = all_pods;      // pods holding every block seen so far
  int64_t best_len = 0;      // longest prefix held by any pod
  u64 best_set = 0;          // the pods holding it
  int64_t fallback_len = 0;  // prefix held by the fallback pod
  // the next tile's sets are requested while this tile is scanned
  u64 v_next = lane < n_r ? pod_sets[b0 + lane] : all_pods;
  for (int64_t base = 0; base < n_r && alive != 0; base += kWave) {
    const bool valid = base + lane < n_r;
    u64 v = v_next;
    v_next = base + kWave + lane < n_r ? pod_sets[b0 + base + kWave + lane] : all_pods;
    v = v == kNoValue ? 0ull : (v & all_pods);
    if (!valid) v = all_pods;  // lanes past the end do not shrink the set
    // inclusive AND scan across lanes, then the sets carried in from earlier tiles
    v = and_scan64(v, lane);
    v &= alive;
    const u64 nonempty = __ballot(valid && v != 0);            // a run of ones from lane 0
    const u64 has_fb = __ballot(valid && ((v >> fallback_pod) & 1ull));
    const int cnt = __popcll(nonempty);
    if (cnt > 0) {
      best_len = base + cnt;
      best_set = readlane64(v, cnt - 1);
    }
    fallback_len += __popcll(has_fb);
    alive = readlane64(v, kWave - 1);  // lanes past the end carried the last real set forward
  }
  // prefix-aware choice only if the hit ratio reaches the threshold: best_len/n_r >= num/den
  const bool aware = n_r > 0 && best_len > 0 && (u64)best_len * thr_den >= thr_num * (u64)n_r;
  u64 rank = my_rank;
  if (aware && !((best_set >> lane) & 1ull)) rank = ~0ull;  // candidates: the pods of best_set
  rank = wave_min64(rank);
  if (lane == 0) {
    pod_out[r] = (int32_t)(rank & 0xFF);
    hit_len_out[r] = (int32_t)(aware ? best_len : fallback_len);
  }
}

}  // namespace
}  // namespace aibx

extern "C" int aibx_route(const uint64_t* d_pod_sets, const int64_t* d_blk_off, int32_t n_req,
                          int64_t n_blocks_total, int32_t n_pods, const int32_t* d_pod_load,
                          uint64_t threshold_num, uint64_t threshold_den, int32_t* d_pod_out,
                          int32_t* d_hit_len_out, void* stream) {
  using namespace aibx;
  if (n_req < 0 || n_blocks_total < 0 || n_pods < 1 || n_pods > 63 || threshold_den == 0) return AIBX_ERR_INVALID_ARG;
  if (threshold_num > 0xFFFFFFFFull || threshold_den > 0xFFFFFFFFull) return AIBX_ERR_INVALID_ARG;
  if (n_req == 0) return AIBX_OK;
  if (!d_blk_off || !d_pod_load || !d_pod_out || !d_hit_len_out || (n_blocks_total > 0 && !d_pod_sets))
    return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_pod_sets, 8) || !aligned(d_blk_off, 8) || !aligned(d_pod_load, 4) || !aligned(d_pod_out, 4) ||
      !aligned(d_hit_len_out, 4))
    return AIBX_ERR_ALIGN;
  route_kernel<<<(u32)n_req, kWave, 0, as_stream(stream)>>>(d_pod_sets, d_blk_off, n_pods, d_pod_load, threshold_num,
                                                            threshold_den, d_pod_out, d_hit_len_out);
  return launch_status();
}
