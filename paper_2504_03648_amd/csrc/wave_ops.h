// Cross-lane helpers shared by the kernels: scalar reads of a lane, DPP lane patterns, and the
// inclusive AND scan over a wavefront that the routing forms use.
#pragma once

#include "common.h"

namespace aibx {
namespace {  // internal linkage: each translation unit gets its own copy

// The value lane `lane` holds, in every lane (`lane` must be the same in all of them): a scalar.
__device__ __forceinline__ u64 readlane64(u64 v, int lane) {
  const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)v, lane);
  const u32 hi = (u32)__builtin_amdgcn_readlane((int)(u32)(v >> 32), lane);
  return ((u64)hi << 32) | lo;
}

// 64-bit value through a DPP lane pattern (a VALU operand modifier: no LDS round trip). Lanes
// whose source is outside the row read 0.
template <int kCtrl>
__device__ __forceinline__ u64 dpp64(u64 v) {
  const u32 lo = (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)v, kCtrl, 0xF, 0xF, true);
  const u32 hi = (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)(v >> 32), kCtrl, 0xF, 0xF, true);
  return ((u64)hi << 32) | lo;
}
constexpr int kDppRowMirror = 0x140, kDppRowHalfMirror = 0x141, kDppQuadReverse = 0x1B, kDppQuadSwap = 0xB1;
constexpr int kDppRowShr = 0x110;  // + shift (1..15)

// Like dpp64, but lanes whose source is outside the row keep their own value.
template <int kCtrl>
__device__ __forceinline__ u64 dpp64_or_self(u64 v) {
  const u32 lo = (u32)__builtin_amdgcn_update_dpp((int)(u32)v, (int)(u32)v, kCtrl, 0xF, 0xF, false);
  const u32 hi = (u32)__builtin_amdgcn_update_dpp((int)(u32)(v >> 32), (int)(u32)(v >> 32), kCtrl, 0xF, 0xF, false);
  return ((u64)hi << 32) | lo;
}

// Minimum over the 64 lanes, the same scalar in every lane: a running minimum along each row of 16
// lanes (four DPP row shifts), then the rows' last lanes.
__device__ __forceinline__ u64 wave_min64(u64 v) {
  u64 o;
  o = dpp64_or_self<kDppRowShr + 1>(v); v = o < v ? o : v;
  o = dpp64_or_self<kDppRowShr + 2>(v); v = o < v ? o : v;
  o = dpp64_or_self<kDppRowShr + 4>(v); v = o < v ? o : v;
  o = dpp64_or_self<kDppRowShr + 8>(v); v = o < v ? o : v;
  const u64 a = readlane64(v, 15), b = readlane64(v, 31), c = readlane64(v, 47), d = readlane64(v, 63);
  const u64 ab = a < b ? a : b, cd = c < d ? c : d;
  return ab < cd ? ab : cd;
}

// Inclusive AND scan over the 64 lanes: lane l gets v_0 & v_1 & ... & v_l. Inside a row of 16 lanes
// four DPP row shifts on the complement (a shift feeds zeros into the row's first lanes, and zero is
// the identity of OR); across rows three scalar reads of the rows' last lanes. No LDS traffic, where
// six rounds of shuffles cost twelve trips through the LDS crossbar.
__device__ __forceinline__ u64 and_scan64(u64 v, int lane) {
  u64 c = ~v;
  c |= dpp64<kDppRowShr + 1>(c);
  c |= dpp64<kDppRowShr + 2>(c);
  c |= dpp64<kDppRowShr + 4>(c);
  c |= dpp64<kDppRowShr + 8>(c);
  const u64 t0 = readlane64(c, 15), t1 = readlane64(c, 31), t2 = readlane64(c, 47);
  const int row = lane >> 4;
  u64 before = 0;  // what the rows below this lane's row are missing
  before = row >= 1 ? t0 : before;
  before = row >= 2 ? (t0 | t1) : before;
  before = row >= 3 ? (t0 | t1 | t2) : before;
  return ~(c | before);
}

}  // namespace
}  // namespace aibx
