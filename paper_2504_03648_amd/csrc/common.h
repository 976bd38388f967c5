// Shared host-side helpers of the aibx library (status codes, HIP error capture, argument checks).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "aibx.h"

namespace aibx {

typedef uint64_t u64;
typedef uint32_t u32;

constexpr int kWave = 64;  // CDNA wavefront width

// Records the text of a failed HIP call for aibx_last_hip_error() and returns AIBX_ERR_HIP.
int hip_failed(hipError_t e);

// After a kernel launch: AIBX_OK, or AIBX_ERR_HIP with the error text recorded.
inline int launch_status() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? AIBX_OK : hip_failed(e);
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

// How the copy kernels split a call into launches. One workgroup moves one tile, and a launch
// whose grid times its workgroup size reaches 2^32 threads is refused by the runtime, so a launch
// takes at most floor((2^32 - 1) / threads) workgroups - rounded down to whole rounds of the 8
// XCDs, because the tile map deals the workgroups of a launch to the XCDs in eighths. Entries are
// never split between launches. Returns 0 when a single entry does not fit one launch.
inline int64_t max_entries_per_launch(u64 tiles_per_entry, u32 threads) {
  const u64 max_groups = (0xFFFFFFFFull / threads) & ~7ull;
  return tiles_per_entry == 0 ? 0 : (int64_t)(max_groups / tiles_per_entry);
}

}  // namespace aibx
