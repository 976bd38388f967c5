// Device-side view of the cache index shared by the index kernels and the fused hash+match kernel:
// handle, table descriptor, probe sequence and the one-lane lookup. Layout and invariants are
// described at the top of index.hip.
#pragma once

#include "common.h"

struct aibx_index {
  aibx::u64* slots;       // device, 2*n_slots words: {key, value} pairs
  aibx::u32* usage;       // device, n_slots words behind the slots: (touch count << 24) | last epoch
  aibx::u64 n_slots;
  aibx::u64 n_buckets;    // n_slots / 8, power of two
  int lg_buckets;
};

namespace aibx {
namespace {  // internal linkage: each translation unit gets its own copy

constexpr u64 kEmpty = AIBX_KEY_EMPTY;
constexpr u64 kTomb = AIBX_KEY_TOMBSTONE;
constexpr u64 kNoValue = AIBX_NO_VALUE;
constexpr int kBucket = 8;                       // slots per bucket (8 x 16 B = one 128-byte line)
constexpr u64 kHomeMul = 0x9E3779B97F4A7C15ull;  // multiplicative (Fibonacci) bucket hash
constexpr int kIndexThreads = 256;
constexpr int kWavesPerGroup = kIndexThreads / kWave;

constexpr int kSlotBytes = 16, kUsageBytes = 4;  // storage per slot: the slot, then its usage word
constexpr u32 kEpochMask = 0xFFFFFFu;             // usage word: [31:24] touch count, [23:0] last epoch

struct Table {
  u64* slots;
  u32* usage;
  u64 bucket_mask;
  int shift;  // 64 - lg(n_buckets); home = (key * kHomeMul) >> shift (0 buckets bits -> 0)
};

__device__ __forceinline__ u64 home_bucket(const Table& t, u64 key) {
  return t.shift >= 64 ? 0ull : (key * kHomeMul) >> t.shift;
}

// Double hashing over buckets: the k-th bucket of a key's probe sequence is home + k*step with an
// odd step taken from other bits of the key's product, so full buckets do not cluster the way they
// do under linear probing (which buys nothing here: a neighbouring line costs as much as any other).
// An odd step modulo a power of two visits every bucket once.
__device__ __forceinline__ u64 probe_step(u64 key) { return ((key * kHomeMul) >> 7) | 1ull; }

typedef __attribute__((ext_vector_type(2))) u64 slot_t;  // .x = key, .y = value

// ---- lookup ------------------------------------------------------------------------------------
// One lane per key: the lane reads its key's whole bucket (8 x 16 bytes, one 128-byte line) and
// compares the 8 keys itself. Random line reads on this GPU are bound by the number of lines
// requested (about 55-80 G lines/s whether a line is fetched by one lane or by eight), so this
// costs the memory system no more than a cooperative read and needs no cross-lane work at all.
// Read-only: plain cached loads. Returns the key's value or kNoValue.
__device__ __forceinline__ u64 lookup_one(const Table& t, u64 key, bool valid) {
  u64 result = kNoValue;
  bool open = valid && key != kEmpty && key != kTomb;
  u64 b = home_bucket(t, key);
  const u64 step = probe_step(key);
  for (u64 seen_buckets = 0; open; ++seen_buckets) {
    const slot_t* bucket = reinterpret_cast<const slot_t*>(t.slots + 2 * b * kBucket);
    slot_t s[kBucket];
#pragma unroll
    for (int j = 0; j < kBucket; ++j) s[j] = bucket[j];
    bool ends = seen_buckets >= t.bucket_mask;  // that was the last bucket of the table
#pragma unroll
    for (int j = 0; j < kBucket; ++j) {
      if (s[j].x == key) {
        result = s[j].y;
        ends = true;
      }
      ends |= s[j].x == kEmpty;  // a bucket with an EMPTY slot ends the probe sequence
    }
    open = !ends;
    b = (b + step) & t.bucket_mask;
  }
  return result;
}

inline Table table_of(const aibx_index* ix) {
  Table t;
  t.slots = ix->slots;
  t.usage = ix->usage;
  t.bucket_mask = ix->n_buckets - 1;
  t.shift = 64 - ix->lg_buckets;
  return t;
}

}  // namespace
}  // namespace aibx
