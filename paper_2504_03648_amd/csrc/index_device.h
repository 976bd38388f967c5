// Device-side view of the cache index shared by the index kernels and the fused hash+match kernel:
// handle, table descriptor, probe sequence and the one-lane lookup. Layout and invariants are
// described at the top of index.hip.
#pragma once

#include "common.h"
#include "wave_ops.h"

struct aibx_index {
  aibx::u64* slots;       // device, 2*n_slots words: buckets of 8 keys followed by their 8 values
  aibx::u32* usage;       // device, n_slots words behind the slots: (touch count << 24) | last epoch
  unsigned char* tags;    // device, n_slots bytes behind the usage words: one tag per slot
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

constexpr int kSlotBytes = 16, kUsageBytes = 4, kTagBytes = 1;  // storage per slot: slot, usage word, tag
constexpr int kStorageBytesPerSlot = kSlotBytes + kUsageBytes + kTagBytes;
constexpr u32 kEpochMask = 0xFFFFFFu;             // usage word: [31:24] touch count, [23:0] last epoch

// A key is stored within the first kMaxProbeBuckets buckets of its probe sequence or not at all, and
// no lookup goes further. Below a load factor of 0.99 this never binds (a sequence of 4,096 full
// buckets has a probability under 1e-18 even when 99 % of the buckets are full); it bounds what a
// table with no EMPTY slot left - full, or worn down to tombstones - can cost a batch: without it
// every absent key walks the whole table.
constexpr u64 kMaxProbeBuckets = 4096;

struct Table {
  u64* slots;
  u32* usage;
  unsigned char* tags;
  u64 bucket_mask;
  u64 probe_limit;  // min(n_buckets, kMaxProbeBuckets): buckets of a probe sequence that are ever used
  int shift;  // 64 - lg(n_buckets); home = (key * kHomeMul) >> shift (0 buckets bits -> 0)
  bool guess_present;  // lookups of a tile may go through the key words (lookup_tile)
};
// Tables from this many slots on let lookup_tile guess: their tags (4 MiB and more) no longer stay in
// an XCD's L2, so a key that is present costs a line of tags besides its slot's line, and every line
// that leaves the L2 is 128 bytes at the rate of a streaming read. Measured with every key present:
// lookup time -24 % (2^22 slots at load 0.7 and 2^24 at 0.75), -13 % in the kernel that also hashes;
// with every key absent no difference beyond the run-to-run spread (the question is asked on the
// scalar side: two readlanes, scalar multiplies, one 8-byte read). In smaller tables the tags are
// cached, and going through the key words costs present keys 10 % (2^20 slots) to 40 % (2^12).
constexpr u64 kGuessPresentFrom = 1ull << 22;

__device__ __forceinline__ u64 home_bucket(const Table& t, u64 key) {
  return t.shift >= 64 ? 0ull : (key * kHomeMul) >> t.shift;
}

// Probe sequence: buckets are visited in pairs of neighbours (b, b ^ 1), and the pairs by double
// hashing: bucket 2k of a key's sequence is home + 2*k*step, bucket 2k+1 its neighbour, with an odd
// step taken from other bits of the key's product. An odd step over the pairs visits every pair
// once, so the sequence visits every bucket once; full buckets do not cluster the way they do under
// linear probing; and the tags of a pair are 16 aligned bytes, which a lookup fetches with ONE
// request where two separate buckets cost two (lookups here are bound by the number of requests:
// at a load factor of 0.75 an absent key costs 1.22 requests this way instead of 1.47).
__device__ __forceinline__ u64 probe_step(u64 key) { return ((key * kHomeMul) >> 7) | 1ull; }
// The bucket after b, where `probes` buckets of the sequence came before b (b is the first of its
// pair when that count is even). In a table of one bucket the result is never used (its sequences have
// length 1).
__device__ __forceinline__ u64 next_bucket(const Table& t, u64 b, u64 step, u64 probes) {
  b ^= 1ull;
  return (probes & 1ull) ? (b + 2ull * step) & t.bucket_mask : b;
}

// Bucket layout: 16 words; words 0..7 are the 8 keys, words 8..15 the 8 values (slot j of bucket b:
// key word 16b+j, value word 16b+8+j). A probe reads the 64 bytes of keys only and fetches one
// value on a hit: measured against {key,value} pairs side by side this is +20 % probes/s on a
// 16 MiB table at load 0.5, +40 % at load 0.75, and no slower when every probe hits.
constexpr int kBucketWords = 2 * kBucket;
typedef __attribute__((ext_vector_type(2))) u64 key_pair_t;  // two neighbouring keys of a bucket
typedef __attribute__((ext_vector_type(2))) u64 tag_pair_t;  // the tag words of a pair of buckets

__device__ __forceinline__ u64* bucket_words(const Table& t, u64 b) { return t.slots + kBucketWords * b; }
// word index of slot i's key (i = 8*bucket + j); its value is kBucket words further
__device__ __forceinline__ u64 key_word_of_slot(u64 i) { return (i / kBucket) * kBucketWords + (i % kBucket); }

// The 8 keys of a bucket with ordinary cached loads (4 x 16 bytes).
__device__ __forceinline__ void load_bucket_keys(const u64* bucket, u64 (&keys)[kBucket]) {
  const key_pair_t* p = reinterpret_cast<const key_pair_t*>(bucket);
#pragma unroll
  for (int j = 0; j < kBucket / 2; ++j) {
    const key_pair_t kp = p[j];
    keys[2 * j] = kp.x;
    keys[2 * j + 1] = kp.y;
  }
}

// ---- tags --------------------------------------------------------------------------------------
// One byte per slot, the 8 tags of a bucket in one 64-bit word: 0 = the slot is EMPTY, 0xFF = it
// is a TOMBSTONE, anything else = bits 24..31 of the key's product. The home bucket is the
// product's top lg(n_buckets) bits, so up to 2^35 slots the tag is independent of it (keys that
// meet in a bucket still differ in their tags); the probe step (bits 7 and up) does share bits
// with the tag in tables of 2^18 buckets or more, which costs nothing: keys with equal tags in
// one bucket are told apart by the key comparison, whatever their steps. The update kernels write a
// slot's tag after they have won its key word, so between launches the tags mirror the keys
// exactly. A lookup walks the tags only - an eighth of
// the bytes of the key words, so the tags of a table stay in cache where its slots do not (16 Mi
// slots: 16 MiB of tags against 256 MiB of slots) - and touches a slot only where the tag matches:
// always for a key that is present, with probability 1/254 per occupied slot for one that is not.
constexpr unsigned kTagEmpty = 0x00u, kTagTomb = 0xFFu;
constexpr u64 kOnes = 0x0101010101010101ull, kLow7 = 0x7F7F7F7F7F7F7F7Full;

__device__ __forceinline__ unsigned tag_of(u64 key) {
  const unsigned x = (unsigned)((key * kHomeMul) >> 24) & 0xFFu;
  return x == kTagEmpty ? 1u : (x == kTagTomb ? 0xFEu : x);
}
// 0x80 in every byte of x that is zero, 0 elsewhere (exact: no carry crosses a byte)
__device__ __forceinline__ u64 zero_bytes(u64 x) { return ~(((x & kLow7) + kLow7) | x | kLow7); }

__device__ __forceinline__ const u64* tag_word(const Table& t, u64 b) {
  return reinterpret_cast<const u64*>(t.tags) + b;
}

// ---- lookup ------------------------------------------------------------------------------------
// One lane per key: the lane reads the 16 tags of its key's pair of buckets (one 16-byte load) and
// compares them itself; random reads on this GPU are bound by the number of lines requested (about
// 55-80 G lines/s whether a line is fetched by one lane or by eight), so this costs the memory
// system no more than a cooperative read and needs no cross-lane work at all.
// Read-only: plain cached loads. find_slot returns the key's slot (8*bucket + j) or -1, and the
// slot's value through value_out: key and value of a candidate slot sit in one 128-byte line and
// are requested together, so a probe that hits makes two dependent accesses (tags, slot), not three.
__device__ __forceinline__ int64_t find_slot(const Table& t, u64 key, bool valid, u64& value_out) {
  int64_t found = -1;
  bool open = valid && key != kEmpty && key != kTomb;
  u64 b = home_bucket(t, key);
  const u64 step = probe_step(key);
  const u64 mine = (u64)tag_of(key) * kOnes;
  const bool one_bucket = t.bucket_mask == 0;  // the only table without a pair of buckets
  for (u64 seen_buckets = 0; open; seen_buckets += 2) {
    // the tags of the pair that b belongs to: b's own first
    u64 tags, tags_of_neighbour;
    if (one_bucket) {
      tags = *tag_word(t, 0);
      tags_of_neighbour = 0;  // never looked at: the sequence ends behind its first bucket
    } else {
      const tag_pair_t both = *reinterpret_cast<const tag_pair_t*>(tag_word(t, b & ~1ull));
      tags = (b & 1ull) ? both.y : both.x;
      tags_of_neighbour = (b & 1ull) ? both.x : both.y;
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const u64 bb = b ^ (u64)half;
      bool ends = seen_buckets + half + 1 >= t.probe_limit;  // that was the last bucket a key may be in
      ends |= zero_bytes(tags) != 0;                         // a bucket with an EMPTY slot ends the probe sequence
      u64 cand = open ? zero_bytes(tags ^ mine) : 0;         // slots whose tag equals the key's
      const u64* bucket = bucket_words(t, bb);
      while (cand) {
        const int j = (__ffsll((unsigned long long)cand) - 1) >> 3;
        cand &= cand - 1;
        const u64 slot_key = bucket[j];
        u64 slot_value = bucket[kBucket + j];
        // both words are requested before the key is compared: left to itself the compiler asks for
        // the value only behind the comparison, a third dependent access (16 MiB of slots, every key
        // present: lookups 15 % faster with both in flight together)
        asm volatile("" : "+v"(slot_value));
        if (slot_key == key) {
          found = (int64_t)(bb * kBucket + j);
          value_out = slot_value;
          ends = true;
          cand = 0;
        }
      }
      open = open && !ends;
      tags = tags_of_neighbour;
    }
    b = (b + 2ull * step) & t.bucket_mask;
  }
  return found;
}

// The same search through the key words themselves, without the tags: the lane reads the 8 keys of a
// bucket (half of its 128-byte line) and, where its key is among them, the value from the same line.
// For a key that is present in the first bucket of its sequence this is ONE line instead of a line
// of tags plus the slot's line; for an absent key it is a line of slots where the tags would have
// been 16 bytes that are mostly cached.
__device__ __forceinline__ int64_t find_slot_in_keys(const Table& t, u64 key, bool valid, u64& value_out) {
  int64_t found = -1;
  bool open = valid && key != kEmpty && key != kTomb;
  u64 b = home_bucket(t, key);
  const u64 step = probe_step(key);
  for (u64 probes = 0; open; ++probes) {
    const u64* bucket = bucket_words(t, b);
    u64 seen[kBucket];
    load_bucket_keys(bucket, seen);
    int hit = -1;
    bool any_empty = false;
#pragma unroll
    for (int j = 0; j < kBucket; ++j) {
      if (seen[j] == key) hit = j;
      any_empty |= seen[j] == kEmpty;
    }
    if (hit >= 0) {
      found = (int64_t)(b * kBucket + hit);
      value_out = bucket[kBucket + hit];
    }
    open = hit < 0 && !any_empty && probes + 1 < t.probe_limit;
    b = next_bucket(t, b, step, probes);
  }
  return found;
}

// Lookup of one tile: up to 64 consecutive blocks of one request, one per lane (every lane of the
// wavefront must call). Consecutive blocks of a request are present as a prefix - a block's hash
// covers everything before it, and caches drop a sequence from its end - so the tile's LAST block
// says what to expect of the others: the wavefront reads the tags of that one key (one request) and,
// where they show the key, looks all its keys up in the key words directly (one line per key that
// is present); otherwise in the tags. Both searches return the same result for every key whatever
// the guess; only their cost differs. `ask` is the caller's state per request: it starts as the
// table's guess_present and goes off behind the first tile whose last block was absent (what
// follows a miss is not expected to be present, and need not pay for the question).
__device__ __forceinline__ u64 lookup_tile(const Table& t, u64 key, bool valid, bool& ask) {
  u64 value = kNoValue;
  const u64 live = __ballot(valid);
  bool in_keys = false;
  if (ask && live) {
    const int last = 63 - __clzll((unsigned long long)live);
    // the tile's last key as a scalar: its bucket, its tag, the read of its tags and their test
    // then cost the vector unit nothing
    const u64 k = readlane64(key, last);
    if (k != kEmpty && k != kTomb) {
      const u64 b = home_bucket(t, k);
      const u64 tags = *tag_word(t, b);
      in_keys = zero_bytes(tags ^ ((u64)tag_of(k) * kOnes)) != 0;
    }
    ask = in_keys;  // behind a tile whose last block is absent nothing is expected to be present
  }
  if (in_keys) (void)find_slot_in_keys(t, key, valid, value);
  else (void)find_slot(t, key, valid, value);
  return value;
}

// Request -> workgroup map of the kernels that probe the index once per block. Workgroup ids are
// dealt round-robin over the 8 XCDs; the requests go to the XCDs in runs, so that
// neighbouring requests - which tend to share a prefix, i.e. keys - meet in one L2 and run at the
// same time, while any long stretch of the batch (say, its longest requests, if the caller sorted
// it) is still spread over all XCDs.
// The run is 2^lg_run requests: 64 in a large batch, shorter in a small one so that every XCD
// still gets its share (64 requests: runs of 1, i.e. plain round-robin).
__device__ __forceinline__ int request_of_workgroup(unsigned id, int lg_run) {
  const unsigned xcd = id & 7u, k = id >> 3;  // k-th workgroup of this XCD
  return (int)((((k >> lg_run) * 8u + xcd) << lg_run) + (k & ((1u << lg_run) - 1u)));
}
inline int request_run_lg(int n_req) {
  int lg = 0;
  while (lg < 6 && (n_req >> (lg + 7)) > 0) ++lg;  // at least 8 runs per XCD before runs grow
  return lg;
}
inline unsigned workgroups_for_requests(int n_req, int lg_run) {
  const unsigned per_round = 8u << lg_run;
  return ((unsigned)n_req + per_round - 1) / per_round * per_round;
}

inline Table table_of(const aibx_index* ix) {
  Table t;
  t.slots = ix->slots;
  t.usage = ix->usage;
  t.tags = ix->tags;
  t.bucket_mask = ix->n_buckets - 1;
  t.probe_limit = ix->n_buckets < kMaxProbeBuckets ? ix->n_buckets : kMaxProbeBuckets;
  t.shift = 64 - ix->lg_buckets;
  t.guess_present = ix->n_slots >= kGuessPresentFrom;
  return t;
}

}  // namespace
}  // namespace aibx
