// GPU-resident cache index and prefix match (the cache pool's metadata and its "asynchronous
// metadata updates", Section 3.2.5 of the paper; the reusable-prefix test of the
// prefix-cache-aware policy, Section 3.2.2). Semantics are stated in aibx.h.
//
// Table: open addressing over buckets of 8 slots; a slot is {u64 key, u64 value}, so a bucket is
// one 128-byte line. Key 0 = EMPTY, key 2^64-1 = TOMBSTONE. A key lives in the first bucket of
// its probe sequence (home, home+step, home+2*step, ... mod n_buckets, step odd and key-dependent)
// that had a free slot when it was inserted.
// Invariant kept by every kernel: a probe sequence continues past a bucket only if that bucket
// has no EMPTY slot; so a lookup stops at the first bucket that has one.
//
// Execution shape. Lookups (prefix match): one lane per key, the lane reads the whole bucket.
// Updates (insert, evict): 8 lanes cooperate on one key - each reads one 16-byte slot, the 8 reads
// are one coalesced 128-byte line - so that the group can agree on the slot to claim; a wavefront
// owns 64 consecutive keys, loads them coalesced, and hands key 8g+r to lane group g in step r
// through cross-lane reads.
#include "common.h"

struct aibx_index {
  aibx::u64* slots;       // device, 2*n_slots words: {key, value} pairs
  aibx::u64 n_slots;
  aibx::u64 n_buckets;    // n_slots / 8, power of two
  int lg_buckets;
};

namespace aibx {
namespace {

constexpr u64 kEmpty = AIBX_KEY_EMPTY;
constexpr u64 kTomb = AIBX_KEY_TOMBSTONE;
constexpr u64 kNoValue = AIBX_NO_VALUE;
#ifndef AIBX_BUCKET_SLOTS
#define AIBX_BUCKET_SLOTS 8
#endif
constexpr int kBucket = AIBX_BUCKET_SLOTS;       // slots per bucket = lanes per key (4 or 8)
constexpr u64 kHomeMul = 0x9E3779B97F4A7C15ull;  // multiplicative (Fibonacci) bucket hash
constexpr int kIndexThreads = 256;
constexpr int kWavesPerGroup = kIndexThreads / kWave;

struct Table {
  u64* slots;
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

__device__ __forceinline__ u64 shfl64(u64 v, int src) {
  u32 lo = (u32)v, hi = (u32)(v >> 32);
  lo = __shfl(lo, src);
  hi = __shfl(hi, src);
  return ((u64)hi << 32) | lo;
}

// The 8 bits of a wavefront-wide ballot that belong to this lane's group.
__device__ __forceinline__ u32 group_bits(bool pred, int group) {
  return (u32)(__ballot(pred) >> (group * kBucket)) & ((1u << kBucket) - 1u);
}

__device__ __forceinline__ u64 load_key_fresh(const u64* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

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

// One workgroup of 4 wavefronts per request; wavefront w takes the request's blocks
// [64(w + 4k), +64) and requests the next tile's keys while this tile's buckets are in flight.
// Measured alternatives that lost: one wavefront per request (-20 %: long requests serialise),
// a flat pass over all blocks plus a first-miss pass (-15 %: second launch, values re-read), and
// lanes that refill themselves with their next key (no gain: the bound is lines requested).
__global__ __launch_bounds__(kIndexThreads) void prefix_match_kernel(
    Table t, const u64* __restrict__ hashes, const int64_t* __restrict__ blk_off,
    u64* __restrict__ values_out, int32_t* __restrict__ match_len) {
  __shared__ int lds_first[kWavesPerGroup];
  const int r = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t b0 = blk_off[r];
  const int64_t n_r = blk_off[r + 1] - b0;
  int64_t first_miss = n_r;
  int64_t base = (int64_t)wave * kWave;
  u64 k_next = base + lane < n_r ? hashes[b0 + base + lane] : kEmpty;
  for (; base < n_r; base += kIndexThreads) {
    const bool valid = base + lane < n_r;
    const u64 k = k_next;
    k_next = base + kIndexThreads + lane < n_r ? hashes[b0 + base + kIndexThreads + lane] : kEmpty;
    const u64 v = lookup_one(t, k, valid);
    if (valid && values_out) values_out[b0 + base + lane] = v;
    const u64 miss = __ballot(valid && v == kNoValue);
    if (miss && first_miss == n_r) first_miss = base + (__ffsll((unsigned long long)miss) - 1);
  }
  if (lane == 0) lds_first[wave] = (int)first_miss;
  __syncthreads();
  if (threadIdx.x == 0) {
    int m = lds_first[0];
    for (int w = 1; w < kWavesPerGroup; ++w) m = lds_first[w] < m ? lds_first[w] : m;
    match_len[r] = m;
  }
}

// ---- insert ------------------------------------------------------------------------------------
// Counters are summed per wavefront and added once.
__global__ __launch_bounds__(kIndexThreads) void index_insert_kernel(
    Table t, const u64* __restrict__ keys, const u64* __restrict__ values, int64_t n,
    u64* __restrict__ counters3) {
  const int lane = threadIdx.x & (kWave - 1);
  const int group = lane / kBucket, sub = lane % kBucket;
  const int64_t base = ((int64_t)blockIdx.x * kWavesPerGroup + threadIdx.x / kWave) * kWave;
  if (base >= n) return;
  const int64_t left = n - base;
  const int n_valid = left < kWave ? (int)left : kWave;
  const u64 my_key = lane < n_valid ? keys[base + lane] : kEmpty;
  const u64 my_val = lane < n_valid ? values[base + lane] : 0ull;
  u32 n_ins = 0, n_upd = 0, n_full = 0;  // meaningful in lanes with sub == 0
  const u64 n_buckets = t.bucket_mask + 1;

  for (int r = 0; r < kBucket; ++r) {
    const u64 key = shfl64(my_key, group * kBucket + r);
    const u64 val = shfl64(my_val, group * kBucket + r);
    const bool real = group * kBucket + r < n_valid;
    bool active = real && key != kEmpty && key != kTomb;
    if (real && !active) ++n_full;  // reserved key: dropped
    u64 b = home_bucket(t, key);
    const u64 step = probe_step(key);
    u64 probes = 0;                 // buckets fully scanned so far
    // candidate free slot (first in probe order); kept by the lane that owns it
    bool have_cand = false;         // group-uniform
    u64 cand_bucket = 0, cand_probes = 0;
    int cand_sub = 0;               // group-uniform
    u64 cand_expected = 0;          // valid in lane cand_sub
    // Proven bound on loop trips: a scan visits at most n_buckets buckets, and a scan is repeated
    // only after a lost claim, i.e. after some other insert filled a slot (at most n_slots times).
    u64 guard = n_buckets > (1ull << 30) ? ~0ull : n_buckets * (n_buckets * kBucket + 1);
    while (__any(active)) {
      u64* slot = t.slots + 2 * (b * kBucket + sub);
      const u64 seen = active ? load_key_fresh(slot) : kEmpty;
      const u32 hit = group_bits(active && seen == key, group);
      const u32 free_ = group_bits(active && (seen == kEmpty || seen == kTomb), group);
      const u32 empty = group_bits(active && seen == kEmpty, group);
      // the probe sequence ends at a bucket with an EMPTY slot, or after every bucket was seen
      const bool chain_ends = empty != 0 || probes + 1 >= n_buckets;
      bool claim = false;
      if (active) {
        if (hit) {  // present: overwrite the value
          if (sub == __ffs(hit) - 1) __hip_atomic_store(slot + 1, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ++n_upd;
          active = false;
        } else {
          if (!have_cand && free_) {
            have_cand = true;
            cand_sub = __ffs(free_) - 1;
            cand_bucket = b;
            cand_probes = probes;
            if (sub == cand_sub) cand_expected = seen;
          }
          if (!chain_ends) {
            b = (b + step) & t.bucket_mask;
            ++probes;
          } else if (!have_cand) {
            ++n_full;  // every slot of the table is taken
            active = false;
          } else {
            claim = true;  // key is absent: take the first free slot of its probe sequence
          }
        }
      }
      // claim step (all lanes take part in the cross-lane reads)
      u64* cslot = t.slots + 2 * (cand_bucket * kBucket + sub);
      u64 old = 0;
      if (claim && sub == cand_sub)
        old = atomicCAS((unsigned long long*)cslot, (unsigned long long)cand_expected, (unsigned long long)key);
      const u64 old_g = shfl64(old, group * kBucket + cand_sub);
      const u64 exp_g = shfl64(cand_expected, group * kBucket + cand_sub);
      if (claim) {
        if (old_g == exp_g) {          // slot is ours
          if (sub == cand_sub) __hip_atomic_store(cslot + 1, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ++n_ins;
          active = false;
        } else if (old_g == key) {     // the same key was stored there a moment ago
          if (sub == cand_sub) __hip_atomic_store(cslot + 1, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ++n_upd;
          active = false;
        } else {                       // another key took it: rescan from that bucket
          b = cand_bucket;
          probes = cand_probes;
          have_cand = false;
        }
      }
      if (--guard == 0 && active) {
        ++n_full;
        active = false;
      }
    }
  }
  if (counters3) {
    const bool leader = sub == 0;
    u32 a = leader ? n_ins : 0, u = leader ? n_upd : 0, f = leader ? n_full : 0;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      a += __shfl_xor(a, m);
      u += __shfl_xor(u, m);
      f += __shfl_xor(f, m);
    }
    if (lane == 0) {
      if (a) atomicAdd((unsigned long long*)counters3 + 0, (unsigned long long)a);
      if (u) atomicAdd((unsigned long long*)counters3 + 1, (unsigned long long)u);
      if (f) atomicAdd((unsigned long long*)counters3 + 2, (unsigned long long)f);
    }
  }
}

// ---- evict -------------------------------------------------------------------------------------
__global__ __launch_bounds__(kIndexThreads) void index_evict_kernel(
    Table t, const u64* __restrict__ keys, int64_t n, u64* __restrict__ values_out,
    u64* __restrict__ counters2) {
  const int lane = threadIdx.x & (kWave - 1);
  const int group = lane / kBucket, sub = lane % kBucket;
  const int64_t base = ((int64_t)blockIdx.x * kWavesPerGroup + threadIdx.x / kWave) * kWave;
  if (base >= n) return;
  const int64_t left = n - base;
  const int n_valid = left < kWave ? (int)left : kWave;
  const u64 my_key = lane < n_valid ? keys[base + lane] : kEmpty;
  u64 my_out = kNoValue;
  u32 n_ev = 0, n_miss = 0;
  const u64 n_buckets = t.bucket_mask + 1;

  for (int r = 0; r < kBucket; ++r) {
    const u64 key = shfl64(my_key, group * kBucket + r);
    const bool real = group * kBucket + r < n_valid;
    bool active = real && key != kEmpty && key != kTomb;
    if (real && !active) ++n_miss;
    u64 b = home_bucket(t, key);
    const u64 step = probe_step(key);
    u64 probes = 0;
    u64 result = kNoValue;  // group-uniform
    while (__any(active)) {
      u64* slot = t.slots + 2 * (b * kBucket + sub);
      const u64 seen = active ? load_key_fresh(slot) : kEmpty;
      const u32 hit = group_bits(active && seen == key, group);
      const u32 empty = group_bits(active && seen == kEmpty, group);
      u64 old = 0, val = 0;
      const int hit_sub = hit ? __ffs(hit) - 1 : 0;
      if (active && hit && sub == hit_sub) {
        // a bucket that still has an EMPTY slot ends every probe sequence through it, so its
        // removed slots can go straight back to EMPTY; otherwise leave a tombstone
        old = atomicCAS((unsigned long long*)slot, (unsigned long long)key,
                        (unsigned long long)(empty ? kEmpty : kTomb));
        if (old == key) val = slot[1];
      }
      const u64 old_g = shfl64(old, group * kBucket + hit_sub);
      const u64 val_g = shfl64(val, group * kBucket + hit_sub);
      if (active) {
        if (hit) {
          if (old_g == key) { result = val_g; ++n_ev; }
          else ++n_miss;              // another entry of this batch removed it first
          active = false;
        } else if (empty || probes + 1 >= n_buckets) {
          ++n_miss;
          active = false;
        } else {
          b = (b + step) & t.bucket_mask;
          ++probes;
        }
      }
    }
    if (sub == r) my_out = result;
  }
  if (values_out && lane < n_valid) values_out[base + lane] = my_out;
  if (counters2) {
    const bool leader = sub == 0;
    u32 e = leader ? n_ev : 0, m2 = leader ? n_miss : 0;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      e += __shfl_xor(e, m);
      m2 += __shfl_xor(m2, m);
    }
    if (lane == 0) {
      if (e) atomicAdd((unsigned long long*)counters2 + 0, (unsigned long long)e);
      if (m2) atomicAdd((unsigned long long*)counters2 + 1, (unsigned long long)m2);
    }
  }
}

// ---- whole-table passes ------------------------------------------------------------------------
__global__ __launch_bounds__(kIndexThreads) void fill_zero_kernel(uint4* p, u64 n_vec) {
  for (u64 i = (u64)blockIdx.x * kIndexThreads + threadIdx.x; i < n_vec; i += (u64)gridDim.x * kIndexThreads)
    p[i] = uint4{0, 0, 0, 0};
}

__global__ void zero_word_kernel(u64* p) { *p = 0; }

__global__ __launch_bounds__(kIndexThreads) void index_count_kernel(const u64* slots, u64 n_slots, u64* live_out) {
  u32 mine = 0;
  for (u64 i = (u64)blockIdx.x * kIndexThreads + threadIdx.x; i < n_slots; i += (u64)gridDim.x * kIndexThreads) {
    const u64 k = slots[2 * i];
    mine += (k != kEmpty && k != kTomb);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) mine += __shfl_xor(mine, m);
  if ((threadIdx.x & (kWave - 1)) == 0 && mine) atomicAdd((unsigned long long*)live_out, (unsigned long long)mine);
}

__global__ __launch_bounds__(kIndexThreads) void index_dump_kernel(const u64* slots, u64 n_slots, u64* keys_out,
                                                                  u64* values_out, u64 capacity, u64* n_out) {
  const int lane = threadIdx.x & (kWave - 1);
  const u64 stride = (u64)gridDim.x * kIndexThreads;
  // trip count is the same for all lanes of a wavefront (the ballot needs them all)
  for (u64 i0 = (u64)blockIdx.x * kIndexThreads + (threadIdx.x - lane); i0 < n_slots; i0 += stride) {
    const u64 i = i0 + lane;
    u64 k = kEmpty, v = 0;
    if (i < n_slots) {
      k = slots[2 * i];
      v = slots[2 * i + 1];
    }
    const bool live = k != kEmpty && k != kTomb;
    const u64 mask = __ballot(live);
    if (mask == 0) continue;
    u64 start = 0;
    if (lane == 0) start = atomicAdd((unsigned long long*)n_out, (unsigned long long)__popcll(mask));
    start = shfl64(start, 0);
    if (live) {
      const u64 pos = start + __popcll(mask & ((1ull << lane) - 1ull));
      if (pos < capacity) {
        keys_out[pos] = k;
        values_out[pos] = v;
      }
    }
  }
}

Table table_of(const aibx_index* ix) {
  Table t;
  t.slots = ix->slots;
  t.bucket_mask = ix->n_buckets - 1;
  t.shift = 64 - ix->lg_buckets;
  return t;
}

int check_slots(u64 n_slots) {
  if (n_slots < 8 || n_slots > (1ull << 36) || (n_slots & (n_slots - 1))) return AIBX_ERR_UNSUPPORTED;
  return AIBX_OK;
}

u32 pass_grid(u64 n_items) {
  const u64 want = (n_items + kIndexThreads - 1) / kIndexThreads;
  return (u32)(want < 1 ? 1 : (want > 8192 ? 8192 : want));
}

}  // namespace
}  // namespace aibx

using namespace aibx;

extern "C" {

int aibx_index_storage_bytes(uint64_t n_slots, size_t* out_bytes) {
  if (!out_bytes) return AIBX_ERR_INVALID_ARG;
  const int rc = check_slots(n_slots);
  if (rc != AIBX_OK) return rc;
  *out_bytes = (size_t)n_slots * 16;
  return AIBX_OK;
}

int aibx_index_clear(aibx_index_t* index, void* stream) {
  if (!index) return AIBX_ERR_INVALID_ARG;
  const u64 n_vec = index->n_slots;  // one 16-byte vector per slot
  fill_zero_kernel<<<pass_grid(n_vec), kIndexThreads, 0, as_stream(stream)>>>(
      reinterpret_cast<uint4*>(index->slots), n_vec);
  return launch_status();
}

int aibx_index_create(void* d_storage, size_t bytes, uint64_t n_slots, void* stream,
                      aibx_index_t** out) {
  if (!out || !d_storage) return AIBX_ERR_INVALID_ARG;
  *out = nullptr;
  const int rc = check_slots(n_slots);
  if (rc != AIBX_OK) return rc;
  if (bytes < (size_t)n_slots * 16) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_storage, 256)) return AIBX_ERR_ALIGN;
  aibx_index* ix = new aibx_index();
  ix->slots = static_cast<u64*>(d_storage);
  ix->n_slots = n_slots;
  ix->n_buckets = n_slots / kBucket;
  ix->lg_buckets = 0;
  while ((1ull << ix->lg_buckets) < ix->n_buckets) ++ix->lg_buckets;
  const int rc2 = aibx_index_clear(ix, stream);
  if (rc2 != AIBX_OK) {
    delete ix;
    return rc2;
  }
  *out = ix;
  return AIBX_OK;
}

int aibx_index_destroy(aibx_index_t* index) {
  delete index;
  return AIBX_OK;
}

int aibx_index_insert(aibx_index_t* index, const uint64_t* d_keys, const uint64_t* d_values,
                      int64_t n, uint64_t* d_counters3, void* stream) {
  if (!index || n < 0) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!d_keys || !d_values) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_keys, 8) || !aligned(d_values, 8) || !aligned(d_counters3, 8)) return AIBX_ERR_ALIGN;
  const int64_t groups = (n + kIndexThreads - 1) / kIndexThreads;
  if (groups > 0x7FFFFFFF) return AIBX_ERR_UNSUPPORTED;
  index_insert_kernel<<<(u32)groups, kIndexThreads, 0, as_stream(stream)>>>(table_of(index), d_keys, d_values, n,
                                                                            d_counters3);
  return launch_status();
}

int aibx_index_evict(aibx_index_t* index, const uint64_t* d_keys, int64_t n, uint64_t* d_values_out,
                     uint64_t* d_counters2, void* stream) {
  if (!index || n < 0) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!d_keys) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_keys, 8) || !aligned(d_values_out, 8) || !aligned(d_counters2, 8)) return AIBX_ERR_ALIGN;
  const int64_t groups = (n + kIndexThreads - 1) / kIndexThreads;
  if (groups > 0x7FFFFFFF) return AIBX_ERR_UNSUPPORTED;
  index_evict_kernel<<<(u32)groups, kIndexThreads, 0, as_stream(stream)>>>(table_of(index), d_keys, n,
                                                                           d_values_out, d_counters2);
  return launch_status();
}

int aibx_index_count(const aibx_index_t* index, uint64_t* d_live_out, void* stream) {
  if (!index || !d_live_out) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_live_out, 8)) return AIBX_ERR_ALIGN;
  hipStream_t st = as_stream(stream);
  zero_word_kernel<<<1, 1, 0, st>>>(d_live_out);
  index_count_kernel<<<pass_grid(index->n_slots), kIndexThreads, 0, st>>>(index->slots, index->n_slots, d_live_out);
  return launch_status();
}

int aibx_index_dump(const aibx_index_t* index, uint64_t* d_keys_out, uint64_t* d_values_out,
                    uint64_t capacity, uint64_t* d_n_out, void* stream) {
  if (!index || !d_n_out) return AIBX_ERR_INVALID_ARG;
  if (capacity && (!d_keys_out || !d_values_out)) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_keys_out, 8) || !aligned(d_values_out, 8) || !aligned(d_n_out, 8)) return AIBX_ERR_ALIGN;
  hipStream_t st = as_stream(stream);
  zero_word_kernel<<<1, 1, 0, st>>>(d_n_out);
  index_dump_kernel<<<pass_grid(index->n_slots), kIndexThreads, 0, st>>>(index->slots, index->n_slots, d_keys_out,
                                                                         d_values_out, capacity, d_n_out);
  return launch_status();
}

int aibx_prefix_match(const aibx_index_t* index, const uint64_t* d_hashes, const int64_t* d_blk_off,
                      int32_t n_req, int64_t n_blocks_total, uint64_t* d_values_out,
                      int32_t* d_match_len, void* stream) {
  if (!index || n_req < 0 || n_blocks_total < 0) return AIBX_ERR_INVALID_ARG;
  if (n_req == 0) return AIBX_OK;
  if (!d_blk_off || !d_match_len || (n_blocks_total > 0 && !d_hashes)) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_hashes, 8) || !aligned(d_blk_off, 8) || !aligned(d_values_out, 8) || !aligned(d_match_len, 4))
    return AIBX_ERR_ALIGN;
  prefix_match_kernel<<<(u32)n_req, kIndexThreads, 0, as_stream(stream)>>>(table_of(index), d_hashes, d_blk_off,
                                                                           d_values_out, d_match_len);
  return launch_status();
}

}  // extern "C"
