// GPU-resident cache index and prefix match (the cache pool's metadata, which Section 3.2.5 of the
// paper updates asynchronously, off the engines' critical path; the reusable-prefix test of the
// prefix-cache-aware policy, Section 3.2.2). Semantics are stated in aibx.h.
//
// Behind the slots the storage holds one 32-bit usage word per slot (touch count and last epoch)
// for the victim selection of the eviction policy, and behind those one tag byte per slot, which
// is all a lookup reads until a tag matches (index_device.h).
// Table: open addressing over buckets of 8 slots; a bucket is one 128-byte line holding its 8 keys
// and then its 8 values. Key 0 = EMPTY, key 2^64-1 = TOMBSTONE. A key lives in the first bucket of
// its probe sequence (home, its neighbour home^1, home+2*step, that one's neighbour, ... mod
// n_buckets, step odd and key-dependent: pairs of neighbouring buckets visited by double hashing)
// that had a free slot when it was inserted.
// Invariant kept by every kernel: a probe sequence continues past a bucket only if that bucket
// has no EMPTY slot; so a lookup stops at the first bucket that has one.
//
// Execution shape: one lane per key in every kernel; the lane reads its key's whole bucket. Random
// line reads on this GPU are bound by the number of lines requested (about 55-80 G lines/s whether
// a line is fetched by one lane or by eight cooperating ones), so lane-per-key costs the memory
// system nothing extra, needs no cross-lane traffic, and keeps 64 probes per wavefront in flight.
#include "index_device.h"

namespace aibx {
namespace {

// One workgroup of kWaves wavefronts per request; wavefront w takes the request's blocks
// [64(w + kWaves*k), +64) and requests the next tile's keys while this tile's buckets are in flight.
// Measured alternatives that lost: one wavefront per request (-20 %: long requests serialise),
// a flat pass over all blocks plus a first-miss pass (-15 %: second launch, values re-read), and
// lanes that refill themselves with their next key (no gain: the bound is lines requested).
template <int kWaves>
__global__ __launch_bounds__(kWaves* kWave) void prefix_match_kernel(
    Table t, const u64* __restrict__ hashes, const int64_t* __restrict__ blk_off,
    u64* __restrict__ values_out, int32_t* __restrict__ match_len, int n_req, int lg_run) {
  __shared__ int lds_first[kWaves];
  // (config 2, groups of 8 neighbouring requests sharing half their blocks: 58 -> 77 G probes/s
  // against request = workgroup id)
  const int r = request_of_workgroup(blockIdx.x, lg_run);
  if (r >= n_req) return;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t b0 = blk_off[r];
  const int64_t n_r = blk_off[r + 1] - b0;
  // a request of at most 64 blocks is one wavefront's work: the others leave, and no barrier is needed
  const bool solo = kWaves == 1 || n_r <= kWave;
  if (solo && wave != 0) return;
  constexpr int kStride = kWaves * kWave;
  int64_t first_miss = n_r;
  int64_t base = (int64_t)wave * kWave;
  u64 k_next = base + lane < n_r ? hashes[b0 + base + lane] : kEmpty;
  bool ask = t.guess_present;
  for (; base < n_r; base += kStride) {
    const bool valid = base + lane < n_r;
    const u64 k = k_next;
    k_next = base + kStride + lane < n_r ? hashes[b0 + base + kStride + lane] : kEmpty;
    const u64 v = lookup_tile(t, k, valid, ask);
    if (valid && values_out) values_out[b0 + base + lane] = v;
    const u64 miss = __ballot(valid && v == kNoValue);
    if (miss && first_miss == n_r) first_miss = base + (__ffsll((unsigned long long)miss) - 1);
    // without per-block values to report, nothing behind this wavefront's first miss matters
    // (its tiles come in rising order)
    if (!values_out && first_miss != n_r) break;
  }
  if (solo) {
    if (lane == 0) match_len[r] = (int)first_miss;
    return;
  }
  if (lane == 0) lds_first[wave] = (int)first_miss;
  __syncthreads();
  if (threadIdx.x == 0) {
    int m = lds_first[0];
    for (int w = 1; w < kWaves; ++w) m = lds_first[w] < m ? lds_first[w] : m;
    match_len[r] = m;
  }
}

// ---- insert ------------------------------------------------------------------------------------
// One lane per key, like the lookups: the lane reads the buckets of its probe sequence, remembers
// the first free slot, and when the sequence ends without a hit claims that slot with a 64-bit
// compare-and-swap. Losing the claim to another key means rescanning from that bucket; losing it
// to the same key (a duplicate in the batch) is an update. Slots only ever go from free to taken
// while this kernel runs, so two lanes inserting the same key always race for the same slot and
// the key cannot end up stored twice.
// The first scan uses ordinary cached loads. Other workgroups are claiming slots at the same time,
// so that view can be stale - but only towards "free" (a slot it shows taken is taken for good,
// with the same key), and the compare-and-swap is the arbiter: a claim on a slot that is no longer
// free fails, and from then on the lane rescans with agent-scope loads. This keeps the common paths
// (update of a present key, claim of a free slot) at one line read plus one write.
__device__ __forceinline__ u64 load_key_fresh(const u64* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Values are written with ordinary stores: nothing reads a value before the kernel ends (lookups
// and evictions run in later launches), and the bytes of a value are written by one key's lanes
// only (duplicates of a key in a batch carry the same value).
__device__ __forceinline__ void store_value(u64* p, u64 v) { *p = v; }

__device__ __forceinline__ u32 wave_sum(u32 v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}

// Sum over the workgroup (every thread must call it); valid in thread 0. Counters are added with
// one atomic per workgroup and the grids are capped, because atomics on one address serialise at
// about 13 ns each: one per wavefront made a 12 M-key insert spend 2.3 ms on its counters alone.
__device__ __forceinline__ u32 group_sum(u32 v) {
  __shared__ u32 part[kWavesPerGroup];
  v = wave_sum(v);
  __syncthreads();  // a previous call's readers are done with part[]
  if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = v;
  __syncthreads();
  u32 total = 0;
  if (threadIdx.x == 0)
    for (int w = 0; w < kWavesPerGroup; ++w) total += part[w];
  return total;
}

// Where the (key, value) pairs of an insert come from: a batch handed in by the caller, or the
// live slots of another table (rebuild), which also bring their usage word along.
struct BatchSource {
  const u64* __restrict__ keys;
  const u64* __restrict__ values;
  int64_t n;
  __device__ __forceinline__ bool get(int64_t i, u64& key, u64& val, u32& use) const {
    key = keys[i];
    val = values[i];
    use = 0;  // a new key starts untouched
    return true;
  }
};
struct TableSource {
  const u64* __restrict__ slots;
  const u32* __restrict__ usage;
  int64_t n;  // slots of the source table
  __device__ __forceinline__ bool get(int64_t i, u64& key, u64& val, u32& use) const {
    const u64 w = key_word_of_slot((u64)i);
    key = slots[w];
    if (key == kEmpty || key == kTomb) return false;  // nothing stored here
    val = slots[w + kBucket];
    use = usage[i];
    return true;
  }
};

template <class Source>
__global__ __launch_bounds__(kIndexThreads) void index_insert_kernel(Table t, Source src,
                                                                    u64* __restrict__ counters3) {
  u32 n_ins = 0, n_upd = 0, n_full = 0;
  const u64 n_buckets = t.bucket_mask + 1;
  const int64_t n = src.n;
  for (int64_t i = (int64_t)blockIdx.x * kIndexThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kIndexThreads) {
  u64 key, val;
  u32 use;
  if (!src.get(i, key, val, use)) continue;
  bool active = key != kEmpty && key != kTomb;
  if (!active) ++n_full;  // reserved key: dropped
  const u64 step = probe_step(key);
  u64 b = home_bucket(t, key);
  u64 probes = 0;  // buckets of the probe sequence already examined
  bool have_cand = false;
  u64 cand_bucket = 0, cand_probes = 0, cand_expected = 0;
  int cand_slot = 0;
  // Proven bound on loop trips: a scan visits at most probe_limit buckets, and a scan is repeated
  // only after a lost claim, i.e. after some other insert filled a slot (at most n_slots times).
  u64 guard = t.probe_limit * (n_buckets * kBucket + 1);  // < 2^12 * 2^37
  bool fresh = false;  // set after a lost claim
  while (active) {
    u64* bucket = bucket_words(t, b);
    u64 seen[kBucket];
    if (fresh) {
#pragma unroll
      for (int j = 0; j < kBucket; ++j) seen[j] = load_key_fresh(bucket + j);
    } else {
      load_bucket_keys(bucket, seen);
    }
    int hit = -1, first_free = -1;
    bool any_empty = false;
#pragma unroll
    for (int j = kBucket - 1; j >= 0; --j) {
      if (seen[j] == key) hit = j;
      if (seen[j] == kEmpty || seen[j] == kTomb) first_free = j;
      any_empty |= seen[j] == kEmpty;
    }
    if (hit >= 0) {  // present: overwrite the value
      store_value(bucket + kBucket + hit, val);
      ++n_upd;
      break;
    }
    if (!have_cand && first_free >= 0) {
      have_cand = true;
      cand_bucket = b;
      cand_probes = probes;
      cand_slot = first_free;
      cand_expected = seen[0];
#pragma unroll
      for (int j = 1; j < kBucket; ++j) cand_expected = first_free == j ? seen[j] : cand_expected;
    }
    // the probe sequence ends at a bucket with an EMPTY slot, or after every bucket was seen
    if (!any_empty && probes + 1 < t.probe_limit) {
      b = next_bucket(t, b, step, probes);
      ++probes;
    } else if (!have_cand) {
      ++n_full;  // every slot the key may use is taken
      break;
    } else {
      u64* cslot = bucket_words(t, cand_bucket) + cand_slot;  // the candidate's key word
      const u64 old = atomicCAS((unsigned long long*)cslot, (unsigned long long)cand_expected,
                                (unsigned long long)key);
      if (old == cand_expected) {  // the slot is ours
        store_value(cslot + kBucket, val);
        t.usage[cand_bucket * kBucket + cand_slot] = use;
        t.tags[cand_bucket * kBucket + cand_slot] = (unsigned char)tag_of(key);
        ++n_ins;
        break;
      }
      if (old == key) {  // the same key was stored there a moment ago
        store_value(cslot + kBucket, val);
        ++n_upd;
        break;
      }
      b = cand_bucket;  // another key took it: rescan from that bucket, with fresh loads
      probes = cand_probes;
      have_cand = false;
      fresh = true;
    }
    if (--guard == 0) {
      ++n_full;
      break;
    }
  }
  }  // keys of this lane
  if (counters3) {
    const u32 a = group_sum(n_ins), u = group_sum(n_upd), f = group_sum(n_full);
    if (threadIdx.x == 0) {
      if (a) atomicAdd((unsigned long long*)counters3 + 0, (unsigned long long)a);
      if (u) atomicAdd((unsigned long long*)counters3 + 1, (unsigned long long)u);
      if (f) atomicAdd((unsigned long long*)counters3 + 2, (unsigned long long)f);
    }
  }
}

// ---- evict -------------------------------------------------------------------------------------
// One lane per key. The key's slot goes back to EMPTY when its bucket still has an EMPTY slot
// (such a bucket ends every probe sequence that reaches it, so nothing lies beyond it), otherwise
// it becomes a tombstone. The compare-and-swap decides which of several entries naming the same
// key reports the value. Ordinary cached loads suffice: while this kernel runs slots only go from
// taken to free, so a stale view can only show a key that is already gone (the swap then fails and
// the entry counts as missing) or overlook a fresh EMPTY (a tombstone is written where EMPTY
// would have done, or the scan goes one bucket further than needed).
__global__ __launch_bounds__(kIndexThreads) void index_evict_kernel(
    Table t, const u64* __restrict__ keys, int64_t n, u64* __restrict__ values_out,
    u64* __restrict__ counters2) {
  u32 n_ev = 0, n_miss = 0;
  for (int64_t i = (int64_t)blockIdx.x * kIndexThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kIndexThreads) {
  const u64 key = keys[i];
  u64 result = kNoValue;
  bool active = key != kEmpty && key != kTomb;
  const u64 step = probe_step(key);
  u64 b = home_bucket(t, key);
  for (u64 probes = 0; active; ++probes) {
    u64* bucket = bucket_words(t, b);
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
      u64* slot = bucket + hit;
      const u64 old = atomicCAS((unsigned long long*)slot, (unsigned long long)key,
                                (unsigned long long)(any_empty ? kEmpty : kTomb));
      if (old == key) {  // otherwise another entry of this batch removed it first
        result = slot[kBucket];
        t.tags[b * kBucket + hit] = (unsigned char)(any_empty ? kTagEmpty : kTagTomb);
      }
      break;
    }
    if (any_empty || probes + 1 >= t.probe_limit) break;
    b = next_bucket(t, b, step, probes);
  }
  if (values_out) values_out[i] = result;
  if (result != kNoValue) ++n_ev;
  else ++n_miss;
  }  // keys of this lane
  if (counters2) {
    const u32 e = group_sum(n_ev), m = group_sum(n_miss);
    if (threadIdx.x == 0) {
      if (e) atomicAdd((unsigned long long*)counters2 + 0, (unsigned long long)e);
      if (m) atomicAdd((unsigned long long*)counters2 + 1, (unsigned long long)m);
    }
  }
}

// ---- usage tracking and victim selection -------------------------------------------------------
// (the eviction policy of Section 3.2.5, which a one-off scan must not disturb; the rule is stated in aibx.h)
// touch: one lane per key; finds the key's slot like a lookup and bumps its usage word with a
// compare-and-swap loop (count saturates at 255, epoch only moves forward).
__global__ __launch_bounds__(kIndexThreads) void index_touch_kernel(Table t, const u64* __restrict__ keys,
                                                                   int64_t n, u32 epoch) {
  for (int64_t i = (int64_t)blockIdx.x * kIndexThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kIndexThreads) {
    u64 unused_value;
    const int64_t slot = find_slot(t, keys[i], true, unused_value);
    if (slot < 0) continue;  // absent keys are ignored
    u32* word = t.usage + slot;
    u32 seen = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {  // ends: every failed swap means another touch of this key went through
      const u32 count = seen >> 24, last = seen & kEpochMask;
      const u32 want = ((count < 255 ? count + 1 : 255u) << 24) | (epoch > last ? epoch : last);
      const u32 old = atomicCAS(word, seen, want);
      if (old == seen) break;
      seen = old;
    }
  }
}

// age: halves every touch count (one streaming pass over the usage words).
__global__ __launch_bounds__(kIndexThreads) void index_age_kernel(u32* usage, u64 n_slots) {
  for (u64 i = (u64)blockIdx.x * kIndexThreads + threadIdx.x; i < n_slots; i += (u64)gridDim.x * kIndexThreads) {
    const u32 w = usage[i];
    usage[i] = ((w >> 25) << 24) | (w & kEpochMask);
  }
}

// ---- whole-table passes ------------------------------------------------------------------------
__global__ __launch_bounds__(kIndexThreads) void fill_zero_kernel(u64* p, u64 n_words) {
  for (u64 i = (u64)blockIdx.x * kIndexThreads + threadIdx.x; i < n_words; i += (u64)gridDim.x * kIndexThreads)
    p[i] = 0ull;
}

__global__ void zero_word_kernel(u64* p, int n) {
  for (int i = 0; i < n; ++i) p[i] = 0;
}

// out2[0] += live slots; out2[1] += tombstones when want_tombstones (else out2 has one word only)
__global__ __launch_bounds__(kIndexThreads) void index_count_kernel(const u64* slots, u64 n_slots, u64* out2,
                                                                   bool want_tombstones) {
  u32 live = 0, tombs = 0;
  for (u64 i = (u64)blockIdx.x * kIndexThreads + threadIdx.x; i < n_slots; i += (u64)gridDim.x * kIndexThreads) {
    const u64 k = slots[key_word_of_slot(i)];
    live += (k != kEmpty && k != kTomb);
    tombs += k == kTomb;
  }
  const u32 total = group_sum(live);
  if (threadIdx.x == 0 && total) atomicAdd((unsigned long long*)out2, (unsigned long long)total);
  if (want_tombstones) {
    const u32 total_t = group_sum(tombs);
    if (threadIdx.x == 0 && total_t) atomicAdd((unsigned long long*)out2 + 1, (unsigned long long)total_t);
  }
}

// Dump and victim selection: emit the (key, value) pairs of the slots that pass a test, in no
// particular order. Every workgroup owns one contiguous stretch of the table, every wavefront a
// quarter of it, and goes over it twice: first it counts its matches (a ballot per 64 slots, so the
// count is a scalar) and the workgroup reserves that many output positions with ONE atomic (an
// atomic per wavefront on the shared counter serialises at ~13 ns each and made a scan of a
// 16 M-slot table take 3 ms); then every wavefront re-reads its quarter - mostly from cache - and
// writes its matches behind those of the wavefronts before it. Two barriers per workgroup, none
// per tile.
constexpr int kEmitBatch = 4;
struct EmitTest {
  bool victims;        // false: every live key; true: live, count < protect_count, last < before_epoch
  u32 protect_count, before_epoch;
};

__device__ __forceinline__ bool emit_passes(const EmitTest& e, u64 key, u32 usage) {
  const bool live = key != kEmpty && key != kTomb;
  if (!e.victims) return live;
  return live && (usage >> 24) < e.protect_count && (usage & kEpochMask) < e.before_epoch;
}

__global__ __launch_bounds__(kIndexThreads) void index_emit_kernel(const u64* slots, const u32* usage, u64 n_slots,
                                                                  EmitTest test, u64* keys_out, u64* values_out,
                                                                  u64 capacity, u64* n_out) {
  __shared__ u64 lds_base;
  __shared__ u32 lds_wave[kWavesPerGroup];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  u64 chunk = (n_slots + gridDim.x - 1) / gridDim.x;
  chunk = (chunk + kIndexThreads - 1) / kIndexThreads * kIndexThreads;  // a multiple of 64 per wavefront
  const u64 part = chunk / kWavesPerGroup;
  const u64 begin = (u64)blockIdx.x * chunk + (u64)wave * part;       // this wavefront's slots
  const u64 end = begin + part < n_slots ? begin + part : n_slots;
  // kEmitBatch tiles of 64 slots per trip, all their loads requested before the first is used: one
  // memory latency per trip instead of one (two with the value behind the test) per tile
  u32 mine = 0;  // the same in every lane of the wavefront
  for (u64 tile = begin; tile < end; tile += kEmitBatch * kWave) {
    u64 k[kEmitBatch];
    u32 u[kEmitBatch];
#pragma unroll
    for (int j = 0; j < kEmitBatch; ++j) {
      const u64 i = tile + (u64)j * kWave + lane;
      k[j] = i < end ? slots[key_word_of_slot(i)] : kEmpty;
      u[j] = (i < end && test.victims) ? usage[i] : 0u;
    }
#pragma unroll
    for (int j = 0; j < kEmitBatch; ++j) mine += (u32)__popcll(__ballot(emit_passes(test, k[j], u[j])));
  }
  if (lane == 0) lds_wave[wave] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    u32 total = 0;
    for (int w = 0; w < kWavesPerGroup; ++w) total += lds_wave[w];
    lds_base = total ? atomicAdd((unsigned long long*)n_out, (unsigned long long)total) : 0ull;
  }
  __syncthreads();
  u64 pos0 = lds_base;  // next free output position of this wavefront
  for (int w = 0; w < wave; ++w) pos0 += lds_wave[w];
  for (u64 tile = begin; tile < end; tile += kEmitBatch * kWave) {
    u64 k[kEmitBatch], v[kEmitBatch];
    u32 u[kEmitBatch];
#pragma unroll
    for (int j = 0; j < kEmitBatch; ++j) {  // the value comes with its key: same 128-byte line
      const u64 i = tile + (u64)j * kWave + lane;
      k[j] = i < end ? slots[key_word_of_slot(i)] : kEmpty;
      v[j] = i < end ? slots[key_word_of_slot(i) + kBucket] : 0ull;
      u[j] = (i < end && test.victims) ? usage[i] : 0u;
    }
#pragma unroll
    for (int j = 0; j < kEmitBatch; ++j) {
      const bool pass = emit_passes(test, k[j], u[j]);
      const u64 mask = __ballot(pass);
      if (pass) {
        const u64 pos = pos0 + __popcll(mask & ((1ull << lane) - 1ull));
        if (pos < capacity) {
          keys_out[pos] = k[j];
          values_out[pos] = v[j];
        }
      }
      pos0 += __popcll(mask);
    }
  }
}

int check_slots(u64 n_slots) {
  if (n_slots < 8 || n_slots > (1ull << 36) || (n_slots & (n_slots - 1))) return AIBX_ERR_UNSUPPORTED;
  return AIBX_OK;
}

u32 pass_grid(u64 n_items) {
  const u64 want = (n_items + kIndexThreads - 1) / kIndexThreads;
  return (u32)(want < 1 ? 1 : (want > 2048 ? 2048 : want));  // 2048 x 256 lanes fill the GPU once
}

}  // namespace
}  // namespace aibx

using namespace aibx;

extern "C" {

int aibx_index_storage_bytes(uint64_t n_slots, size_t* out_bytes) {
  if (!out_bytes) return AIBX_ERR_INVALID_ARG;
  const int rc = check_slots(n_slots);
  if (rc != AIBX_OK) return rc;
  *out_bytes = (size_t)n_slots * kStorageBytesPerSlot;
  return AIBX_OK;
}

int aibx_index_clear(aibx_index_t* index, void* stream) {
  if (!index) return AIBX_ERR_INVALID_ARG;
  const u64 n_words = index->n_slots * kStorageBytesPerSlot / 8;  // slots, usage words and tags (n_slots % 8 == 0)
  fill_zero_kernel<<<pass_grid(n_words), kIndexThreads, 0, as_stream(stream)>>>(index->slots, n_words);
  return launch_status();
}

int aibx_index_create(void* d_storage, size_t bytes, uint64_t n_slots, void* stream,
                      aibx_index_t** out) {
  if (!out || !d_storage) return AIBX_ERR_INVALID_ARG;
  *out = nullptr;
  const int rc = check_slots(n_slots);
  if (rc != AIBX_OK) return rc;
  if (bytes < (size_t)n_slots * kStorageBytesPerSlot) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_storage, 256)) return AIBX_ERR_ALIGN;
  aibx_index* ix = new aibx_index();
  ix->slots = static_cast<u64*>(d_storage);
  ix->usage = reinterpret_cast<u32*>(ix->slots + 2 * n_slots);
  ix->tags = reinterpret_cast<unsigned char*>(ix->usage + n_slots);
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
  index_insert_kernel<<<pass_grid((u64)n), kIndexThreads, 0, as_stream(stream)>>>(
      table_of(index), BatchSource{d_keys, d_values, n}, d_counters3);
  return launch_status();
}

int aibx_index_evict(aibx_index_t* index, const uint64_t* d_keys, int64_t n, uint64_t* d_values_out,
                     uint64_t* d_counters2, void* stream) {
  if (!index || n < 0) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!d_keys) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_keys, 8) || !aligned(d_values_out, 8) || !aligned(d_counters2, 8)) return AIBX_ERR_ALIGN;
  index_evict_kernel<<<pass_grid((u64)n), kIndexThreads, 0, as_stream(stream)>>>(table_of(index), d_keys, n,
                                                                                  d_values_out, d_counters2);
  return launch_status();
}

int aibx_index_touch(aibx_index_t* index, const uint64_t* d_keys, int64_t n, uint32_t epoch, void* stream) {
  if (!index || n < 0 || epoch > kEpochMask) return AIBX_ERR_INVALID_ARG;
  if (n == 0) return AIBX_OK;
  if (!d_keys) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_keys, 8)) return AIBX_ERR_ALIGN;
  index_touch_kernel<<<pass_grid((u64)n), kIndexThreads, 0, as_stream(stream)>>>(table_of(index), d_keys, n, epoch);
  return launch_status();
}

int aibx_index_age(aibx_index_t* index, void* stream) {
  if (!index) return AIBX_ERR_INVALID_ARG;
  index_age_kernel<<<pass_grid(index->n_slots), kIndexThreads, 0, as_stream(stream)>>>(index->usage, index->n_slots);
  return launch_status();
}

int aibx_index_select_victims(const aibx_index_t* index, uint32_t protect_count, uint32_t before_epoch,
                              uint64_t* d_keys_out, uint64_t* d_values_out, uint64_t capacity,
                              uint64_t* d_n_out, void* stream) {
  if (!index || !d_n_out) return AIBX_ERR_INVALID_ARG;
  if (capacity && (!d_keys_out || !d_values_out)) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_keys_out, 8) || !aligned(d_values_out, 8) || !aligned(d_n_out, 8)) return AIBX_ERR_ALIGN;
  hipStream_t st = as_stream(stream);
  zero_word_kernel<<<1, 1, 0, st>>>(d_n_out, 1);
  index_emit_kernel<<<pass_grid(index->n_slots), kIndexThreads, 0, st>>>(
      index->slots, index->usage, index->n_slots, EmitTest{true, protect_count, before_epoch}, d_keys_out,
      d_values_out, capacity, d_n_out);
  return launch_status();
}

int aibx_index_count(const aibx_index_t* index, uint64_t* d_live_out, void* stream) {
  if (!index || !d_live_out) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_live_out, 8)) return AIBX_ERR_ALIGN;
  hipStream_t st = as_stream(stream);
  zero_word_kernel<<<1, 1, 0, st>>>(d_live_out, 1);
  index_count_kernel<<<pass_grid(index->n_slots), kIndexThreads, 0, st>>>(index->slots, index->n_slots, d_live_out,
                                                                         false);
  return launch_status();
}

int aibx_index_stats(const aibx_index_t* index, uint64_t* d_out2, void* stream) {
  if (!index || !d_out2) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_out2, 8)) return AIBX_ERR_ALIGN;
  hipStream_t st = as_stream(stream);
  zero_word_kernel<<<1, 1, 0, st>>>(d_out2, 2);
  index_count_kernel<<<pass_grid(index->n_slots), kIndexThreads, 0, st>>>(index->slots, index->n_slots, d_out2, true);
  return launch_status();
}

int aibx_index_rebuild(const aibx_index_t* src, aibx_index_t* dst, uint64_t* d_counters3, void* stream) {
  if (!src || !dst || src == dst || src->slots == dst->slots) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_counters3, 8)) return AIBX_ERR_ALIGN;
  const int rc = aibx_index_clear(dst, stream);
  if (rc != AIBX_OK) return rc;
  index_insert_kernel<<<pass_grid(src->n_slots), kIndexThreads, 0, as_stream(stream)>>>(
      table_of(dst), TableSource{src->slots, src->usage, (int64_t)src->n_slots}, d_counters3);
  return launch_status();
}

int aibx_index_dump(const aibx_index_t* index, uint64_t* d_keys_out, uint64_t* d_values_out,
                    uint64_t capacity, uint64_t* d_n_out, void* stream) {
  if (!index || !d_n_out) return AIBX_ERR_INVALID_ARG;
  if (capacity && (!d_keys_out || !d_values_out)) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_keys_out, 8) || !aligned(d_values_out, 8) || !aligned(d_n_out, 8)) return AIBX_ERR_ALIGN;
  hipStream_t st = as_stream(stream);
  zero_word_kernel<<<1, 1, 0, st>>>(d_n_out, 1);
  index_emit_kernel<<<pass_grid(index->n_slots), kIndexThreads, 0, st>>>(
      index->slots, index->usage, index->n_slots, EmitTest{false, 0, 0}, d_keys_out, d_values_out, capacity,
      d_n_out);
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
  const int lg_run = request_run_lg(n_req);
  const unsigned grid = workgroups_for_requests(n_req, lg_run);
  // Thousands of requests averaging at most 64 blocks: one wavefront per request and nothing else.
  // Otherwise four per request (those of a short request beyond the first leave at once); eight in a
  // batch of fewer than 4,096 requests, which leaves the GPU room and ends with its longest request
  // (1,024 lognormal requests of up to 2,048 blocks: 20.5 -> 17.2 us; sixteen are slower again).
  if (n_req >= 4096 && n_blocks_total <= (int64_t)n_req * kWave)
    prefix_match_kernel<1><<<grid, kWave, 0, as_stream(stream)>>>(table_of(index), d_hashes, d_blk_off,
                                                                   d_values_out, d_match_len, n_req, lg_run);
  else if (n_req < 4096)
    prefix_match_kernel<8><<<grid, 8 * kWave, 0, as_stream(stream)>>>(
        table_of(index), d_hashes, d_blk_off, d_values_out, d_match_len, n_req, lg_run);
  else
    prefix_match_kernel<kWavesPerGroup><<<grid, kIndexThreads, 0, as_stream(stream)>>>(
        table_of(index), d_hashes, d_blk_off, d_values_out, d_match_len, n_req, lg_run);
  return launch_status();
}

}  // extern "C"
