// CPU oracle for the KV-cache hot path: chained per-block prefix hashing, prefix match
// against a cache index, index insert/evict, and paged-KV gather/scatter.
//
// THIS IS TEST INFRASTRUCTURE. It is the plain, slow, single-threaded statement of what the
// GPU library must compute. Only the tests, the smoke check and the benchmark's CPU-baseline
// leg may call it; the product library never links, loads or falls back to it, and it shares
// no code, header, table or constant generator with the HIP sources.
//
// What the paper fixes and what it leaves open: the paper (Section 3.2.5, "Distributed KV
// Cache Pool", and the prefix-cache-aware policy in the routing list of Section 3.2.2) states
// the problem - overlapping token prefixes across requests, reuse of their KV blocks across
// engines, eviction, metadata updates, data movement between the engine and the cache - but
// prints no hash function, no index structure and no copy layout. Every concrete rule below is
// therefore a reading chosen for this implementation; each is marked "reading:".
//
// All functions take host pointers. Integers wrap modulo 2^64 where stated.

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <utility>
#include <vector>

namespace {

typedef uint64_t u64;

// reading: four 64-bit odd constants taken from the fractional parts of the golden ratio and
// of sqrt(2), sqrt(3), sqrt(5) ("nothing up my sleeve" numbers).
const u64 kPhi   = 0x9E3779B97F4A7C15ull;
const u64 kSqrt2 = 0x6A09E667F3BCC909ull;
const u64 kSqrt3 = 0xBB67AE8584CAA73Bull;
const u64 kSqrt5 = 0x3C6EF372FE94F82Bull;

const u64 kEmptyKey = 0ull;            // reserved: never a valid index key
const u64 kTombKey  = ~0ull;           // reserved: never a valid index key
const u64 kNoValue  = ~0ull;           // "not in the index"

// 64-bit finaliser: xor-shift, multiply, xor-shift, multiply, xor-shift. A bijection on u64.
u64 finalise(u64 x) {
  x ^= x >> 32;
  x *= kSqrt2;
  x ^= x >> 29;
  x *= kSqrt3;
  x ^= x >> 32;
  return x;
}

// Contribution of one token at position i (0-based) inside its block.
// reading: the token id is the int32 bit pattern, zero-extended to 64 bits.
u64 token_term(int32_t token, int64_t i) {
  u64 t = (u64)(uint32_t)token;
  u64 x = (t ^ (kPhi * (u64)(i + 1))) * kSqrt2;
  return x ^ (x >> 32);
}

// Keeps the two reserved key values out of the hash range.
u64 avoid_reserved(u64 h) {
  return (h == kEmptyKey || h == kTombKey) ? (h ^ kPhi) : h;
}

struct Usage {
  uint32_t count;   // touches since insertion (saturating at 255), halved by ageing
  uint32_t last;    // largest epoch the key was touched in (0 = never)
};

struct Index {
  u64 capacity;
  std::unordered_map<u64, u64> map;      // abstract key -> value map; no slots, no probing
  std::unordered_map<u64, Usage> usage;  // same keys as `map`
};

}  // namespace

extern "C" {

// The hash's three building blocks, exported so that tests can pin each on its own.
u64 orc_finalise(u64 x) { return finalise(x); }
u64 orc_token_term(int32_t token, int64_t i) { return token_term(token, i); }
u64 orc_avoid_reserved(u64 h) { return avoid_reserved(h); }

// ---------------------------------------------------------------------------------------------
// Per-block chained prefix hash (the "token pattern" analysis behind prefix-cache-aware routing,
// Section 3.2.2, and the prefix reuse of Section 3.2.5).
//
// Request r owns tokens[tok_off[r] .. tok_off[r+1]) and hash_out[blk_off[r] .. blk_off[r+1]).
// reading: only full blocks are hashed, n_r = floor(len_r / B); a tail shorter than B has no hash.
// For block j of a request:
//   content  c_j = sum over i < B of token_term(tok[j*B + i], i)          (mod 2^64)
//   digest   d_j = finalise(c_j)
//   chain    s_j = kSqrt3 * s_{j-1} + d_j,   s_{-1} = finalise(seed ^ kSqrt5)
//   output   h_j = avoid_reserved(finalise(s_j ^ kSqrt5))
// so h_j depends on the seed and on tokens [0, (j+1)*B) of the request only.
// Returns 0, or -1 on invalid arguments.
int orc_block_hash(const int32_t* tokens, const int64_t* tok_off, const int64_t* blk_off,
                   int32_t n_req, int64_t n_blocks_total, int32_t block_size, u64 seed,
                   u64* hash_out) {
  if (n_req < 0 || n_blocks_total < 0 || block_size < 1 || block_size > 1024) return -1;
  if (n_req == 0) return 0;
  if (!tok_off || !blk_off) return -1;
  if (blk_off[n_req] != n_blocks_total) return -1;
  for (int32_t r = 0; r < n_req; ++r) {
    const int64_t len = tok_off[r + 1] - tok_off[r];
    const int64_t n_r = len / block_size;
    if (blk_off[r + 1] - blk_off[r] != n_r) return -1;
    const int32_t* tok = tokens + tok_off[r];
    u64* out = hash_out + blk_off[r];
    u64 s = finalise(seed ^ kSqrt5);
    for (int64_t j = 0; j < n_r; ++j) {
      u64 c = 0;
      for (int64_t i = 0; i < block_size; ++i) c += token_term(tok[j * block_size + i], i);
      s = kSqrt3 * s + finalise(c);
      out[j] = avoid_reserved(finalise(s ^ kSqrt5));
    }
  }
  return 0;
}

// ---------------------------------------------------------------------------------------------
// Cache index (the metadata of the KV cache pool, Section 3.2.5: which blocks are cached, where;
// updated on insert, removed on eviction). Modelled as an abstract map with a capacity, so that
// nothing observable depends on how a table lays out or probes its slots.

void* orc_index_create(u64 n_slots) {
  Index* ix = new Index();
  ix->capacity = n_slots;
  return ix;
}

void orc_index_destroy(void* h) { delete static_cast<Index*>(h); }

void orc_index_clear(void* h) {
  static_cast<Index*>(h)->map.clear();
  static_cast<Index*>(h)->usage.clear();
}

// Batch upsert, applied in array order. counters3 accumulates {inserted, updated, full}.
// reading: absent key -> added (inserted); present key -> value overwritten (updated);
// a reserved key (0 or 2^64-1) or a new key when the map already holds `capacity` keys is
// dropped (full).
int orc_index_insert(void* h, const u64* keys, const u64* values, int64_t n, u64* counters3) {
  if (!h || n < 0) return -1;
  Index* ix = static_cast<Index*>(h);
  u64 inserted = 0, updated = 0, full = 0;
  for (int64_t i = 0; i < n; ++i) {
    const u64 k = keys[i];
    if (k == kEmptyKey || k == kTombKey) { ++full; continue; }
    auto it = ix->map.find(k);
    if (it != ix->map.end()) { it->second = values[i]; ++updated; continue; }
    if (ix->map.size() >= ix->capacity) { ++full; continue; }
    ix->map.emplace(k, values[i]);
    ix->usage[k] = Usage{0, 0};          // a new key starts untouched
    ++inserted;
  }
  if (counters3) { counters3[0] += inserted; counters3[1] += updated; counters3[2] += full; }
  return 0;
}

// Batch removal, applied in array order. values_out (nullable) receives the removed value or
// kNoValue. counters2 accumulates {evicted, missing}.
int orc_index_evict(void* h, const u64* keys, int64_t n, u64* values_out, u64* counters2) {
  if (!h || n < 0) return -1;
  Index* ix = static_cast<Index*>(h);
  u64 evicted = 0, missing = 0;
  for (int64_t i = 0; i < n; ++i) {
    u64 v = kNoValue;
    auto it = ix->map.find(keys[i]);
    if (it != ix->map.end()) { v = it->second; ix->map.erase(it); ix->usage.erase(keys[i]); ++evicted; }
    else ++missing;
    if (values_out) values_out[i] = v;
  }
  if (counters2) { counters2[0] += evicted; counters2[1] += missing; }
  return 0;
}

// ---------------------------------------------------------------------------------------------
// Usage tracking and victim selection (Section 3.2.5 names a "scan-resistant eviction policy" that
// keeps hot KV and does not describe it).
// reading: every indexed key carries a touch count and the last epoch it was touched in. A touch
// (the caller reports the blocks a request actually reused, with its logical clock `epoch`) adds
// one to the count, saturating at 255, and raises `last` to `epoch`; absent keys are ignored; a key
// named several times in one batch is touched that many times. Ageing halves every count.
// Victims are the keys with count < protect_count AND last < before_epoch: a block brought in by a
// one-off scan has been touched at most once and goes as soon as it is old, while a block that
// was reused keeps a count >= 2 until ageing wears it down. Upserting a present key keeps its usage.
int orc_index_touch(void* h, const u64* keys, int64_t n, uint32_t epoch) {
  if (!h || n < 0 || epoch > 0xFFFFFFu) return -1;
  Index* ix = static_cast<Index*>(h);
  for (int64_t i = 0; i < n; ++i) {
    auto it = ix->usage.find(keys[i]);
    if (it == ix->usage.end()) continue;
    if (it->second.count < 255) ++it->second.count;
    it->second.last = std::max(it->second.last, epoch);
  }
  return 0;
}

void orc_index_age(void* h) {
  for (auto& kv : static_cast<Index*>(h)->usage) kv.second.count >>= 1;
}

// Victims in ascending key order; returns their number (which may exceed `capacity`).
u64 orc_index_select_victims(const void* h, uint32_t protect_count, uint32_t before_epoch, u64* keys_out,
                             u64* values_out, u64 capacity) {
  const Index* ix = static_cast<const Index*>(h);
  std::vector<std::pair<u64, u64>> out;
  for (const auto& kv : ix->usage)
    if (kv.second.count < protect_count && kv.second.last < before_epoch)
      out.emplace_back(kv.first, ix->map.at(kv.first));
  std::sort(out.begin(), out.end());
  const u64 m = std::min<u64>(capacity, out.size());
  for (u64 i = 0; i < m; ++i) { keys_out[i] = out[i].first; values_out[i] = out[i].second; }
  return out.size();
}

u64 orc_index_count(const void* h) { return static_cast<const Index*>(h)->map.size(); }

// Rebuild into a second index (compaction or resize of the pool's metadata, Section 3.2.5).
// reading: dst is emptied and then holds exactly src's keys with their values and usage; src is
// unchanged. Only when dst's capacity is below src's key count are keys left out - `capacity` of
// them move, the others are dropped, and which ones is not specified (here: ascending key order).
// counters3 accumulates {moved, 0, dropped}.
int orc_index_rebuild(const void* src_h, void* dst_h, u64* counters3) {
  if (!src_h || !dst_h || src_h == dst_h) return -1;
  const Index* src = static_cast<const Index*>(src_h);
  Index* dst = static_cast<Index*>(dst_h);
  dst->map.clear();
  dst->usage.clear();
  std::vector<u64> keys;
  for (const auto& kv : src->map) keys.push_back(kv.first);
  std::sort(keys.begin(), keys.end());
  u64 moved = 0, dropped = 0;
  for (u64 k : keys) {
    if (dst->map.size() >= dst->capacity) { ++dropped; continue; }
    dst->map.emplace(k, src->map.at(k));
    dst->usage[k] = src->usage.at(k);
    ++moved;
  }
  if (counters3) { counters3[0] += moved; counters3[2] += dropped; }
  return 0;
}

// Writes up to `capacity` (key, value) pairs in ascending key order; returns the number of live
// keys (which may exceed `capacity`).
u64 orc_index_dump(const void* h, u64* keys_out, u64* values_out, u64 capacity) {
  const Index* ix = static_cast<const Index*>(h);
  std::vector<std::pair<u64, u64>> kv(ix->map.begin(), ix->map.end());
  std::sort(kv.begin(), kv.end());
  const u64 m = std::min<u64>(capacity, kv.size());
  for (u64 i = 0; i < m; ++i) { keys_out[i] = kv[i].first; values_out[i] = kv[i].second; }
  return kv.size();
}

// ---------------------------------------------------------------------------------------------
// Prefix match (the "reusable prefix cache ... cache hit" of the prefix-cache-aware policy,
// Section 3.2.2). For every block the raw lookup result; for every request the number of
// leading blocks present.
// reading: first miss - match_len[r] = smallest j with hash[blk_off[r] + j] absent, or n_r if
// all are present. A block found after the first miss still reports its value but does not
// extend the match, because an onload needs every block 0 .. match_len-1.
int orc_prefix_match(const void* h, const u64* hashes, const int64_t* blk_off, int32_t n_req,
                     int64_t n_blocks_total, u64* values_out, int32_t* match_len) {
  if (!h || n_req < 0 || n_blocks_total < 0) return -1;
  const Index* ix = static_cast<const Index*>(h);
  for (int32_t r = 0; r < n_req; ++r) {
    const int64_t b0 = blk_off[r], n_r = blk_off[r + 1] - blk_off[r];
    int64_t first_miss = n_r;
    for (int64_t j = 0; j < n_r; ++j) {
      auto it = ix->map.find(hashes[b0 + j]);
      const u64 v = (it == ix->map.end()) ? kNoValue : it->second;
      if (values_out) values_out[b0 + j] = v;
      if (v == kNoValue && j < first_miss) first_miss = j;
    }
    match_len[r] = (int32_t)first_miss;
  }
  return 0;
}

// ---------------------------------------------------------------------------------------------
// Prefix-cache-aware routing decision (Section 3.2.2: route to an instance with a reusable prefix
// cache if the hit exceeds a threshold).
// reading: a block's index value is the set of pods holding it (bit p = pod p, p < n_pods <= 63;
// kNoValue = none). For request r and pod p, len_p = number of leading blocks whose set contains p.
// reading: best = max_p len_p; if n_r > 0, best > 0 and best*den >= num*n_r the candidates are the
// pods with len_p == best, otherwise (fallback: the least-request policy of the same list) every
// pod; among the candidates the smallest load wins, ties to the smallest pod id.
int orc_route(const u64* pod_sets, const int64_t* blk_off, int32_t n_req, int32_t n_pods,
              const int32_t* pod_load, u64 thr_num, u64 thr_den, int32_t* pod_out, int32_t* hit_len_out) {
  if (n_req < 0 || n_pods < 1 || n_pods > 63 || thr_den == 0) return -1;
  std::vector<int64_t> len(n_pods);
  for (int32_t r = 0; r < n_req; ++r) {
    const int64_t b0 = blk_off[r], n_r = blk_off[r + 1] - blk_off[r];
    int64_t best = 0;
    for (int32_t p = 0; p < n_pods; ++p) {
      int64_t j = 0;
      while (j < n_r && pod_sets[b0 + j] != kNoValue && ((pod_sets[b0 + j] >> p) & 1ull)) ++j;
      len[p] = j;
      best = std::max(best, j);
    }
    const bool aware = n_r > 0 && best > 0 && (u64)best * thr_den >= thr_num * (u64)n_r;
    int32_t chosen = -1;
    for (int32_t p = 0; p < n_pods; ++p) {
      if (aware && len[p] != best) continue;
      if (chosen < 0 || pod_load[p] < pod_load[chosen]) chosen = p;
    }
    pod_out[r] = chosen;
    hit_len_out[r] = (int32_t)len[chosen];
  }
  return 0;
}

// ---------------------------------------------------------------------------------------------
// Paged-KV gather / scatter (moving KV blocks between the engine's paged memory and the cache's
// contiguous buffers, Section 3.2.5). Pure byte copies.
//
// The pool is n_seg planes; segment s of page p is the seg_bytes bytes at
// base + s*seg_stride + p*page_stride. reading: a staging block is the n_seg segments of one
// page back to back in plane order, block q at staging + q*staging_block_stride.
// Entry i moves page page_id[i] <-> staging block (slot_id ? slot_id[i] : i).
// reading: page_id < 0 marks a hole and is skipped; page_id >= n_pages is skipped and counted
// in *bad_page (nullable).

struct orc_pool_desc {
  void* base;
  int32_t n_seg;
  u64 seg_stride;
  u64 page_stride;
  u64 seg_bytes;
  int64_t n_pages;
};

// Partly filled blocks (the last block of a sequence whose length is not a multiple of the block
// size; a conversation's KV ends wherever its last turn ended, Section 3.2.5): with seg_fill given,
// entry i moves only the first seg_fill[i] bytes of each of its segments - the bytes of the tokens
// the block holds, which come first in every segment - and leaves the rest of the segment alone on
// both sides. reading: the count is clamped to [0, seg_bytes] and rounded down to a multiple of 16
// (the unit every layout here is a multiple of); seg_fill == nullptr means whole segments.
static int copy_pages(const orc_pool_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                      const int32_t* seg_fill, int64_t n, unsigned char* staging, u64 stride, u64* bad_page,
                      bool to_staging) {
  if (!pool || n < 0 || pool->n_seg < 1) return -1;
  if (stride < (u64)pool->n_seg * pool->seg_bytes) return -1;
  unsigned char* base = static_cast<unsigned char*>(pool->base);
  for (int64_t i = 0; i < n; ++i) {
    const int64_t p = page_id[i];
    const int64_t q = slot_id ? (int64_t)slot_id[i] : i;
    if (p < 0) continue;
    if (p >= pool->n_pages) { if (bad_page) ++*bad_page; continue; }
    u64 moved = pool->seg_bytes;
    if (seg_fill) {
      const int64_t f = seg_fill[i];
      moved = f <= 0 ? 0 : ((u64)f < pool->seg_bytes ? (u64)f : pool->seg_bytes);
      moved -= moved % 16;
    }
    for (int32_t s = 0; s < pool->n_seg; ++s) {
      unsigned char* in_pool = base + (u64)s * pool->seg_stride + (u64)p * pool->page_stride;
      unsigned char* in_stage = staging + (u64)q * stride + (u64)s * pool->seg_bytes;
      if (to_staging) std::memcpy(in_stage, in_pool, moved);
      else            std::memcpy(in_pool, in_stage, moved);
    }
  }
  return 0;
}

int orc_kv_gather(const orc_pool_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                  int64_t n, void* staging, u64 staging_block_stride, u64* bad_page) {
  return copy_pages(pool, page_id, slot_id, nullptr, n, static_cast<unsigned char*>(staging),
                    staging_block_stride, bad_page, true);
}

int orc_kv_scatter(const orc_pool_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                   int64_t n, const void* staging, u64 staging_block_stride, u64* bad_page) {
  return copy_pages(pool, page_id, slot_id, nullptr, n,
                    const_cast<unsigned char*>(static_cast<const unsigned char*>(staging)),
                    staging_block_stride, bad_page, false);
}

int orc_kv_gather_fill(const orc_pool_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                       const int32_t* seg_fill, int64_t n, void* staging, u64 staging_block_stride,
                       u64* bad_page) {
  return copy_pages(pool, page_id, slot_id, seg_fill, n, static_cast<unsigned char*>(staging),
                    staging_block_stride, bad_page, true);
}

int orc_kv_scatter_fill(const orc_pool_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                        const int32_t* seg_fill, int64_t n, const void* staging, u64 staging_block_stride,
                        u64* bad_page) {
  return copy_pages(pool, page_id, slot_id, seg_fill, n,
                    const_cast<unsigned char*>(static_cast<const unsigned char*>(staging)),
                    staging_block_stride, bad_page, false);
}

// ---------------------------------------------------------------------------------------------
// The same copies for a pool whose segments are not contiguous: segment s of page p is n_run runs
// of run_bytes, run t at base + p*page_stride + s*seg_stride + t*run_stride. A token-major pool
// ([page][token][layer]...) is the case run = one token's bytes of one layer, run_stride = one
// token's bytes of all layers. The staging block is unchanged: segment after segment, each
// segment's runs back to back - i.e. the copy converts between the two layouts (cross-engine
// reuse of KV, Section 3.2.5, when the engines lay their pages out differently).
// reading: holes and out-of-range pages as above.
struct orc_pool_runs_desc {
  void* base;
  int32_t n_seg;
  int32_t n_run;
  u64 seg_stride;
  u64 page_stride;
  u64 run_stride;
  u64 run_bytes;
  int64_t n_pages;
};

static int copy_runs(const orc_pool_runs_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                     int64_t n, unsigned char* staging, u64 stride, u64* bad_page, bool to_staging) {
  if (!pool || n < 0 || pool->n_seg < 1 || pool->n_run < 1) return -1;
  const u64 seg_bytes = (u64)pool->n_run * pool->run_bytes;
  if (stride < (u64)pool->n_seg * seg_bytes) return -1;
  unsigned char* base = static_cast<unsigned char*>(pool->base);
  for (int64_t i = 0; i < n; ++i) {
    const int64_t p = page_id[i];
    const int64_t q = slot_id ? (int64_t)slot_id[i] : i;
    if (p < 0) continue;
    if (p >= pool->n_pages) { if (bad_page) ++*bad_page; continue; }
    for (int32_t s = 0; s < pool->n_seg; ++s)
      for (int32_t t = 0; t < pool->n_run; ++t) {
        unsigned char* in_pool = base + (u64)p * pool->page_stride + (u64)s * pool->seg_stride +
                                 (u64)t * pool->run_stride;
        unsigned char* in_stage = staging + (u64)q * stride + (u64)s * seg_bytes + (u64)t * pool->run_bytes;
        if (to_staging) std::memcpy(in_stage, in_pool, pool->run_bytes);
        else            std::memcpy(in_pool, in_stage, pool->run_bytes);
      }
  }
  return 0;
}

int orc_kv_gather_runs(const orc_pool_runs_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                       int64_t n, void* staging, u64 staging_block_stride, u64* bad_page) {
  return copy_runs(pool, page_id, slot_id, n, static_cast<unsigned char*>(staging), staging_block_stride,
                   bad_page, true);
}

int orc_kv_scatter_runs(const orc_pool_runs_desc* pool, const int32_t* page_id, const int32_t* slot_id,
                        int64_t n, const void* staging, u64 staging_block_stride, u64* bad_page) {
  return copy_runs(pool, page_id, slot_id, n,
                   const_cast<unsigned char*>(static_cast<const unsigned char*>(staging)),
                   staging_block_stride, bad_page, false);
}

}  // extern "C"
