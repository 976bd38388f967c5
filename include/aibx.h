/*
 * aibx - GPU hot path of a distributed KV cache with prefix-aware routing (MI355X / gfx950).
 *
 * The paper (AIBrix, arXiv 2504.03648) describes a KV cache pool shared across inference
 * engines (Section 3.2.5, "Distributed KV Cache Pool") and a gateway policy that routes a
 * request to the instance holding a reusable prefix of its KV cache (Section 3.2.2, the
 * "prefix-cache-aware" policy). This library implements the data-parallel work behind both:
 *
 *   aibx_block_hash    chained per-block hashes of request token streams
 *   aibx_prefix_match  lookup of those hashes in a GPU-resident cache index + first-miss length
 *   aibx_hash_match    the two above in one launch
 *   aibx_route         per request: the pod with the longest cached prefix, if above a threshold
 *   aibx_hash_match_route  tokens in, pod out: the three above in one launch
 *   aibx_index_insert  metadata update: (key -> value) upsert           (Section 3.2.5)
 *   aibx_index_evict   metadata update: removal of evicted keys          (Section 3.2.5)
 *   aibx_index_touch / _age / _select_victims   scan-resistant victim selection (Section 3.2.5)
 *   aibx_index_rebuild compaction / resize of the index into a second table   (Section 3.2.5)
 *   aibx_kv_gather     paged KV pool -> contiguous staging (offload)     (Section 3.2.5)
 *   aibx_kv_scatter    contiguous staging -> paged KV pool (onload)      (Section 3.2.5)
 *   aibx_kv_gather_fill / _scatter_fill  the same for partly filled blocks (a sequence's last block)
 *   aibx_kv_gather_runs / _scatter_runs  the same with a layout conversion (token-major pools)
 *   aibx_kv_offload / aibx_kv_onload   paged KV pool <-> pinned host memory, one kernel each way
 *
 * The paper prints no hash function, index layout or copy layout; the rules stated below are
 * this library's own and are what its results are checked against.
 *
 * General conventions
 *   - Every pointer named d_* is DEVICE memory owned by the caller. The library allocates no
 *     device memory; the only allocation it makes is the small host handle of an index.
 *     Pointers without the d_ prefix (descriptors, out-parameters) are HOST memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Every call only
 *     enqueues work on that stream and returns; it never synchronises. Calls that touch the
 *     same index, pool pages or staging slots must be ordered by the caller (same stream, or
 *     events). Concurrent gather/scatter calls are safe iff their destination bytes are disjoint
 *     and no call reads what another writes.
 *   - Return value: AIBX_OK (0) or a negative aibx_status. Conditions only the device can see
 *     (table full, page id out of range, key absent) are counted in caller-provided device
 *     counters, not raised.
 *   - A count of zero (n = 0, n_req = 0) is a valid no-op and returns AIBX_OK.
 */
#ifndef AIBX_H_
#define AIBX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AIBX_OK = 0,
  AIBX_ERR_INVALID_ARG = -1, /* null pointer, negative count, value out of its stated range   */
  AIBX_ERR_ALIGN = -2,       /* a pointer, stride or size is not a multiple of what is stated */
  AIBX_ERR_UNSUPPORTED = -3, /* e.g. n_slots not a power of two, or below the minimum         */
  AIBX_ERR_HIP = -4          /* the HIP runtime refused a launch; see aibx_last_hip_error()   */
} aibx_status;

/* Value reported for a key that is not in the index. Never store it as a value. */
#define AIBX_NO_VALUE 0xFFFFFFFFFFFFFFFFull
/* The two key values the index reserves; aibx_block_hash never produces them. */
#define AIBX_KEY_EMPTY 0x0000000000000000ull
#define AIBX_KEY_TOMBSTONE 0xFFFFFFFFFFFFFFFFull

/* Library version (major*10000 + minor*100 + patch) and the version of the hash definition;
 * hashes are comparable only between equal hash versions. */
int aibx_version(void);
int aibx_hash_version(void);
/* Static, human-readable text for a status code. */
const char* aibx_strerror(int status);
/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char* aibx_last_hip_error(void);

/* ------------------------------------------------------------------------------------------
 * Chained per-block prefix hash.  (Token-pattern analysis for prefix-cache-aware routing,
 * Section 3.2.2; detection of overlapping token sequences across requests, Section 3.2.5.)
 *
 * Requests are concatenated: request r owns d_tokens[d_tok_off[r] .. d_tok_off[r+1]) and
 * d_hash_out[d_blk_off[r] .. d_blk_off[r+1]), where the caller has set
 * d_blk_off[r+1]-d_blk_off[r] = floor(len_r / block_size): only full blocks are hashed.
 * With all arithmetic on uint64 modulo 2^64 and
 *   K0=0x9E3779B97F4A7C15 K1=0x6A09E667F3BCC909 K2=0xBB67AE8584CAA73B K3=0x3C6EF372FE94F82B
 *   F(x): x^=x>>32; x*=K1; x^=x>>29; x*=K2; x^=x>>32
 *   term(t,i) = y ^ (y>>32),  y = (zero_extend(uint32(t)) ^ K0*(i+1)) * K1
 * block j of a request gets
 *   c_j = sum_{i<block_size} term(tok[j*block_size+i], i)
 *   s_j = K2*s_{j-1} + F(c_j),   s_{-1} = F(seed ^ K3)
 *   h_j = F(s_j ^ K3), except that 0 and 2^64-1 are replaced by h_j ^ K0.
 * h_j depends on `seed` and on the first (j+1)*block_size tokens of the request only, so two
 * requests share h_0..h_{k-1} exactly when they share their first k blocks of tokens (up to
 * 64-bit collisions). `seed` separates key spaces (model, adapter, tenant).
 *
 *   d_tokens   int32[d_tok_off[n_req]]   token ids (bit patterns; negative ids are allowed)
 *   d_tok_off  int64[n_req+1]            non-decreasing, d_tok_off[0] >= 0
 *   d_blk_off  int64[n_req+1]            d_blk_off[0] = 0, d_blk_off[n_req] = n_blocks_total
 *   block_size in [1, 1024]
 *   d_hash_out uint64[n_blocks_total]    written
 * The offsets are trusted (they are device data); n_blocks_total must equal d_blk_off[n_req].
 * Pointers must be aligned to their element size. Errors: INVALID_ARG, ALIGN, HIP.
 */
int aibx_block_hash(const int32_t* d_tokens, const int64_t* d_tok_off, const int64_t* d_blk_off,
                    int32_t n_req, int64_t n_blocks_total, int32_t block_size, uint64_t seed,
                    uint64_t* d_hash_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Cache index: a GPU-resident open-addressing table key -> value (the cache pool's metadata of
 * Section 3.2.5: which blocks are cached and where). Keys are any uint64 except the two
 * reserved values; values are any uint64 except AIBX_NO_VALUE. Observable behaviour is that of
 * a map with capacity n_slots; where a key sits in the table is not observable.
 * One bound applies to tables of more than 32,768 slots: a key is stored within the first 4,096
 * buckets (32,768 slots) of its probe sequence or not at all, so that a table with no free slot
 * left cannot make every absent key walk all of it. A key whose 4,096 buckets are all taken is
 * reported `full` although slots remain elsewhere; below a load factor of 0.99 the probability of
 * that is under 1e-18 per key.
 */
typedef struct aibx_index aibx_index_t; /* opaque host handle */

/* Bytes of device storage a table of n_slots needs (21 per slot: the 16-byte slot, a 4-byte
 * usage word and a tag byte). n_slots: power of two, 8 <= n_slots <= 2^36.
 * Errors: INVALID_ARG (null out), UNSUPPORTED. */
int aibx_index_storage_bytes(uint64_t n_slots, size_t* out_bytes);

/* Binds a handle to caller-owned storage (256-byte aligned, >= aibx_index_storage_bytes) and
 * enqueues a clear. The storage must outlive the handle. Errors: INVALID_ARG, ALIGN,
 * UNSUPPORTED, HIP. */
int aibx_index_create(void* d_storage, size_t bytes, uint64_t n_slots, void* stream,
                      aibx_index_t** out);
/* Frees the host handle only (never the device storage). NULL is accepted. */
int aibx_index_destroy(aibx_index_t* index);
/* Enqueues removal of every key. */
int aibx_index_clear(aibx_index_t* index, void* stream);

/* Batch upsert (the cache's metadata updates, Section 3.2.5). For each i < n: key absent -> stored with
 * d_values[i] (inserted); key present -> its value is overwritten (updated). A reserved key, or
 * a new key when no slot is free, is dropped (full). The same key may appear several times in one
 * batch if its values are identical: it then counts once as inserted (or updated) and the other
 * occurrences as updated; with differing values one of them wins.
 *   d_counters3 uint64[3], nullable: {inserted, updated, full} are ADDED to it.
 * Errors: INVALID_ARG, ALIGN (8-byte), HIP. */
int aibx_index_insert(aibx_index_t* index, const uint64_t* d_keys, const uint64_t* d_values,
                      int64_t n, uint64_t* d_counters3, void* stream);

/* Batch removal of evicted keys (Section 3.2.5 names eviction; choosing the victims is the
 * caller's policy). For each i < n: key present -> removed, d_values_out[i] = its value
 * (evicted); absent or reserved -> d_values_out[i] = AIBX_NO_VALUE (missing). If a key appears
 * several times in one batch exactly one occurrence reports the value.
 *   d_values_out uint64[n], nullable;  d_counters2 uint64[2], nullable: {evicted, missing} ADDED.
 * Errors: INVALID_ARG, ALIGN, HIP. */
int aibx_index_evict(aibx_index_t* index, const uint64_t* d_keys, int64_t n,
                     uint64_t* d_values_out, uint64_t* d_counters2, void* stream);

/* Usage tracking and victim selection.  (Section 3.2.5 asks for an eviction policy that a one-off
 * scan cannot disturb and that keeps the frequently reused KV; it names the policy without
 * describing it. This is the rule used here.)
 * Every indexed key carries a touch count and the last epoch it was touched in; a newly inserted
 * key has count 0 and epoch 0, an upsert of a present key keeps its usage, eviction discards it.
 *   aibx_index_touch: for each i < n, if d_keys[i] is present its count goes up by one (saturating
 *     at 255) and its last epoch becomes max(last, epoch); absent and reserved keys are ignored; a
 *     key named k times in a batch is touched k times. `epoch` is the caller's logical clock,
 *     0 <= epoch < 2^24. The caller reports the blocks a request actually reused.
 *   aibx_index_age: halves every count (call it once per ageing period).
 *   aibx_index_select_victims: writes, in no particular order, every live (key, value) with
 *     count < protect_count AND last < before_epoch, and their number to *d_n_out (the call
 *     resets it; pairs beyond `capacity` are counted but not written). With protect_count = 2 a
 *     block brought in by a one-off scan (touched at most once) goes as soon as it is older than
 *     before_epoch, while a block that was reused stays until ageing has worn its count down.
 *     The victims then go to aibx_kv_gather (offload) and aibx_index_evict.
 * Errors: INVALID_ARG (also epoch >= 2^24), ALIGN, HIP. */
int aibx_index_touch(aibx_index_t* index, const uint64_t* d_keys, int64_t n, uint32_t epoch,
                     void* stream);
int aibx_index_age(aibx_index_t* index, void* stream);
int aibx_index_select_victims(const aibx_index_t* index, uint32_t protect_count,
                              uint32_t before_epoch, uint64_t* d_keys_out, uint64_t* d_values_out,
                              uint64_t capacity, uint64_t* d_n_out, void* stream);

/* *d_live_out (device uint64) = number of keys in the index. */
int aibx_index_count(const aibx_index_t* index, uint64_t* d_live_out, void* stream);

/* d_out2 (device uint64[2]) = {number of keys, number of tombstones}. Tombstones are slots whose
 * key was evicted from a bucket with no free slot; they keep probe sequences intact, are reused by
 * later inserts, and lengthen lookups while they last. Their number is a property of this table's
 * history, not of its contents. */
int aibx_index_stats(const aibx_index_t* index, uint64_t* d_out2, void* stream);

/* Rebuild (the metadata side of the pool's lifecycle, Section 3.2.5): dst is cleared and receives
 * every (key, value) of src together with its usage word (touch count, last epoch); src is only
 * read. With equal capacities this is a compaction - dst has no tombstones and every key sits in
 * the first bucket of its probe sequence that had room; with different capacities it is a resize.
 * d_counters3 (nullable, device uint64[3]) accumulates {moved, 0, dropped}: keys are dropped only
 * when dst has fewer slots than src has keys (which ones is unspecified).
 *   src, dst: two handles over disjoint storage. dst answers lookups once the call has completed
 *   in stream order; the caller then swaps the handles and may destroy or reuse src.
 * Errors: INVALID_ARG (also src == dst), ALIGN, HIP. */
int aibx_index_rebuild(const aibx_index_t* src, aibx_index_t* dst, uint64_t* d_counters3,
                       void* stream);

/* Writes the live (key, value) pairs, in no particular order, to d_keys_out/d_values_out (each
 * uint64[capacity]) and the number of live keys to *d_n_out (device uint64; the caller zeroes
 * nothing - the call resets it). Pairs beyond `capacity` are counted but not written. */
int aibx_index_dump(const aibx_index_t* index, uint64_t* d_keys_out, uint64_t* d_values_out,
                    uint64_t capacity, uint64_t* d_n_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Prefix match.  (The test behind the prefix-cache-aware routing policy of Section 3.2.2 - how
 * much of a request's prefix is already cached; the caller compares match_len / n_r with its
 * threshold.)
 * For every block b: d_values_out[b] = value of d_hashes[b] in the index, or AIBX_NO_VALUE.
 * For every request r: d_match_len[r] = the smallest j with block d_blk_off[r]+j absent, or its
 * block count if none is absent ("first miss": a block found behind a missing one still reports
 * its value but does not extend the match).
 *   d_hashes uint64[n_blocks_total]; d_blk_off int64[n_req+1] as for aibx_block_hash;
 *   d_values_out uint64[n_blocks_total], nullable; d_match_len int32[n_req].
 * With d_values_out NULL only the match lengths are produced (all a routing decision needs), and
 * the kernel stops probing a request behind its first missing block.
 * Errors: INVALID_ARG, ALIGN, HIP. */
int aibx_prefix_match(const aibx_index_t* index, const uint64_t* d_hashes,
                      const int64_t* d_blk_off, int32_t n_req, int64_t n_blocks_total,
                      uint64_t* d_values_out, int32_t* d_match_len, void* stream);

/* Hash and match in one launch: the same results as aibx_block_hash followed by
 * aibx_prefix_match on its output (Section 3.2.2: the routing path hashes a request's tokens only
 * to look the blocks up), without the hashes travelling through memory between two launches.
 *   d_hash_out   uint64[n_blocks_total], nullable (required when block_size is not 16, 32 or 64:
 *                those sizes run as the two separate launches);
 *   d_values_out uint64[n_blocks_total], nullable; d_match_len int32[n_req];
 *   every other argument as in aibx_block_hash / aibx_prefix_match.
 * With d_hash_out and d_values_out both NULL the match lengths are the only output (tokens in,
 * lengths out: all a routing decision needs), and the kernel stops working on a request behind its
 * first missing block.
 * Errors: INVALID_ARG, ALIGN, UNSUPPORTED (block size outside {16,32,64} with d_hash_out NULL), HIP. */
int aibx_hash_match(const aibx_index_t* index, const int32_t* d_tokens, const int64_t* d_tok_off,
                    const int64_t* d_blk_off, int32_t n_req, int64_t n_blocks_total,
                    int32_t block_size, uint64_t seed, uint64_t* d_hash_out,
                    uint64_t* d_values_out, int32_t* d_match_len, void* stream);

/* ------------------------------------------------------------------------------------------
 * Prefix-cache-aware routing decision.  (Section 3.2.2: among the gateway's routing policies, the
 * one that prefers an instance already holding a reusable prefix of the request's KV cache when the
 * hit is large enough; below that threshold this library falls back to the least-request policy of
 * the same list.)
 * The index value of a block is read as the SET OF PODS holding it: bit p = pod p, p < n_pods <= 63
 * (AIBX_NO_VALUE = no pod; higher bits are ignored). d_pod_sets is the per-block output of
 * aibx_prefix_match / aibx_hash_match. For request r with n_r blocks and pod p,
 *   len_p = number of leading blocks of r whose set contains p,   best = max_p len_p.
 * If n_r > 0, best > 0 and best/n_r >= threshold_num/threshold_den (compared as integers,
 * best*den >= num*n_r), the candidates are the pods with len_p = best; otherwise every pod is a
 * candidate. The request goes to the candidate with the smallest d_pod_load (admitted requests),
 * ties to the smallest pod id: d_pod_out[r] = that pod, d_hit_len_out[r] = its len_p.
 * Loads are read once; requests of one batch do not see each other's assignment.
 *   d_pod_sets uint64[n_blocks_total]; d_blk_off int64[n_req+1]; d_pod_load int32[n_pods], >= 0;
 *   threshold_num, threshold_den < 2^32, den > 0; d_pod_out, d_hit_len_out int32[n_req].
 * Errors: INVALID_ARG, ALIGN, HIP. */
int aibx_route(const uint64_t* d_pod_sets, const int64_t* d_blk_off, int32_t n_req,
               int64_t n_blocks_total, int32_t n_pods, const int32_t* d_pod_load,
               uint64_t threshold_num, uint64_t threshold_den, int32_t* d_pod_out,
               int32_t* d_hit_len_out, void* stream);

/* The routing decision straight from the tokens, in one launch: aibx_block_hash, then the lookups of
 * aibx_prefix_match, then the decision of aibx_route on the values found, with no hash, value or
 * length array in between (what the gateway of Section 3.2.2 needs per batch of requests, where
 * three launches cost more than the work). Results are exactly those of the three calls in a row:
 * d_pod_out and d_hit_len_out as for aibx_route with d_pod_sets = the per-block index values.
 * Work on a request ends at the first block that no single pod holds together with all blocks
 * before it. Arguments as for aibx_hash_match and aibx_route.
 * Errors: INVALID_ARG, ALIGN, UNSUPPORTED (block size outside {16, 32, 64}), HIP. */
int aibx_hash_match_route(const aibx_index_t* index, const int32_t* d_tokens, const int64_t* d_tok_off,
                          const int64_t* d_blk_off, int32_t n_req, int64_t n_blocks_total,
                          int32_t block_size, uint64_t seed, int32_t n_pods, const int32_t* d_pod_load,
                          uint64_t threshold_num, uint64_t threshold_den, int32_t* d_pod_out,
                          int32_t* d_hit_len_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Paged-KV gather / scatter.  (Moving KV blocks between the engine's paged memory and the
 * cache's contiguous buffers: offload of blocks chosen to persist, onload of matched ones,
 * Section 3.2.5.)  Pure byte copies - no conversion of any kind.
 *
 * The pool is n_seg planes; segment s of page p is the seg_bytes bytes at
 *   base + s*seg_stride + p*page_stride.
 * (n_seg = 1: page-major pool; n_seg = 2*layers: one plane per layer and K/V; n_seg = layers:
 * latent-only pages.) A staging block holds the n_seg segments of one page back to back in
 * plane order; block q starts at d_staging + q*staging_block_stride.
 */
typedef struct {
  void* base;           /* DEVICE pointer, 16-byte aligned                           */
  int32_t n_seg;        /* >= 1                                                      */
  uint64_t seg_stride;  /* bytes between planes; multiple of 16                      */
  uint64_t page_stride; /* bytes between pages of one plane; multiple of 16, >= seg_bytes */
  uint64_t seg_bytes;   /* contiguous bytes per (plane, page); multiple of 16, > 0   */
  int64_t n_pages;      /* >= 0                                                      */
} aibx_pool_desc;

/* Gather: for i < n, page p = d_page_ids[i], slot q = d_slot_ids ? d_slot_ids[i] : i:
 *   staging block q <- page p.            Scatter: page p <- staging block q.
 * p < 0 marks a hole: the entry is skipped. p >= n_pages: the entry is skipped and
 * *d_bad_page_counter (device uint64, nullable) is incremented. Slot ids are trusted: the
 * caller guarantees 0 <= q and (q+1)*staging_block_stride <= size of the staging buffer.
 * Entries of one call must not share a destination (slot in gather, page in scatter).
 *   pool (host struct, read during the call); d_page_ids int32[n]; d_slot_ids int32[n] or NULL;
 *   d_staging 16-byte aligned; staging_block_stride multiple of 16, >= n_seg*seg_bytes.
 * Errors: INVALID_ARG, ALIGN, HIP. */
int aibx_kv_gather(const aibx_pool_desc* pool, const int32_t* d_page_ids,
                   const int32_t* d_slot_ids, int64_t n, void* d_staging,
                   uint64_t staging_block_stride, uint64_t* d_bad_page_counter, void* stream);
int aibx_kv_scatter(const aibx_pool_desc* pool, const int32_t* d_page_ids,
                    const int32_t* d_slot_ids, int64_t n, const void* d_staging,
                    uint64_t staging_block_stride, uint64_t* d_bad_page_counter, void* stream);

/* The same copies for partly filled blocks. (The last block of a sequence whose length is not a
 * multiple of the block size: a conversation's KV ends wherever its last turn ended, and offloading,
 * migrating or re-loading it, Section 3.2.5, has to move that block's tokens too.) In every layout
 * served here the tokens a block holds come first in each of its segments, so entry i moves only the
 * first d_seg_fill[i] bytes of each segment and leaves the rest of the segment alone on both sides.
 * The count is clamped to [0, seg_bytes] and rounded down to a multiple of 16; d_seg_fill = NULL
 * moves whole segments (the calls above). Everything else - holes, out-of-range pages, slots,
 * strides, errors - is as for aibx_kv_gather / aibx_kv_scatter.
 *   d_seg_fill int32[n] (device), or NULL. */
int aibx_kv_gather_fill(const aibx_pool_desc* pool, const int32_t* d_page_ids,
                        const int32_t* d_slot_ids, const int32_t* d_seg_fill, int64_t n, void* d_staging,
                        uint64_t staging_block_stride, uint64_t* d_bad_page_counter, void* stream);
int aibx_kv_scatter_fill(const aibx_pool_desc* pool, const int32_t* d_page_ids,
                         const int32_t* d_slot_ids, const int32_t* d_seg_fill, int64_t n,
                         const void* d_staging, uint64_t staging_block_stride,
                         uint64_t* d_bad_page_counter, void* stream);

/* How aibx_kv_gather / aibx_kv_scatter split a call of n entries into kernel launches (host
 * arithmetic only; nothing is launched and no device is needed). One workgroup of 256 lanes moves
 * 4 KiB, and one launch may hold at most 2^32 - 1 threads, so a call that moves 64 GiB or more
 * (e.g. offloading half of a 160 GiB pool, Section 3.2.5) takes more than one launch; entries are
 * never split between launches. Launch k < capacity is written as (first_entry_out[k],
 * n_entries_out[k], workgroups_out[k]); only pool->n_seg and pool->seg_bytes are read.
 * Returns the number of launches (>= 0; it may exceed capacity), or INVALID_ARG / UNSUPPORTED (a
 * single block that exceeds one launch). All pointers are HOST memory (nullable if capacity = 0). */
int aibx_kv_copy_launches(const aibx_pool_desc* pool, int64_t n, int64_t* first_entry_out,
                          int64_t* n_entries_out, uint32_t* workgroups_out, int32_t capacity);

/* ------------------------------------------------------------------------------------------
 * The same copies for a pool whose segments are not contiguous (cross-engine reuse of KV,
 * Section 3.2.5, between engines that lay their pages out differently). Segment s of page p is
 * n_run runs of run_bytes; run t starts at base + p*page_stride + s*seg_stride + t*run_stride.
 * A token-major pool [page][token][layer...] is the case run = one token's bytes of one layer:
 * n_run = tokens per page, seg_stride = run_bytes, run_stride = n_seg*run_bytes, page_stride =
 * n_run*n_seg*run_bytes. The staging block is as above - segment after segment, each segment's
 * runs back to back (n_seg*n_run*run_bytes bytes) - so the copy converts between the two layouts.
 * Everything else (holes, out-of-range pages, slot ids, strides, errors) is as for
 * aibx_kv_gather / aibx_kv_scatter.
 *   base 16-byte aligned; run_bytes, seg_stride, run_stride, page_stride multiples of 16, > 0
 *   where used; n_run*run_bytes < 2^31. Runs of one page must not overlap (not checked).
 * Errors: INVALID_ARG, ALIGN, UNSUPPORTED, HIP. */
typedef struct {
  void* base;           /* DEVICE pointer                         */
  int32_t n_seg;        /* >= 1                                   */
  int32_t n_run;        /* >= 1: runs per segment                 */
  uint64_t seg_stride;  /* bytes between segments of one page     */
  uint64_t page_stride; /* bytes between pages                    */
  uint64_t run_stride;  /* bytes between runs of one segment      */
  uint64_t run_bytes;   /* contiguous bytes per run               */
  int64_t n_pages;      /* >= 0                                   */
} aibx_pool_runs_desc;

int aibx_kv_gather_runs(const aibx_pool_runs_desc* pool, const int32_t* d_page_ids,
                        const int32_t* d_slot_ids, int64_t n, void* d_staging,
                        uint64_t staging_block_stride, uint64_t* d_bad_page_counter, void* stream);
int aibx_kv_scatter_runs(const aibx_pool_runs_desc* pool, const int32_t* d_page_ids,
                         const int32_t* d_slot_ids, int64_t n, const void* d_staging,
                         uint64_t staging_block_stride, uint64_t* d_bad_page_counter, void* stream);

/* ------------------------------------------------------------------------------------------
 * Host-tier leg: paged pool <-> pinned host memory, moved by one kernel that addresses the host
 * buffer directly. (Section 3.2.5: the cache pool is DRAM-based and exchanges KV with the
 * colocated engine through host memory.)
 *   Entry i < n moves page p = d_page_ids[i] <-> host block i at h_buf + i*host_block_stride (the
 *   n_seg segments back to back, as in a staging block). aibx_kv_offload: host block i <- page p;
 *   aibx_kv_onload: page p <- host block i. p < 0 marks a hole and p >= n_pages is counted in
 *   *d_bad_page_counter (device uint64, nullable), as in aibx_kv_gather/_scatter; either way the
 *   entry is skipped and neither its host block nor any page is touched. Entries of one onload
 *   call must not share a page. Bytes between host blocks (stride > block) are never written.
 *   h_dst / h_src: HOST memory that is pinned and mapped for the GPU (hipHostMalloc, or what a
 *   framework allocates through it), 16-byte aligned, at least (n-1)*host_block_stride +
 *   n_seg*seg_bytes bytes inside one allocation; host_block_stride multiple of 16, >=
 *   n_seg*seg_bytes. Pageable memory, device memory and buffers that are too short are refused
 *   with INVALID_ARG before anything is launched.
 * The call only enqueues one launch on `stream`, with a small fixed grid sized for the host link,
 * so kernels on other streams keep running beside it. The host buffer holds the data (offload) or
 * may be reused (onload) once `stream` has drained past the call.
 * Errors: INVALID_ARG, ALIGN, UNSUPPORTED (a block of 2^31 or more 4 KiB pieces), HIP. */
int aibx_kv_offload(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, void* h_dst,
                    uint64_t host_block_stride, uint64_t* d_bad_page_counter, void* stream);
int aibx_kv_onload(const aibx_pool_desc* pool, const int32_t* d_page_ids, int64_t n, const void* h_src,
                   uint64_t host_block_stride, uint64_t* d_bad_page_counter, void* stream);

/* ------------------------------------------------------------------------------------------
 * Measurement aid (not a step of the path; for benchmarks that want to place the lookup rates of
 * aibx_prefix_match beside what independent random reads reach on a table of the same size).
 * Lane i of the launch reads the first read_bytes bytes of a pseudo-random line_bytes-sized line
 * of d_table, n_reads reads in all. Nothing is computed from what is read: *d_sink is written
 * only if the XOR of a lane's reads happens to equal one fixed 64-bit constant.
 *   d_table 128-byte aligned, table_bytes a power of two >= line_bytes; line_bytes a power of two
 *   in [8, 4096]; read_bytes in {8, 16, 64, 128}, <= line_bytes; d_sink device uint64.
 * Errors: INVALID_ARG, ALIGN, HIP. */
int aibx_calib_random_reads(const void* d_table, uint64_t table_bytes, uint32_t line_bytes,
                            uint32_t read_bytes, int64_t n_reads, uint64_t seed, uint64_t* d_sink,
                            void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AIBX_H_ */
