// Chained per-block prefix hash (the token-pattern analysis behind the paper's prefix-cache-aware
// routing, Section 3.2.2, and its cross-request KV reuse, Section 3.2.5). The definition is in
// aibx.h; this file evaluates it on the GPU.
//
// Layout of the work: one workgroup per request; the request is hashed by one wavefront or by
// four together, depending on its length and on the shape of the batch (see launch_hash). A
// wavefront takes 1024 consecutive tokens at a time (64 coalesced tokens per load, 16 loads in
// flight), so a lane always sees the same position-in-block and folds its position constant once
// (request starts are only 4-byte aligned, so wider loads would need peeling); as many such
// sub-steps as give 64 blocks make a tile. The per-block sums
// are formed by a transposing butterfly across the lanes that share a block (DPP lane patterns
// inside a row of 16 lanes, bpermute only across rows), the block digests are scanned with the
// chain's affine step (s -> K2*s + d) by DPP row shifts inside each row and a 4-step scalar chain
// across rows, and the carry between tiles of one request goes through LDS.
#include "index_device.h"

namespace aibx {
namespace {

constexpr u64 K0 = 0x9E3779B97F4A7C15ull;
constexpr u64 K1 = 0x6A09E667F3BCC909ull;
constexpr u64 K2 = 0xBB67AE8584CAA73Bull;
constexpr u64 K3 = 0x3C6EF372FE94F82Bull;

constexpr int kGeneralWaves = 4;  // wavefronts per request on the general path

__host__ __device__ constexpr u64 ipow(u64 base, u64 e) {
  u64 r = 1;
  while (e) {
    if (e & 1) r *= base;
    base *= base;
    e >>= 1;
  }
  return r;
}

// K2^(i+1) for i < 64: the weight of the chain state entering a lane's row (or tile) at the lane's
// block. Read from constant memory: forming the power with multiplies cost every wavefront about
// a fifth of a tile's arithmetic before its first token.
struct ChainPowers {
  u64 v[kWave];
  constexpr ChainPowers() : v() {
    for (int i = 0; i < kWave; ++i) v[i] = ipow(0xBB67AE8584CAA73Bull, (u64)i + 1);
  }
};
__constant__ const ChainPowers kChainPowers{};

__device__ __forceinline__ u64 fin(u64 x) {
  x ^= x >> 32;
  x *= K1;
  x ^= x >> 29;
  x *= K2;
  x ^= x >> 32;
  return x;
}

__device__ __forceinline__ u64 out_hash(u64 s) {
  u64 h = fin(s ^ K3);
  return (h == 0ull || h == ~0ull) ? (h ^ K0) : h;
}

__device__ __forceinline__ u64 shfl_xor64(u64 v, int mask) {
  u32 lo = (u32)v, hi = (u32)(v >> 32);
  lo = __shfl_xor(lo, mask);
  hi = __shfl_xor(hi, mask);
  return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 shfl64(u64 v, int src) {
  u32 lo = (u32)v, hi = (u32)(v >> 32);
  lo = __shfl(lo, src);
  hi = __shfl(hi, src);
  return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 shfl_up64(u64 v, int d) {
  u32 lo = (u32)v, hi = (u32)(v >> 32);
  lo = __shfl_up(lo, d);
  hi = __shfl_up(hi, d);
  return ((u64)hi << 32) | lo;
}

// Inclusive scan of the affine chain over lanes 0..kN-1: on return lane l holds
// sum_{k<=l} K2^(l-k) * d_k. (General path.)
template <int kN>
__device__ __forceinline__ u64 chain_scan(u64 d, int lane) {
#pragma unroll
  for (int o = 1; o < kN; o <<= 1) {
    const u64 up = shfl_up64(d, o);
    if (lane >= o) d += ipow(K2, o) * up;
  }
  return d;
}

// Value of the butterfly partner across lane bit kMask. Any partner on the other side of that bit
// will do as long as later levels stay inside the halves this level made, so inside a row of 16
// lanes the mirror patterns serve (15-i, 7-i, 3-i, i^1); across rows it takes a bpermute.
template <int kMask>
__device__ __forceinline__ u64 partner64(u64 v) {
  if constexpr (kMask >= 16) return shfl_xor64(v, kMask);
  else if constexpr (kMask == 8) return dpp64<kDppRowMirror>(v);
  else if constexpr (kMask == 4) return dpp64<kDppRowHalfMirror>(v);
  else if constexpr (kMask == 2) return dpp64<kDppQuadReverse>(v);
  else return dpp64<kDppQuadSwap>(v);
}

// One step of the transposing butterfly across lane bit kMask: of the two partials a and b, lanes
// with the bit clear keep a and receive their partner's a, lanes with the bit set keep b and
// receive their partner's b; the result is the sum. Across rows (16 or 32 lanes apart) this is
// what the row-swapping instructions of this GPU do to a pair of registers - one swap per 32-bit
// half and no selects, where the LDS crossbar (ds_bpermute) needs a select of what to send, a
// select of what to keep and a round trip through the LDS for each half. Inside a row the DPP
// patterns serve.
typedef __attribute__((ext_vector_type(2))) unsigned swapped_t;
template <int kMask>
__device__ __forceinline__ u64 exchange_add(u64 a, u64 b, bool bit_set) {
  if constexpr (kMask == 32 || kMask == 16) {
    swapped_t lo, hi;
    if constexpr (kMask == 32) {  // rows 2,3 of the first operand <-> rows 0,1 of the second
      lo = __builtin_amdgcn_permlane32_swap((u32)a, (u32)b, false, false);
      hi = __builtin_amdgcn_permlane32_swap((u32)(a >> 32), (u32)(b >> 32), false, false);
    } else {                      // odd rows of the first operand <-> even rows of the second
      lo = __builtin_amdgcn_permlane16_swap((u32)a, (u32)b, false, false);
      hi = __builtin_amdgcn_permlane16_swap((u32)(a >> 32), (u32)(b >> 32), false, false);
    }
    // first result: the lane's own kept partial; second: the partner's partial of the same kind
    return (((u64)hi.x << 32) | lo.x) + (((u64)hi.y << 32) | lo.y);
  } else {
    const u64 send = bit_set ? a : b;
    const u64 keep = bit_set ? b : a;
    return keep + partner64<kMask>(send);
  }
}

// ---- fast path: block sizes 16, 32, 64 -------------------------------------------------------
// With kMatch the kernel also looks every hash up in the index as soon as it is formed (one lane
// per block, the lane reads the whole bucket) and reduces the first miss of the request, so the
// probe latency of one wavefront overlaps the hash arithmetic of the others and the hashes need not
// travel through memory between two launches.
struct MatchOut {
  Table table;
  u64* values_out;      // nullable
  int32_t* match_len;
  // routing decision in the same launch (kRoute): index values are read as pod sets
  int n_pods;
  const int32_t* pod_load;
  u64 thr_num, thr_den;
  int32_t* pod_out;
  int32_t* hit_len_out;
};

constexpr int kSubTokens = 1024;  // tokens a wavefront loads at a time: 16 loads of 64 tokens
constexpr int kLoads = kSubTokens / kWave;

// A tile is kSub sub-steps of 1024 tokens. Each sub-step reduces its tokens to block sums (one per
// lane, 1024 / kB of them); the finalisers, the chain scan and the lookup run once per tile over
// the block sums of all its sub-steps, so with kSub = kB / 16 they always work on 64 blocks and
// their cost per token does not grow with the block size (they are 40 % of a sub-step's arithmetic:
// 64-token blocks hashed with one sub-step per tile spend 1.9 times as long per block as with four).
// kSub = 1 keeps a tile at 1024 tokens, which is what the lengths-only form wants: a miss is seen
// after 1024 tokens and everything behind it is dropped.
//
// kRoute (with kMatch and kLengths) turns the launch into the whole routing decision: a block's
// index value is the set of pods holding it, the pods holding ALL of blocks 0..j are the running
// AND of those sets, and the request is done where that AND becomes empty - the longest prefix any
// pod holds and its holders fall out of a cross-lane AND scan per tile (carried between the
// wavefronts of a shared request through LDS, like the chain state), then the last wavefront left
// picks the least-loaded candidate. Tokens go in, a pod comes out; no hash or value array exists.
template <int kB, int kSub, int kHashWaves, bool kMatch, bool kLengths, bool kRoute = false>
// (7 wavefronts per SIMD: the register budget this sets - 72 instead of 95 with the lookups - costs
// nothing in the loops and is worth 2-7 % on the fused kernel)
// (the routing form carries more state across its tiles and gets the registers for it: 5 wavefronts)
__global__ __launch_bounds__(kHashWaves* kWave)
    __attribute__((amdgpu_waves_per_eu(kRoute ? 5 : 7, kRoute ? 5 : 7))) void block_hash_pow2_kernel(
    const int32_t* __restrict__ tokens, const int64_t* __restrict__ tok_off,
    const int64_t* __restrict__ blk_off, int n_req, int lg_run, u64 seed, u64* __restrict__ hash_out,
    MatchOut mo, int solo_tiles) {
  static_assert(kB == 16 || kB == 32 || kB == 64, "block size");
  constexpr int kTileTokens = kSub * kSubTokens;
  constexpr int kNBs = kSubTokens / kB;   // blocks per sub-step
  constexpr int kNB = kSub * kNBs;        // blocks per tile
  static_assert(kNB <= kWave && kNB >= 16, "a tile's blocks fit one wavefront");
  constexpr int kGroups = kWave / kB;     // blocks covered by one 64-token load
  constexpr int kLgB = kB == 16 ? 4 : (kB == 32 ? 5 : 6);
  __shared__ u64 lds_aggr[2][kHashWaves];
  __shared__ int lds_first[kHashWaves];
  __shared__ int lds_stop[2];  // a wavefront of the workgroup missed in the round of this parity
  __shared__ u64 lds_set[2][kHashWaves];        // kRoute: AND of a tile's pod sets
  __shared__ u64 lds_last_set[kHashWaves];      // kRoute: per wavefront, the last non-empty running AND ...
  __shared__ int64_t lds_last_pos[kHashWaves];  // ... the block it belongs to ...
  __shared__ int lds_count[kHashWaves][2];      // ... and how many of its blocks had a non-empty AND / held the fallback pod
  static_assert(!kRoute || (kMatch && kLengths), "the routing form stops at the first empty set");

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const u64 pos_const = K0 * (u64)((lane & (kB - 1)) + 1);
  // K2^(pos+1), pos = lane within its row of 16: weight of the state entering the row
  constexpr int kRows = kNB / 16;
  const int row = lane >> 4;
  const u64 row_w = kChainPowers.v[lane & 15];
  // This lane ends up with block `lane` of the tile, i.e. block lane % kNBs of sub-step lane / kNBs;
  // src_lane is the lane that holds that block's sum after the sub-step's butterfly.
  const int sub_of_lane = lane / kNBs;
  const int blk_in_sub = lane % kNBs;
  const int src_lane = ((blk_in_sub % kGroups) * kB + ((blk_in_sub / kGroups) << (kLgB - 4))) & (kWave - 1);

  // One request per workgroup. A request of at most solo_tiles tiles is hashed by wavefront 0 on
  // its own (carry in registers, no barrier; the other wavefronts leave at once); a longer one is
  // shared by all wavefronts (carry through LDS, one barrier per round).
  // With the lookups in this kernel the requests are dealt to the XCDs in runs (see
  // request_of_workgroup; config 2: -6 % time). Hashing alone streams the tokens faster with
  // neighbouring requests on different XCDs (a contiguous map costs it 8 %).
  const int r = kMatch ? request_of_workgroup(blockIdx.x, lg_run) : (int)blockIdx.x;
  if (r >= n_req) return;
  const int64_t b0 = blk_off[r];
  const int64_t n_r = blk_off[r + 1] - b0;
  const int64_t n_tiles = (n_r + kNB - 1) / kNB;
  const bool solo = kHashWaves == 1 || n_tiles <= solo_tiles;
  if (solo && wave != 0) return;
  // kRoute: one lane per pod. The least-request pod over all pods (the fallback), ties to the lower
  // id, is the minimum of (load, id).
  u64 my_rank = ~0ull, all_pods = 0;
  int fallback_pod = 0;
  if constexpr (kRoute) {
    all_pods = (1ull << mo.n_pods) - 1ull;  // n_pods <= 63
    if (lane < mo.n_pods) my_rank = ((u64)(u32)mo.pod_load[lane] << 8) | (u64)lane;
    fallback_pod = (int)(wave_min64(my_rank) & 0xFF);
  }
  if (n_r <= 0) {
    if constexpr (kRoute) {
      if (lane == 0) {
        mo.pod_out[r] = fallback_pod;
        mo.hit_len_out[r] = 0;
      }
    } else if (kMatch && lane == 0) {
      mo.match_len[r] = 0;
    }
    return;
  }
  u64 alive = all_pods;   // kRoute: pods holding every block before this round's tiles
  u64 last_set = 0;       // the last non-empty running AND this wavefront saw, and its block
  int64_t last_pos = -1;
  int n_nonempty = 0, n_fallback = 0;
  int parity = 0;
  int64_t first_miss = n_r;
  bool miss_seen = false;  // wavefront-uniform: one of this wavefront's lookups has missed
  [[maybe_unused]] bool ask = false;  // whether lookup_tile should still test a tile's last key first
  if constexpr (kMatch) ask = mo.table.guess_present;
  if constexpr (kLengths && !kRoute) {
    if (!solo && threadIdx.x < 2) lds_stop[threadIdx.x] = 0;  // ordered before its first reader by the first round's barrier
  }
  const int64_t n_tok = n_r * kB;  // tokens that belong to full blocks
  const int32_t* tok = tokens + tok_off[r];
  u64* out = hash_out + b0;
  u64 carry = fin(seed ^ K3);  // chain state before the first block of this round's tiles
  const int stride = solo ? 1 : kHashWaves;
  for (int64_t tile0 = 0; tile0 < n_tiles; tile0 += stride) {
    if (!solo) parity ^= 1;
    const int64_t tile = solo ? tile0 : tile0 + wave;
    const int64_t tbase = tile * kTileTokens;
    u64 csum = 0;  // sum of block `lane` of this tile
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub) {
      const int64_t sbase = tbase + (int64_t)sub * kSubTokens;
      if (sbase >= n_tok) break;  // nothing of the request is left (also a wavefront past the last tile)
      u64 p[kLoads];
      // 16 coalesced loads; tokens past the last full block read as 0 and are never used
      int32_t raw[kLoads];
      if (sbase + kSubTokens <= n_tok) {  // whole sub-step inside the request: no per-load bounds checks
#pragma unroll
        for (int k = 0; k < kLoads; ++k) raw[k] = __builtin_nontemporal_load(tok + sbase + k * kWave + lane);
#pragma unroll
        for (int k = 0; k < kLoads; ++k) {
          const u64 y = ((u64)(u32)raw[k] ^ pos_const) * K1;
          p[k] = y ^ (y >> 32);
        }
      } else {
        // the request's full blocks end inside this sub-step: rows of 64 tokens that lie wholly before
        // that end are read like any other, the row the end falls in lane by lane, the rest not at all
        // (the row counts are the same in every lane, so only one row pays for a comparison)
        const int full_rows = (int)((n_tok - sbase) / kWave), rest = (int)((n_tok - sbase) % kWave);
#pragma unroll
        for (int k = 0; k < kLoads; ++k) {
          raw[k] = 0;
          if (k < full_rows) raw[k] = __builtin_nontemporal_load(tok + sbase + k * kWave + lane);
          else if (k == full_rows && lane < rest) raw[k] = __builtin_nontemporal_load(tok + sbase + k * kWave + lane);
        }
        // loads that lie behind the request's last full block altogether skip their arithmetic
        const int live = full_rows + (rest != 0);
#pragma unroll
        for (int k = 0; k < kLoads; ++k) {
          p[k] = 0;
          if (k < live) {
            const u64 y = ((u64)(u32)raw[k] ^ pos_const) * K1;
            p[k] = y ^ (y >> 32);
          }
        }
      }
      // transposing butterfly: 16 partials per lane -> 1, summed over the lanes of a block
      u64 q8[8], q4[4], q2[2], c;
#pragma unroll
      for (int t = 0; t < 8; ++t) q8[t] = exchange_add<kB / 2>(p[t], p[t + 8], lane & (kB / 2));
#pragma unroll
      for (int t = 0; t < 4; ++t) q4[t] = exchange_add<kB / 4>(q8[t], q8[t + 4], lane & (kB / 4));
#pragma unroll
      for (int t = 0; t < 2; ++t) q2[t] = exchange_add<kB / 8>(q4[t], q4[t + 2], lane & (kB / 8));
      c = exchange_add<kB / 16>(q2[0], q2[1], lane & (kB / 16));
      if constexpr (kB >= 64) c += partner64<2>(c);
      if constexpr (kB >= 32) c += partner64<1>(c);
      // now the lane with load index k = (lane >> (kLgB-4)) & 15 and group g = lane / kB holds the
      // sum of the sub-step's block k*kGroups + g; every lane fetches the block it is to hold, and
      // the lanes of this sub-step keep it
      c = shfl64(c, src_lane);
      if constexpr (kSub == 1) csum = c;
      else csum = sub_of_lane == sub ? c : csum;
    }
    const int64_t jb = tile * kNB + lane;  // block index inside the request
    const bool valid = lane < kNB && jb < n_r;
    u64 local = valid ? fin(csum) : 0ull;
    // chain, level 1: scan inside each row of 16 lanes (DPP row shifts feed 0 into the row's
    // first lanes, so no lane needs a condition)
    local += ipow(K2, 1) * dpp64<kDppRowShr + 1>(local);
    local += ipow(K2, 2) * dpp64<kDppRowShr + 2>(local);
    local += ipow(K2, 4) * dpp64<kDppRowShr + 4>(local);
    local += ipow(K2, 8) * dpp64<kDppRowShr + 8>(local);
    // chain, level 2: the state entering each row. y[r] = state entering row r if the tile started
    // from 0; the tile's aggregate is the state leaving its last row.
    u64 y[kRows + 1];
    y[0] = 0;
#pragma unroll
    for (int r = 0; r < kRows; ++r) y[r + 1] = ipow(K2, 16) * y[r] + readlane64(local, 16 * r + 15);
    const u64 aggr = y[kRows];
    u64 cin = carry;  // chain state entering this wavefront's tile
    if (!solo) {
      if (lane == 0) lds_aggr[parity][wave] = aggr;
      __syncthreads();
      // match lengths as the only output: once some wavefront has missed in the previous round,
      // every tile from here on lies behind that miss and the whole workgroup is done
      if constexpr (kLengths && !kRoute) {
        if (lds_stop[parity ^ 1]) break;
      }
      for (int w = 0; w < wave; ++w) cin = ipow(K2, kNB) * cin + lds_aggr[parity][w];
    }
    // state entering this lane's row = y[row] + K2^(16*row) * cin; this lane's block then adds
    // K2^(pos+1) times that to its in-row scan value
    u64 enter = cin;
#pragma unroll
    for (int r = 1; r < kRows; ++r) enter = row == r ? y[r] + ipow(K2, 16 * r) * cin : enter;
    const u64 h = out_hash(row_w * enter + local);
    if (valid && (!kMatch || hash_out)) out[jb] = h;
    // kLengths: the caller wants neither hashes nor per-block values, so nothing behind this
    // wavefront's first miss can change an output any more (its tiles come in rising order): a
    // wavefront that hashes its request alone is done with it, one that shares it stops looking up
    // and tells the others (see lds_stop).
    if constexpr (kRoute) {
      u64 v = lookup_tile(mo.table, h, valid, ask);
      v = valid ? (v == kNoValue ? 0ull : (v & all_pods)) : all_pods;  // lanes past the end do not shrink the set
      v = and_scan64(v, lane);  // over the tile's blocks
      const u64 tile_set = readlane64(v, kWave - 1);
      u64 before = alive;  // pods holding every block before this wavefront's tile
      if (!solo) {
        if (lane == 0) lds_set[parity][wave] = tile_set;
        __syncthreads();
        for (int w = 0; w < wave; ++w) before &= lds_set[parity][w];
      }
      v &= before;
      const u64 nonempty = __ballot(valid && v != 0);  // a run of ones from lane 0
      const int cnt = __popcll(nonempty);
      if (cnt > 0) {
        last_pos = tile * kNB + cnt - 1;
        last_set = readlane64(v, cnt - 1);
      }
      n_nonempty += cnt;
      n_fallback += __popcll(__ballot(valid && ((v >> fallback_pod) & 1ull)));
      if (solo) {
        alive = before & tile_set;
      } else {
        for (int w = 0; w < kHashWaves; ++w) alive &= lds_set[parity][w];
      }
      if (alive == 0) break;  // the same for every wavefront of the workgroup: no pod holds more
    } else if constexpr (kLengths) {
      if (miss_seen) {
        if (solo) break;
        goto tile_done;
      }
    }
    if constexpr (kMatch && !kRoute) {
      const u64 v = lookup_tile(mo.table, h, valid, ask);
      if (valid && mo.values_out) mo.values_out[b0 + jb] = v;
      const u64 miss = __ballot(valid && v == kNoValue);
      if (miss && first_miss == n_r) first_miss = tile * kNB + (__ffsll((unsigned long long)miss) - 1);
      if constexpr (kLengths) miss_seen = miss != 0 || miss_seen;
    }
  tile_done:
    if constexpr (kLengths && !kRoute) {
      if (!solo && miss_seen && lane == 0) lds_stop[parity] = 1;
    }
    if (!solo) {
      // chain state after all tiles of this iteration (only used if another iteration follows,
      // in which case every tile of this one was full)
      for (int w = 0; w < kHashWaves; ++w) carry = ipow(K2, kNB) * carry + lds_aggr[parity][w];
    } else {
      carry = ipow(K2, kNB) * carry + aggr;
    }
  }
  if constexpr (kRoute) {
    // the longest prefix any pod holds = the blocks with a non-empty running AND (a run from block
    // 0), its holders = the AND at the run's last block, wherever in the workgroup that block was
    if (!solo) {
      if (lane == 0) {
        lds_last_set[wave] = last_set;
        lds_last_pos[wave] = last_pos;
        lds_count[wave][0] = n_nonempty;
        lds_count[wave][1] = n_fallback;
      }
      __syncthreads();
      if (wave != 0) return;
      n_nonempty = n_fallback = 0;
      for (int w = 0; w < kHashWaves; ++w) {
        n_nonempty += lds_count[w][0];
        n_fallback += lds_count[w][1];
        if (lds_last_pos[w] > last_pos || w == 0) {
          last_pos = lds_last_pos[w];
          last_set = lds_last_set[w];
        }
      }
    }
    const int64_t best_len = n_nonempty;
    const bool aware = best_len > 0 && (u64)best_len * mo.thr_den >= mo.thr_num * (u64)n_r;
    u64 rank = my_rank;
    if (aware && !((last_set >> lane) & 1ull)) rank = ~0ull;  // candidates: the holders of the longest prefix
    rank = wave_min64(rank);
    if (lane == 0) {
      mo.pod_out[r] = (int32_t)(rank & 0xFF);
      mo.hit_len_out[r] = (int32_t)(aware ? best_len : n_fallback);
    }
    return;
  }
  if constexpr (kMatch) {
    if (solo) {
      if (lane == 0) mo.match_len[r] = (int)first_miss;
    } else {
      if (lane == 0) lds_first[wave] = (int)first_miss;
      __syncthreads();
      if (threadIdx.x == 0) {
        int m = lds_first[0];
        for (int w = 1; w < kHashWaves; ++w) m = lds_first[w] < m ? lds_first[w] : m;
        mo.match_len[r] = m;
      }
    }
  }
}

// ---- general path: any block size in [1, 1024] ------------------------------------------------
// Phase 1: each wavefront reduces whole blocks to digests and parks them in hash_out.
// Phase 2: wavefront 0 runs the chain over the request's digests, 64 blocks at a time.
__global__ __launch_bounds__(kGeneralWaves* kWave) void block_hash_general_kernel(
    const int32_t* __restrict__ tokens, const int64_t* __restrict__ tok_off,
    const int64_t* __restrict__ blk_off, int block_size, u64 seed, u64* __restrict__ hash_out) {
  const int r = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t b0 = blk_off[r];
  const int64_t n_r = blk_off[r + 1] - b0;
  if (n_r <= 0) return;
  const int32_t* tok = tokens + tok_off[r];
  u64* out = hash_out + b0;
  for (int64_t j = wave; j < n_r; j += kGeneralWaves) {
    const int32_t* blk = tok + j * block_size;
    u64 c = 0;
    for (int i = lane; i < block_size; i += kWave) {
      const u64 y = ((u64)(u32)blk[i] ^ (K0 * (u64)(i + 1))) * K1;
      c += y ^ (y >> 32);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) c += shfl_xor64(c, m);
    if (lane == 0) out[j] = fin(c);
  }
  __syncthreads();  // digests written by this workgroup are visible to it after the barrier
  if (wave != 0) return;
  const u64 carry_w = kChainPowers.v[lane];
  u64 carry = fin(seed ^ K3);
  for (int64_t base = 0; base < n_r; base += kWave) {
    const int64_t j = base + lane;
    const u64 d = j < n_r ? out[j] : 0ull;
    const u64 local = chain_scan<kWave>(d, lane);
    const u64 s = carry_w * carry + local;
    if (j < n_r) out[j] = out_hash(s);
    carry = shfl64(s, kWave - 1);
  }
}

}  // namespace
}  // namespace aibx

namespace aibx {
namespace {

constexpr int kSoloTokens = 8192;       // hashing alone
constexpr int kSoloTokensFused = 4096;  // with the lookups in the launch a wavefront's tile takes longer, so long requests are shared earlier

template <bool kMatch, bool kLengths, bool kRoute = false>
int launch_hash(const int32_t* d_tokens, const int64_t* d_tok_off, const int64_t* d_blk_off, int32_t n_req,
                int64_t n_blocks_total, int32_t block_size, u64 seed, u64* d_hash_out, MatchOut mo, hipStream_t st) {
  // Launch shape, from what the host knows (batch size and mean request length):
  //  - fewer than 4,096 requests: eight wavefronts per request, every request of more than one tile
  //    shared by the eight, so that a small batch finishes in few serial tiles (1,024 lognormal
  //    requests of up to 32,768 tokens, tokens -> values in one launch: 35 us with four wavefronts,
  //    27 us with eight, 35 us with sixteen);
  //  - thousands of requests averaging under two tiles: one wavefront per request and nothing else
  //    (workgroups of four with three idle wavefronts cost +50 % on 100,000 one-tile requests);
  //  - thousands of longer requests: the GPU is full anyway, so a request of up to 8,192 tokens (4,096
  //    with the lookups in the launch; at least one tile) is hashed
  //    by one wavefront of its workgroup, and only longer ones - which would otherwise run on as
  //    the batch's tail - by the four together. Measured on 4 Mi-block batches against one
  //    wavefront for every request: lognormal lengths -15 % time (-24 % with the lookups in the same
  //    launch), uniform 4-tile requests equal, uniform 16-tile requests of 64-token blocks -7 % (+5 %).
  // Wavefronts that share a long request: four; two when only the match lengths (or the routing
  // decision) are wanted from a batch of thousands of requests, where everything a wavefront does
  // behind the first miss is wasted and a round of two wastes less (tokens -> lengths on 4 Mi-block
  // batches whose requests miss early: -12 % to -45 % against rounds of four). A small batch leaves
  // most of the GPU idle, so there wasted work is free and the serial chain is what counts: eight
  // wavefronts and full tiles in every form (128 requests of 16,384 tokens with every block present,
  // tokens -> pod: 26 us with rounds of two 1024-token tiles).
  constexpr int kShared = kLengths ? 2 : 4;
  constexpr int kSubFew = kLengths ? 1 : 0;  // 0: as many sub-steps as fill the 64 lanes
  const int64_t mean_tokens = n_blocks_total * (int64_t)block_size / n_req;
  const bool small_batch = n_req < 4096;
  const bool single = !small_batch && mean_tokens < 2 * kSubTokens;
  const int tile_tokens = (kLengths && !small_batch) ? kSubTokens : block_size * kWave;
  const int solo_tokens = kMatch ? kSoloTokensFused : kSoloTokens;
  const int solo_tiles = small_batch || solo_tokens < tile_tokens ? 1 : solo_tokens / tile_tokens;
  const int lg_run = request_run_lg(n_req);
  dim3 grid(kMatch ? workgroups_for_requests(n_req, lg_run) : (unsigned)n_req);
#define AIBX_LAUNCH_HASH(B)                                                                                    \
  if (single)                                                                                                  \
    block_hash_pow2_kernel<B, (kSubFew ? kSubFew : B / 16), 1, kMatch, kLengths, kRoute><<<grid, kWave, 0, st>>>( \
        d_tokens, d_tok_off, d_blk_off, n_req, lg_run, seed, d_hash_out, mo, 0);                               \
  else if (small_batch)                                                                                        \
    block_hash_pow2_kernel<B, B / 16, 8, kMatch, kLengths, kRoute><<<grid, 8 * kWave, 0, st>>>(                \
        d_tokens, d_tok_off, d_blk_off, n_req, lg_run, seed, d_hash_out, mo, solo_tiles);                      \
  else                                                                                                         \
    block_hash_pow2_kernel<B, (kSubFew ? kSubFew : B / 16), kShared, kMatch, kLengths, kRoute>                 \
        <<<grid, kShared * kWave, 0, st>>>(d_tokens, d_tok_off, d_blk_off, n_req, lg_run, seed, d_hash_out,    \
                                           mo, solo_tiles)
  switch (block_size) {
    case 16: AIBX_LAUNCH_HASH(16); break;
    case 32: AIBX_LAUNCH_HASH(32); break;
    case 64: AIBX_LAUNCH_HASH(64); break;
    default: return AIBX_ERR_UNSUPPORTED;
  }
#undef AIBX_LAUNCH_HASH
  return launch_status();
}

}  // namespace
}  // namespace aibx

extern "C" int aibx_block_hash(const int32_t* d_tokens, const int64_t* d_tok_off,
                               const int64_t* d_blk_off, int32_t n_req, int64_t n_blocks_total,
                               int32_t block_size, uint64_t seed, uint64_t* d_hash_out,
                               void* stream) {
  using namespace aibx;
  if (n_req < 0 || n_blocks_total < 0 || block_size < 1 || block_size > 1024) return AIBX_ERR_INVALID_ARG;
  if (n_req == 0 || n_blocks_total == 0) return AIBX_OK;
  if (!d_tokens || !d_tok_off || !d_blk_off || !d_hash_out) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_tokens, 4) || !aligned(d_tok_off, 8) || !aligned(d_blk_off, 8) || !aligned(d_hash_out, 8))
    return AIBX_ERR_ALIGN;
  hipStream_t st = as_stream(stream);
  if (block_size == 16 || block_size == 32 || block_size == 64)
    return launch_hash<false, false>(d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed, d_hash_out, MatchOut{}, st);
  block_hash_general_kernel<<<dim3((u32)n_req), kGeneralWaves * kWave, 0, st>>>(d_tokens, d_tok_off, d_blk_off,
                                                                               block_size, seed, d_hash_out);
  return launch_status();
}

extern "C" int aibx_hash_match(const aibx_index_t* index, const int32_t* d_tokens, const int64_t* d_tok_off,
                               const int64_t* d_blk_off, int32_t n_req, int64_t n_blocks_total,
                               int32_t block_size, uint64_t seed, uint64_t* d_hash_out,
                               uint64_t* d_values_out, int32_t* d_match_len, void* stream) {
  using namespace aibx;
  if (!index || n_req < 0 || n_blocks_total < 0 || block_size < 1 || block_size > 1024) return AIBX_ERR_INVALID_ARG;
  if (n_req == 0) return AIBX_OK;
  if (!d_tok_off || !d_blk_off || !d_match_len) return AIBX_ERR_INVALID_ARG;
  if (n_blocks_total > 0 && !d_tokens) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_tokens, 4) || !aligned(d_tok_off, 8) || !aligned(d_blk_off, 8) || !aligned(d_hash_out, 8) ||
      !aligned(d_values_out, 8) || !aligned(d_match_len, 4))
    return AIBX_ERR_ALIGN;
  if (block_size != 16 && block_size != 32 && block_size != 64) {
    // other block sizes: the two separate launches, which need the hash array as the hand-over
    if (!d_hash_out) return AIBX_ERR_UNSUPPORTED;
    const int rc = aibx_block_hash(d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed,
                                   d_hash_out, stream);
    if (rc != AIBX_OK) return rc;
    return aibx_prefix_match(index, d_hash_out, d_blk_off, n_req, n_blocks_total, d_values_out, d_match_len,
                             stream);
  }
  MatchOut mo = {};
  mo.table = table_of(index);
  mo.values_out = d_values_out;
  mo.match_len = d_match_len;
  if (!d_hash_out && !d_values_out)  // match lengths only
    return launch_hash<true, true>(d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed, d_hash_out,
                                   mo, as_stream(stream));
  return launch_hash<true, false>(d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed, d_hash_out,
                                  mo, as_stream(stream));
}

extern "C" int aibx_hash_match_route(const aibx_index_t* index, const int32_t* d_tokens, const int64_t* d_tok_off,
                                     const int64_t* d_blk_off, int32_t n_req, int64_t n_blocks_total,
                                     int32_t block_size, uint64_t seed, int32_t n_pods, const int32_t* d_pod_load,
                                     uint64_t threshold_num, uint64_t threshold_den, int32_t* d_pod_out,
                                     int32_t* d_hit_len_out, void* stream) {
  using namespace aibx;
  if (!index || n_req < 0 || n_blocks_total < 0 || block_size < 1 || block_size > 1024) return AIBX_ERR_INVALID_ARG;
  if (n_pods < 1 || n_pods > 63 || threshold_den == 0) return AIBX_ERR_INVALID_ARG;
  if (threshold_num > 0xFFFFFFFFull || threshold_den > 0xFFFFFFFFull) return AIBX_ERR_INVALID_ARG;
  if (n_req == 0) return AIBX_OK;
  if (!d_tok_off || !d_blk_off || !d_pod_load || !d_pod_out || !d_hit_len_out) return AIBX_ERR_INVALID_ARG;
  if (n_blocks_total > 0 && !d_tokens) return AIBX_ERR_INVALID_ARG;
  if (!aligned(d_tokens, 4) || !aligned(d_tok_off, 8) || !aligned(d_blk_off, 8) || !aligned(d_pod_load, 4) ||
      !aligned(d_pod_out, 4) || !aligned(d_hit_len_out, 4))
    return AIBX_ERR_ALIGN;
  // other block sizes would need a hash array to hand over between launches, which this call has not
  if (block_size != 16 && block_size != 32 && block_size != 64) return AIBX_ERR_UNSUPPORTED;
  MatchOut mo = {};
  mo.table = table_of(index);
  mo.n_pods = n_pods;
  mo.pod_load = d_pod_load;
  mo.thr_num = threshold_num;
  mo.thr_den = threshold_den;
  mo.pod_out = d_pod_out;
  mo.hit_len_out = d_hit_len_out;
  return launch_hash<true, true, true>(d_tokens, d_tok_off, d_blk_off, n_req, n_blocks_total, block_size, seed, nullptr,
                                       mo, as_stream(stream));
}
