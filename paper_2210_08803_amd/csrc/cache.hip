// Inference embedding cache: set-associative tags probed by groups of `ways` lanes, a pooled
// gather that reads hits from HBM, and a fully parallel insertion that reproduces "insert the
// distinct missing keys in first-appearance order, LRU victim per set at call granularity".
//
// Insertion without a sequential pass: the victims a set can give up in one call are a fixed list
// once the call's hits are stamped (empty ways by index, then untouched ways by (stamp, way)),
// because an inserted way is stamped with the current epoch and cannot be chosen again.  So the
// k-th distinct missing key of a set (in first-appearance order) takes the k-th entry of that
// list, or is skipped when the list is shorter.
//
// Two code paths compute exactly the same thing:
//   * large calls: probe -> first-appearance dedup of the misses (shared with the embedding hash)
//     -> each distinct missing row is fetched ONCE across the host link into a staging area in
//     HBM -> gather (hits from cache lines, misses from staging) -> stable radix sort of
//     (set, first-appearance index) -> per-set placement -> fill from staging;
//   * small calls (<= kSmallMaxKeys keys): one fused probe+gather kernel (misses read straight
//     from the pinned host table) and one single-block kernel for the whole insertion, because at
//     a few hundred keys the cost is kernel launches, not bytes.
#include <algorithm>

#include "common.h"
#include "rowvec.h"
#include "blockscan.h"
#include "hash_internal.h"

struct hctr_cache {
  char* storage;
  int64_t num_sets;
  int32_t ways, dim;
  const float* host_table;
  int64_t host_rows;
  size_t off_tags, off_stamps, off_data;
  uint32_t epoch;          // host's copy of the call count, kept to see when the count nears its limit
                           // (the kernels read the device's own count, which replays of a captured call advance)
  uint32_t epoch_limit;    // a call that finds epoch >= this first lowers stamps and epoch by half of it
  int64_t small_max_keys;  // calls with at most this many keys take the fused small-call kernels
};

namespace hctr {

typedef unsigned long long u64;
constexpr uint32_t kNoLine = 0xFFFFFFFFu;
constexpr uint32_t kStaged = 0x80000000u;  // line_of value: the row is in the staging area at (v & ~kStaged)
constexpr int kSmallMaxKeys = 8192;   // 104 KB of LDS in cache_insert_small

struct CacheHeader {  // first 256 bytes of the cache storage
  u64 stats[6];       // queries, hits, (misses = queries - hits, filled in on the host), inserts, evictions, skipped
  uint32_t epoch;     // number of query / insert calls so far: the stamp of the last finished call
  uint32_t pad0;
  u64 call_acc;       // classifying kernel in flight: blocks finished << 40 | hits so far (0 between kernels)
  uint32_t pad[48];
};
constexpr int kAccShift = 40;

// The call count lives on the device so that a captured call can be replayed: every block of the
// classifying kernel reads it on entry and works under stamp = count + 1; the kernels that follow in
// the same call read the count as it is then.  Each block reports once, with one atomic that carries
// its hits and counts it as finished; the block that finds all others finished has the call's total
// hits in hand and publishes statistics and the new count (no block waits for another).
__device__ __forceinline__ void cache_block_report(CacheHeader* hdr, uint32_t block_hits, uint32_t epoch,
                                                   uint32_t nnz) {
  const u64 old = atomicAdd(&hdr->call_acc, (1ull << kAccShift) | (u64)block_hits);
  if ((old >> kAccShift) == (u64)gridDim.x - 1ull) {
    hdr->stats[0] += (u64)nnz;
    hdr->stats[1] += (old & ((1ull << kAccShift) - 1ull)) + (u64)block_hits;
    hdr->epoch = epoch;
    hdr->call_acc = 0;
  }
}
static_assert(sizeof(CacheHeader) == 256, "header is one 256-byte block");

__global__ void cache_store_u32(uint32_t* where, uint32_t value) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *where = value;
}

// The divisor of the set index, with the reciprocal that turns the 64-bit remainder (a few hundred
// instructions when left to the compiler) into a multiply-high and at most two subtractions.
struct SetDiv {
  u64 n;      // num_sets
  u64 recip;  // floor((2^64 - 1) / n)
};
static inline SetDiv make_set_div(int64_t num_sets) { return SetDiv{(u64)num_sets, ~0ull / (u64)num_sets}; }

// set = x mod num_sets with x = key * 0x9E3779B97F4A7C15 mod 2^64, x ^= x >> 32 (exact).
__device__ __forceinline__ u64 set_of(u64 key, SetDiv d) {
  u64 x = key * 0x9E3779B97F4A7C15ull;
  x ^= x >> 32;
  const u64 q = __umul64hi(x, d.recip);   // floor(x / n) or one or two less
  u64 r = x - q * d.n;
  if (r >= d.n) r -= d.n;
  if (r >= d.n) r -= d.n;
  return r;
}

__global__ __launch_bounds__(256) void cache_clear(u64* tags, uint32_t* stamps, uint64_t n_lines,
                                                   CacheHeader* hdr) {
  const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (i < n_lines) { tags[i] = kEmptyKey; stamps[i] = 0u; }
  if (i < 6) hdr->stats[i] = 0;
  if (i == 0) { hdr->epoch = 0; hdr->call_acc = 0; }
}

// Stamps are 32-bit call counts; before the count runs out every stamp is lowered by `by` (and the
// host's count with them).  Stamps at or below `by` become 0, "never used".
__global__ __launch_bounds__(256) void cache_lower_stamps(uint32_t* __restrict__ stamps, uint64_t n_lines,
                                                          uint32_t by, CacheHeader* hdr) {
  const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (i == 0) hdr->epoch = hdr->epoch > by ? hdr->epoch - by : 0u;   // nothing else reads it in this kernel
  if (i < n_lines) {
    const uint32_t s = stamps[i];
    stamps[i] = s > by ? s - by : 0u;
  }
}

// Position of this way in its set's victim list (ways used in this call are not in the list), and
// the length of the list.  Called by all WAYS lanes of a group at once, one way per lane.
template <int WAYS>
__device__ __forceinline__ void victim_order(u64 tag, uint32_t stamp, uint32_t epoch, int way, bool* eligible,
                                             bool* empty, uint32_t* pos, uint32_t* n_elig) {
  *empty = tag == kEmptyKey;
  *eligible = *empty || stamp < epoch;
  const u64 okey = !*eligible ? ~0ull : (*empty ? (u64)way : (((u64)stamp + 1ull) << 8) | (u64)way);
  uint32_t p = 0, ne = 0;
#pragma unroll
  for (int w = 0; w < WAYS; ++w) {
    const u64 other = (u64)__shfl((long long)okey, w, WAYS);
    p += other < okey ? 1u : 0u;
    ne += other != ~0ull ? 1u : 0u;
  }
  *pos = p;
  *n_elig = ne;
}

// The same through LDS, for a block whose waves all rank at once: 64 cross-lane reads per call (the
// shuffles above, two per 64-bit word) keep the LDS pipe of the compute unit busy for longer than
// everything else in the placement step; here a lane stores one 32-bit code and reads the group's
// codes four at a time.  code = 0 (empty way), last use + 1, or all ones (used in this call); ties go
// to the lower way, as above.  `codes` = the group's WAYS words; the group's lanes are in one wave,
// whose LDS instructions are served in order.
template <int WAYS>
__device__ __forceinline__ void victim_order_lds(uint32_t* codes, u64 tag, uint32_t stamp, uint32_t epoch,
                                                 int way, bool* eligible, bool* empty, uint32_t* pos,
                                                 uint32_t* n_elig) {
  *empty = tag == kEmptyKey;
  *eligible = *empty || stamp < epoch;
  const uint32_t code = !*eligible ? 0xFFFFFFFFu : (*empty ? 0u : stamp + 1u);
  codes[way] = code;
  __builtin_amdgcn_wave_barrier();
  uint32_t p = 0, ne = 0;
  if constexpr (WAYS >= 4) {
#pragma unroll
    for (int w0 = 0; w0 < WAYS; w0 += 4) {
      const uint4 o = *reinterpret_cast<const uint4*>(codes + w0);
      const uint32_t other[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        p += (other[k] < code || (other[k] == code && w0 + k < way)) ? 1u : 0u;
        ne += other[k] != 0xFFFFFFFFu ? 1u : 0u;
      }
    }
  } else {
#pragma unroll
    for (int w = 0; w < WAYS; ++w) {
      const uint32_t other = codes[w];
      p += (other < code || (other == code && w < way)) ? 1u : 0u;
      ne += other != 0xFFFFFFFFu ? 1u : 0u;
    }
  }
  __builtin_amdgcn_wave_barrier();   // the next call's stores come after these loads
  *pos = p;
  *n_elig = ne;
}

// ------------------------------------------------------------------------------------------------
// Large calls
// ------------------------------------------------------------------------------------------------

// Classify every key against the tags as they stand (nothing writes tags in this kernel).  A group
// of WAYS lanes compares one tag per lane and takes KP = min(8, WAYS) consecutive keys: lane j of
// the group loads key j and works out its set (the 64-bit remainder is the expensive part, so it is
// done once per key, not once per lane), the group then shares both by shuffle and has its KP tag
// loads in flight together.  A block reports its hits with a single atomic (one atomic per wave
// on one address would serialise hundreds of thousands of them).
template <int WAYS>
__global__ __launch_bounds__(256) void cache_probe(const u64* __restrict__ tags,
                                                   uint32_t* __restrict__ stamps, SetDiv num_sets,
                                                   int64_t host_rows, CacheHeader* hdr,
                                                   const int64_t* __restrict__ keys, uint32_t nnz,
                                                   uint32_t* __restrict__ line_of,
                                                   uint8_t* __restrict__ hit_mask,
                                                   uint32_t* __restrict__ miss_flag) {
  constexpr int KP = WAYS >= 8 ? 8 : WAYS;
  __shared__ uint32_t block_hits;
  const uint32_t epoch = hdr->epoch + 1u;   // this call's stamp (see cache_block_report)
  if (threadIdx.x == 0) block_hits = 0;
  __syncthreads();
  const int way = threadIdx.x % WAYS;
  const int lane = threadIdx.x & 63;
  constexpr uint64_t kGroupOnes = WAYS == 64 ? ~0ull : ((1ull << (WAYS & 63)) - 1ull);
  const uint64_t gmask = kGroupOnes << (lane - way);
  const uint32_t n_groups = gridDim.x * (256u / WAYS);
  uint32_t hits = 0;
  // the grid is bounded (each block ends with an atomic on the one hit counter), groups stride over the keys
  for (uint64_t i0_64 = (uint64_t)((blockIdx.x * 256u + threadIdx.x) / WAYS) * KP; i0_64 < nnz;
       i0_64 += (uint64_t)n_groups * KP) {
    const uint32_t i0 = (uint32_t)i0_64;
    const int64_t own_key = (way < KP && i0 + way < nnz) ? keys[i0 + way] : -1;
    const u64 own_set = own_key >= 0 ? set_of((u64)own_key, num_sets) : 0;
    int64_t key[KP];
    u64 tag[KP];
    u64 slot[KP];
#pragma unroll
    for (int j = 0; j < KP; ++j) {
      key[j] = (int64_t)__shfl((long long)own_key, j, WAYS);
      slot[j] = (u64)__shfl((long long)own_set, j, WAYS) * WAYS + way;
      tag[j] = key[j] >= 0 ? tags[slot[j]] : kEmptyKey;
    }
#pragma unroll
    for (int j = 0; j < KP; ++j) {
      const bool match = key[j] >= 0 && tag[j] == (u64)key[j];
      // store only: reading the stamp first, to spare a popular key's line thousands of equal
      // stores, put a load latency on every key and measured slower at every size (1.7 M keys:
      // 572 -> 519 us)
      if (match) stamps[slot[j]] = epoch;
      const uint64_t mine = __ballot(match) & gmask;
      const bool hit = mine != 0;
      uint32_t line = match ? (uint32_t)slot[j] : kNoLine;
      if (hit) line = __shfl(line, __ffsll((unsigned long long)mine) - 1);
      if (way == 0 && i0 + j < nnz) {
        line_of[i0 + j] = hit ? line : kNoLine;
        if (hit_mask) hit_mask[i0 + j] = hit ? 1 : 0;
        if (miss_flag) miss_flag[i0 + j] = (!hit && key[j] >= 0 && key[j] < host_rows) ? 1u : 0u;
        hits += hit ? 1u : 0u;
      }
    }
  }
  if (hits) atomicAdd(&block_hits, hits);
  __syncthreads();
  if (threadIdx.x == 0) cache_block_report(hdr, block_hits, epoch, nnz);
}

// What a pooling pass takes in.  kPoolAll: every key (a one-call query).  kPoolHits: cached rows only,
// a missing key adds nothing (first phase of a two-phase query).  kAddMisses: only the rows of the
// missing keys, added to what the first phase left in the output (second phase).
enum PoolMode { kPoolAll = 0, kPoolHits = 1, kAddMisses = 2 };

// Where a key's vector lives: cache line, staging row, host row, or nowhere (zeros).
template <int MODE>
__device__ __forceinline__ const float* row_source(uint32_t line, int64_t key, const float* data,
                                                   const float* staging, const float* host_table,
                                                   int64_t host_rows, int D) {
  if (line == kNoLine) {
    if (MODE == kPoolHits) return nullptr;
    return (key >= 0 && key < host_rows) ? host_table + key * D : nullptr;
  }
  if (line & kStaged) return MODE == kPoolHits ? nullptr : staging + (int64_t)(line & ~kStaged) * D;
  return MODE == kAddMisses ? nullptr : data + (int64_t)line * D;
}

// Pooled gather of one bag by one wave: 64/LPR lane groups take the bag's keys round robin, U row
// loads each in flight; group partial sums are staged in LDS and added in group order.  With
// kAddMisses the sum of the missing rows is added to the bag's output, and a bag without a missing
// key is left alone.
template <int LPR, int U, int MODE>
__device__ __forceinline__ void gather_bag(const float* __restrict__ data, const float* __restrict__ staging,
                                           const float* __restrict__ host_table, int64_t host_rows, int D,
                                           const int64_t* __restrict__ keys,
                                           const uint32_t* __restrict__ line_of, int64_t b0, int64_t b1,
                                           bool live, uint32_t bag, float* __restrict__ out, float* part) {
  constexpr int G = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int g = lane / LPR, sub = lane % LPR;
  const int col = blockIdx.y * (LPR * 4) + sub * 4;
  const bool active = col < D;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  bool took = false;
  for (int64_t j = b0 + g; j < b1; j += G * U) {
    const float* src[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t jj = j + u * G;
      src[u] = jj < b1 ? row_source<MODE>(line_of[jj], keys[jj], data, staging, host_table, host_rows, D) : nullptr;
      took = took || src[u] != nullptr;
    }
    f32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      v[u] = (src[u] != nullptr && active) ? load4(src[u] + col) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
  }
  if (G > 1) {
    if (g > 0) {
      float* p = &part[((g - 1) * LPR + sub) * 4];
      p[0] = acc.x; p[1] = acc.y; p[2] = acc.z; p[3] = acc.w;
    }
    __syncthreads();
    if (g == 0) {
#pragma unroll
      for (int gg = 1; gg < G; ++gg) {
        const float* p = &part[((gg - 1) * LPR + sub) * 4];
        acc.x += p[0]; acc.y += p[1]; acc.z += p[2]; acc.w += p[3];
      }
    }
  }
  if (MODE == kAddMisses) {
    const bool any = __ballot(took) != 0;   // some lane of the wave met a missing row of this bag
    if (live && g == 0 && active && any) {
      float* to = out + (int64_t)bag * D + col;
      f32x4 o = load4(to);
      o.x += acc.x; o.y += acc.y; o.z += acc.z; o.w += acc.w;
      store4(to, o);
    }
  } else if (live && g == 0 && active) {
    const float v[4] = {acc.x, acc.y, acc.z, acc.w};
    store_stream<4>(out + (int64_t)bag * D + col, v);
  }
}

template <int LPR, int U, int MODE>
__global__ __launch_bounds__(256) void cache_gather(const float* __restrict__ data,
                                                    const float* __restrict__ staging,
                                                    const float* __restrict__ host_table,
                                                    int64_t host_rows, int D,
                                                    const int64_t* __restrict__ keys,
                                                    const uint32_t* __restrict__ line_of,
                                                    const int64_t* __restrict__ offsets, int64_t hotness,
                                                    uint32_t n_bags, float* __restrict__ out) {
  constexpr int G = 64 / LPR;
  __shared__ float part[4][(G > 1 ? (G - 1) : 1) * LPR * 4];
  const int wave = threadIdx.x >> 6;
  const uint32_t bag = blockIdx.x * 4u + wave;
  const bool live = bag < n_bags;
  int64_t b0 = 0, b1 = 0;
  if (live) {
    b0 = offsets ? offsets[bag] : (int64_t)bag * hotness;
    b1 = offsets ? offsets[bag + 1] : (int64_t)(bag + 1) * hotness;
  }
  gather_bag<LPR, U, MODE>(data, staging, host_table, host_rows, D, keys, line_of, b0, b1, live, bag, out,
                           part[wave]);
}

// Positions of the missing keys, ascending: position i goes to list[idx[i]] when its flag is set
// (idx = exclusive scan of the flags).
__global__ __launch_bounds__(256) void cache_list_missing(const uint32_t* __restrict__ flag,
                                                          const uint32_t* __restrict__ idx, uint32_t n,
                                                          uint32_t* __restrict__ list) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < n && flag[i]) list[idx[i]] = i;
}

// First appearances of the missing keys, q = 0..n_new-1 in first-appearance order: remember the
// key, emit the (set, q) sort word, and leave q in the key's scratch slot for the other positions.
__global__ __launch_bounds__(256) void cache_list_new(const HashWsHeader* hdr,
                                                      const int64_t* __restrict__ keys,
                                                      const uint32_t* __restrict__ miss_pos,
                                                      const uint32_t* __restrict__ scr_slot,
                                                      const uint32_t* __restrict__ first,
                                                      const uint32_t* __restrict__ rank, SetDiv num_sets,
                                                      uint32_t* __restrict__ scratch, u64* __restrict__ new_key,
                                                      u64* __restrict__ sort_kv) {
  const uint32_t m = blockIdx.x * 256u + threadIdx.x;
  if (m >= hdr->n_miss || !first[m]) return;
  const uint32_t q = rank[m];
  const u64 key = (u64)keys[miss_pos[m]];
  new_key[q] = key;
  sort_kv[q] = (set_of(key, num_sets) << 32) | (u64)q;   // sorted by set, payload = first-appearance index
  scratch[scr_slot[m]] = q;   // the slot's position has served its purpose (first[] is final)
}

// Every missing position learns the staging row of its key.
__global__ __launch_bounds__(256) void cache_mark_staged(const HashWsHeader* hdr,
                                                         const uint32_t* __restrict__ miss_pos,
                                                         const uint32_t* __restrict__ scr_slot,
                                                         const uint32_t* __restrict__ scratch,
                                                         uint32_t* __restrict__ line_of) {
  const uint32_t m = blockIdx.x * 256u + threadIdx.x;
  if (m >= hdr->n_miss) return;
  line_of[miss_pos[m]] = kStaged | scratch[scr_slot[m]];
}

// One row per group of LPR lanes: host table -> staging (the only trip across the host link).
template <int LPR>
__global__ __launch_bounds__(256) void cache_fetch(const float* __restrict__ host_table, int D,
                                                   const HashWsHeader* hdr, const u64* __restrict__ new_key,
                                                   float* __restrict__ staging) {
  const int sub = threadIdx.x % LPR;
  const uint32_t n_new = hdr->n_new;
  for (uint32_t q = (blockIdx.x * 256u + threadIdx.x) / LPR; q < n_new; q += gridDim.x * (256u / LPR)) {
    const float* src = host_table + (int64_t)new_key[q] * D;
    float* to = staging + (int64_t)q * D;
    for (int col = sub * 4; col < D; col += LPR * 4) store4(to + col, load4(src + col));
  }
}

// One group of WAYS lanes per sorted position; the group at the start of a set's run places the
// whole run.  dst[q] = cache line that key q goes to, or kNoLine when its insert is skipped.
template <int WAYS>
__global__ __launch_bounds__(256) void cache_place(u64* __restrict__ tags, uint32_t* __restrict__ stamps,
                                                   CacheHeader* hdr,
                                                   const HashWsHeader* ws_hdr, const u64* __restrict__ skv,
                                                   const u64* __restrict__ new_key,
                                                   uint32_t* __restrict__ dst) {
  __shared__ uint32_t blk_stats[3];
  const uint32_t epoch = hdr->epoch;   // the classifying kernel of this call has published it
  if (threadIdx.x < 3) blk_stats[threadIdx.x] = 0;
  __syncthreads();
  const int way = threadIdx.x % WAYS;
  const uint32_t n_new = ws_hdr->n_new;
  for (uint32_t j = (blockIdx.x * 256u + threadIdx.x) / WAYS; j < n_new; j += gridDim.x * (256u / WAYS)) {
    const uint32_t set = (uint32_t)(skv[j] >> 32);
    if (j > 0 && (uint32_t)(skv[j - 1] >> 32) == set) continue;  // not the first of its set
    const uint64_t line = (uint64_t)set * WAYS + way;
    bool eligible, empty;
    uint32_t pos, n_elig;
    victim_order<WAYS>(tags[line], stamps[line], epoch, way, &eligible, &empty, &pos, &n_elig);
    uint32_t inserted = 0, evicted = 0, skipped = 0;
    for (uint32_t k = 0; j + k < n_new && (uint32_t)(skv[j + k] >> 32) == set; ++k) {
      const uint32_t q = (uint32_t)skv[j + k];
      if (k < n_elig) {
        if (eligible && pos == k) {
          tags[line] = new_key[q];
          stamps[line] = epoch;
          dst[q] = (uint32_t)line;
          evicted += empty ? 0u : 1u;
        }
        inserted += 1;
      } else {
        if (way == 0) dst[q] = kNoLine;
        skipped += 1;
      }
    }
#pragma unroll
    for (int d = WAYS / 2; d >= 1; d >>= 1) evicted += __shfl_xor(evicted, d, WAYS);  // per lane -> per group
    if (way == 0) {
      if (inserted) atomicAdd(&blk_stats[0], inserted);
      if (evicted) atomicAdd(&blk_stats[1], evicted);
      if (skipped) atomicAdd(&blk_stats[2], skipped);
    }
  }
  __syncthreads();
  if (threadIdx.x < 3 && blk_stats[threadIdx.x]) atomicAdd(&hdr->stats[3 + threadIdx.x], (u64)blk_stats[threadIdx.x]);
}

// Copy the rows of the placed keys from staging into their cache lines.
template <int LPR>
__global__ __launch_bounds__(256) void cache_fill(float* __restrict__ data, const float* __restrict__ staging,
                                                  int D, const HashWsHeader* ws_hdr,
                                                  const uint32_t* __restrict__ dst) {
  const int sub = threadIdx.x % LPR;
  const uint32_t n_new = ws_hdr->n_new;
  for (uint32_t q = (blockIdx.x * 256u + threadIdx.x) / LPR; q < n_new; q += gridDim.x * (256u / LPR)) {
    const uint32_t line = dst[q];
    if (line == kNoLine) continue;
    const float* src = staging + (int64_t)q * D;
    float* to = data + (int64_t)line * D;
    for (int col = sub * 4; col < D; col += LPR * 4) store4(to + col, load4(src + col));
  }
}

// ------------------------------------------------------------------------------------------------
// Small calls
// ------------------------------------------------------------------------------------------------

// Probe + gather in one launch, a block per four bags: the block first classifies the keys of its
// bags (a group of WAYS lanes per key), then each wave pools one bag.  Misses are read straight
// from the host table.  Rows must fit one column chunk (dim <= LPR * 4, i.e. dim <= 256).
template <int WAYS, int LPR, int MODE>
__global__ __launch_bounds__(256) void cache_query_small(const u64* __restrict__ tags,
                                                         uint32_t* __restrict__ stamps, SetDiv num_sets,
                                                         const float* __restrict__ data,
                                                         const float* __restrict__ host_table,
                                                         int64_t host_rows, int D, CacheHeader* hdr,
                                                         const int64_t* __restrict__ keys,
                                                         uint32_t nnz, const int64_t* __restrict__ offsets,
                                                         int64_t hotness, uint32_t n_bags,
                                                         uint32_t* line_of, uint8_t* __restrict__ hit_mask,
                                                         uint32_t* __restrict__ miss_flag,
                                                         float* __restrict__ out) {
  constexpr int G = 64 / LPR;
  __shared__ float part[4][(G > 1 ? (G - 1) : 1) * LPR * 4];
  __shared__ uint32_t block_hits;
  const uint32_t epoch = hdr->epoch + 1u;   // this call's stamp (see cache_block_report)
  if (threadIdx.x == 0) block_hits = 0;
  __syncthreads();
  const uint32_t bag_lo = blockIdx.x * 4u;
  const uint32_t bag_hi = bag_lo + 4u < n_bags ? bag_lo + 4u : n_bags;
  const int64_t k_lo = offsets ? offsets[bag_lo] : (int64_t)bag_lo * hotness;
  const int64_t k_hi = offsets ? offsets[bag_hi] : (int64_t)bag_hi * hotness;
  {
    const int way = threadIdx.x % WAYS;
    const int lane = threadIdx.x & 63;
    constexpr uint64_t kGroupOnes = WAYS == 64 ? ~0ull : ((1ull << (WAYS & 63)) - 1ull);
    const uint64_t gmask = kGroupOnes << (lane - way);
    constexpr int kPerRound = 256 / WAYS;
    uint32_t hits = 0;
    const int64_t n_rounds = (k_hi - k_lo + kPerRound - 1) / kPerRound;
    for (int64_t r = 0; r < n_rounds; ++r) {
      const int64_t i = k_lo + r * kPerRound + threadIdx.x / WAYS;
      const int64_t key = i < k_hi ? keys[i] : -1;
      u64 slot = 0;
      bool match = false;
      if (key >= 0) {
        slot = set_of((u64)key, num_sets) * WAYS + way;
        match = tags[slot] == (u64)key;
        if (match) stamps[slot] = epoch;   // store only, see cache_probe
      }
      const uint64_t mine = __ballot(match) & gmask;
      const bool hit = mine != 0;
      uint32_t line = match ? (uint32_t)slot : kNoLine;
      if (hit) line = __shfl(line, __ffsll((unsigned long long)mine) - 1);
      if (way == 0 && i < k_hi) {
        line_of[i] = hit ? line : kNoLine;
        if (hit_mask) hit_mask[i] = hit ? 1 : 0;
        if (miss_flag) miss_flag[i] = (!hit && key >= 0 && key < host_rows) ? 1u : 0u;
        hits += hit ? 1u : 0u;
      }
    }
    if (hits) atomicAdd(&block_hits, hits);
  }
  __threadfence_block();
  __syncthreads();   // line_of of this block's keys is complete and visible to the whole block
  if (threadIdx.x == 0) cache_block_report(hdr, block_hits, epoch, nnz);
  const int wave = threadIdx.x >> 6;
  const uint32_t bag = bag_lo + wave;
  const bool live = bag < n_bags;
  int64_t b0 = 0, b1 = 0;
  if (live) {
    b0 = offsets ? offsets[bag] : (int64_t)bag * hotness;
    b1 = offsets ? offsets[bag + 1] : (int64_t)(bag + 1) * hotness;
  }
  // no line of a small call is staged; `data` only fills the staging argument
  if (out != nullptr)   // uniform: an insert-only call pools nothing
    gather_bag<LPR, 4, MODE>(data, data, host_table, host_rows, D, keys, line_of, b0, b1, live, bag, out,
                             part[wave]);
}

// The whole insertion of a small call in one block of 1024 threads (n <= kSmallMaxKeys keys).
//   1. compact the missing positions (block scan), keys to LDS;  2. first appearances (pairwise
//   compare);  3. number them (block scan) -> distinct keys q;    4. per key: rank among the earlier
//   keys of its set, victim list of the set read from the state as the probe left it;
//   5. after a barrier, write tags and stamps;                    6. copy the rows host -> cache lines.
template <int WAYS>
__global__ __launch_bounds__(1024) void cache_insert_small(u64* __restrict__ tags, uint32_t* __restrict__ stamps,
                                                           float* __restrict__ data, CacheHeader* hdr,
                                                           const float* __restrict__ host_table, int D,
                                                           SetDiv num_sets,
                                                           const int64_t* __restrict__ keys,
                                                           const uint32_t* __restrict__ miss_flag, uint32_t n) {
  constexpr int T = 1024;
  const uint32_t epoch = hdr->epoch;   // the classifying kernel of this call has published it
  constexpr int PER = kSmallMaxKeys / T;            // positions per thread in the two scans
  __shared__ uint32_t pos_or_dst[kSmallMaxKeys];    // missing positions (steps 1-3), then q -> line (4-6)
  __shared__ u64 wide[kSmallMaxKeys];               // keys of the missing positions (1-2), then two u32 arrays
  __shared__ uint8_t is_first[kSmallMaxKeys];
  __shared__ uint32_t scan_lds[T / 64 + 1];
  __shared__ uint32_t counters[3];                  // inserted, evicted, skipped
  __shared__ __attribute__((aligned(16))) uint32_t way_code[T];   // victim ranking, one word per lane
  u64* mkey = wide;                                               // m -> key
  uint32_t* ukey_pos = reinterpret_cast<uint32_t*>(wide);         // q -> position of the key's first appearance
  uint32_t* uset = reinterpret_cast<uint32_t*>(wide) + kSmallMaxKeys;  // q -> set
  const uint32_t tid = threadIdx.x;
  if (tid < 3) counters[tid] = 0;

  // 1. missing positions, ascending (flags and keys of all the thread's positions requested at once,
  //    index clamped instead of a branch: a load under a branch is waited for before the next one)
  if (n == 0) return;   // block-uniform
  uint32_t f[PER], cnt = 0;
  u64 kk[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const uint32_t p = tid * PER + i;
    const uint32_t pc = p < n ? p : n - 1;
    f[i] = miss_flag[pc];
    kk[i] = (u64)keys[pc];
  }
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    f[i] = (tid * PER + i < n && f[i]) ? 1u : 0u;
    cnt += f[i];
  }
  uint32_t M;
  uint32_t run = block_exclusive_scan<T>(cnt, scan_lds, &M);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    if (f[i]) {
      pos_or_dst[run] = tid * PER + i;
      mkey[run] = kk[i];
      ++run;
    }
  }
  __syncthreads();
  if (M == 0) return;   // block-uniform

  // 2. first appearance <=> no earlier missing position holds the same key
  //    With fewer missing positions than threads, C = T / M threads share the earlier keys of one
  //    position (183 positions: 5 threads each), eight keys per step read independently of each other.
  for (uint32_t m = tid; m < M; m += T) is_first[m] = 1;
  __syncthreads();
  {
    const uint32_t C = M < T ? T / M : 1u;
    for (uint32_t w = tid; w < M * C; w += T) {
      const uint32_t m = w / C, c = w % C;
      const uint32_t len = (m + C - 1) / C;
      const uint32_t j_lo = c * len, j_hi = j_lo + len < m ? j_lo + len : m;
      const u64 key = mkey[m];
      bool first = true;
      for (uint32_t j0 = j_lo; j0 < j_hi && first; j0 += 8) {
        u64 k[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) k[u] = mkey[j0 + u < j_hi ? j0 + u : m];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) first = first && !(j0 + u < j_hi && k[u] == key);
      }
      if (!first) is_first[m] = 0;   // several threads may store the same 0
    }
  }
  __syncthreads();

  // 3. number the first appearances; from here on `wide` holds ukey_pos and uset
  cnt = 0;
  uint32_t my_pos[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const uint32_t m = tid * PER + i;
    f[i] = (m < M && is_first[m]) ? 1u : 0u;
    my_pos[i] = f[i] ? pos_or_dst[m] : 0u;
    cnt += f[i];
  }
  uint32_t Uq;
  run = block_exclusive_scan<T>(cnt, scan_lds, &Uq);   // ends with a barrier: all reads above are done
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    if (f[i]) {
      ukey_pos[run] = my_pos[i];
      uset[run] = (uint32_t)set_of((u64)keys[my_pos[i]], num_sets);
      ++run;
    }
  }
  __syncthreads();

  // 4. placement decisions, one group of WAYS lanes per distinct key (cache state is only read here)
  const int way = tid % WAYS;
  constexpr uint32_t kGroups = T / WAYS;
  const uint64_t gmask = ((WAYS == 64 ? 0ull : (1ull << (WAYS & 63))) - 1ull) << ((tid & 63) - way);   // this group's lanes
  //    The sets' tags and stamps of four keys per group are requested together: one memory round
  //    trip per four keys instead of one per key.
  constexpr uint32_t kKeysAtOnce = 4;
  for (uint32_t q0 = 0; q0 < Uq; q0 += kKeysAtOnce * kGroups) {
    uint32_t setv[kKeysAtOnce], stv[kKeysAtOnce];
    u64 tagv[kKeysAtOnce];
#pragma unroll
    for (uint32_t b = 0; b < kKeysAtOnce; ++b) {
      const uint32_t q = q0 + b * kGroups + tid / WAYS;
      setv[b] = uset[q < Uq ? q : Uq - 1];            // clamped: loads without a branch
      const uint64_t line = (uint64_t)setv[b] * WAYS + way;
      tagv[b] = tags[line];
      stv[b] = stamps[line];
    }
#pragma unroll
    for (uint32_t b = 0; b < kKeysAtOnce; ++b) {
      const uint32_t q = q0 + b * kGroups + tid / WAYS;
      if (q < Uq) {                                     // uniform within the group of WAYS lanes
        const uint32_t set = setv[b];
        uint32_t krank = 0;                             // earlier distinct keys of the same set
        for (uint32_t j0 = 0; j0 < q; j0 += WAYS) {     // counted by ballot: no cross-lane adds
          const uint32_t j = j0 + way;
          krank += (uint32_t)__popcll(__ballot(j < q && uset[j] == set) & gmask);
        }
        const uint64_t line = (uint64_t)set * WAYS + way;
        bool eligible, empty;
        uint32_t pos, n_elig;
        victim_order_lds<WAYS>(way_code + (tid - way), tagv[b], stv[b], epoch, way, &eligible, &empty, &pos, &n_elig);
        if (krank < n_elig) {
          if (eligible && pos == krank) {
            pos_or_dst[q] = (uint32_t)line;
            atomicAdd(&counters[0], 1u);
            if (!empty) atomicAdd(&counters[1], 1u);
          }
        } else if (way == 0) {
          pos_or_dst[q] = kNoLine;
          atomicAdd(&counters[2], 1u);
        }
      }
    }
  }
  __syncthreads();

  // 5. + 6. publish tags and stamps, copy the rows
  for (uint32_t q = tid; q < Uq; q += T) {
    const uint32_t line = pos_or_dst[q];
    if (line != kNoLine) {
      tags[line] = (u64)keys[ukey_pos[q]];
      stamps[line] = epoch;
    }
  }
  // rows cross the host link: each group of lanes keeps eight row pieces in flight (latency-bound;
  // 256 rows per sweep).  The keys come first, all together, then the rows they name.
  constexpr int kCopyLanes = 32;   // lanes per row copy
  constexpr uint32_t kRowsAtOnce = T / kCopyLanes;
  constexpr int kInFlight = 8;
  for (uint32_t q0 = tid / kCopyLanes; q0 < Uq; q0 += kInFlight * kRowsAtOnce) {
    uint32_t line[kInFlight];
    int64_t src[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const uint32_t q = q0 + u * kRowsAtOnce;
      line[u] = q < Uq ? pos_or_dst[q] : kNoLine;
      src[u] = keys[ukey_pos[q < Uq ? q : Uq - 1]];
    }
    for (int col = (tid % kCopyLanes) * 4; col < D; col += kCopyLanes * 4) {
      f32x4 v[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u)   // unconditional (src always names a real row): no branch between the loads
        v[u] = load4(host_table + src[u] * D + col);
#pragma unroll
      for (int u = 0; u < kInFlight; ++u)
        if (line[u] != kNoLine) store4(data + (int64_t)line[u] * D + col, v[u]);
    }
  }
  if (tid < 3 && counters[tid]) atomicAdd(&hdr->stats[3 + tid], (u64)counters[tid]);
}

// ------------------------------------------------------------------------------------------------
// Manipulation operators
// ------------------------------------------------------------------------------------------------

// Update, step 1: position i' of the REVERSED key list (key = keys[n-1-i']) is probed; resident keys
// are flagged and remembered with their line.  The first-appearance dedup over the reversed list
// then marks, per key, its last occurrence in the caller's order - the row that must win.
template <int WAYS>
__global__ __launch_bounds__(256) void cache_update_probe(const u64* __restrict__ tags, SetDiv num_sets,
                                                          const int64_t* __restrict__ keys, uint32_t n,
                                                          int64_t* __restrict__ keys_rev,
                                                          uint32_t* __restrict__ line_of,
                                                          uint32_t* __restrict__ flag) {
  const int way = threadIdx.x % WAYS;
  const int lane = threadIdx.x & 63;
  constexpr uint64_t kGroupOnes = WAYS == 64 ? ~0ull : ((1ull << (WAYS & 63)) - 1ull);
  const uint64_t gmask = kGroupOnes << (lane - way);
  const uint32_t n_groups = gridDim.x * (256u / WAYS);
  const uint32_t rounds = (n + n_groups - 1) / n_groups;   // same trip count for every lane
  for (uint32_t r = 0; r < rounds; ++r) {
    const uint32_t ip = r * n_groups + (blockIdx.x * 256u + threadIdx.x) / WAYS;
    const int64_t key = ip < n ? keys[n - 1 - ip] : -1;
    u64 slot = 0;
    bool match = false;
    if (key >= 0) {
      slot = set_of((u64)key, num_sets) * WAYS + way;
      match = tags[slot] == (u64)key;
    }
    const uint64_t mine = __ballot(match) & gmask;
    const bool hit = mine != 0;
    uint32_t line = match ? (uint32_t)slot : kNoLine;
    if (hit) line = __shfl(line, __ffsll((unsigned long long)mine) - 1);
    if (way == 0 && ip < n) {
      keys_rev[ip] = key;
      line_of[ip] = hit ? line : kNoLine;
      flag[ip] = hit ? 1u : 0u;
    }
  }
}

// Update, step 2: the winners copy their rows into the cache lines.
template <int LPR>
__global__ __launch_bounds__(256) void cache_update_copy(float* __restrict__ data, int D,
                                                         const HashWsHeader* hdr,
                                                         const uint32_t* __restrict__ miss_pos,
                                                         const uint32_t* __restrict__ first,
                                                         const uint32_t* __restrict__ line_of,
                                                         const float* __restrict__ rows, uint32_t n) {
  const int sub = threadIdx.x % LPR;
  const uint32_t n_res = hdr->n_miss;   // here: number of resident positions
  for (uint32_t m = (blockIdx.x * 256u + threadIdx.x) / LPR; m < n_res; m += gridDim.x * (256u / LPR)) {
    if (!first[m]) continue;
    const uint32_t ip = miss_pos[m];
    const float* src = rows + (int64_t)(n - 1 - ip) * D;
    float* to = data + (int64_t)line_of[ip] * D;
    for (int col = sub * 4; col < D; col += LPR * 4) store4(to + col, load4(src + col));
  }
}

// Refresh: every resident line re-reads its row from the host table.
template <int LPR>
__global__ __launch_bounds__(256) void cache_refresh_lines(const u64* __restrict__ tags, float* __restrict__ data,
                                                           const float* __restrict__ host_table, int D,
                                                           uint64_t n_lines) {
  const int sub = threadIdx.x % LPR;
  for (uint64_t line = (blockIdx.x * 256ull + threadIdx.x) / LPR; line < n_lines;
       line += (uint64_t)gridDim.x * (256u / LPR)) {
    const u64 tag = tags[line];
    if (tag == kEmptyKey) continue;
    const float* src = host_table + (int64_t)tag * D;
    float* to = data + (int64_t)line * D;
    for (int col = sub * 4; col < D; col += LPR * 4) store4(to + col, load4(src + col));
  }
}

// ------------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------------
struct CacheWsLayout {
  size_t header, line_of, flag, idx, miss_pos, scr_slot, first, rank, scan_tmp, scratch, new_key, kv0, kv1,
      hist, aux, dst, staging, total;
  uint32_t scratch_cap_max;
  int sort_bits;
  SortPlan sort;
};

static CacheWsLayout cache_ws_layout(const hctr_cache* c, int64_t nnz_max) {
  CacheWsLayout L{};
  const size_t n = (size_t)(nnz_max > 0 ? nnz_max : 1);
  Carver cv(nullptr);
  auto at = [&](size_t bytes) { size_t o = cv.off; cv.take<char>(bytes); return o; };
  L.sort_bits = ceil_log2((uint64_t)c->num_sets + 1);
  L.sort = sort_plan((uint32_t)n, L.sort_bits);
  L.header = at(sizeof(HashWsHeader));
  L.line_of = at(n * 4); L.flag = at(n * 4);
  L.idx = at(n * 4);
  L.scan_tmp = at(scan_tmp_count((uint32_t)n) * 4);
  if ((int64_t)n <= c->small_max_keys && c->dim <= 256) {   // the small-call kernels need nothing else
    L.total = cv.off;
    return L;
  }
  L.miss_pos = at(n * 4);
  L.scr_slot = at(n * 4); L.first = at(n * 4); L.rank = at(n * 4);
  L.scratch_cap_max = dedup_scratch_capacity((uint32_t)n);
  L.scratch = at((size_t)L.scratch_cap_max * 4);
  L.new_key = at(n * 8);
  L.kv0 = at(n * 8); L.kv1 = at(n * 8);
  L.hist = at(L.sort.hist_count * 4);
  L.aux = at(L.sort.aux_count * 4);
  L.dst = at(n * 4);
  L.staging = at(n * (size_t)c->dim * 4);
  L.total = cv.off;
  return L;
}

size_t cache_call_ws_bytes(const hctr_cache* c, int64_t nnz) { return cache_ws_layout(c, nnz).total; }

#define HCTR_BY_WAYS(W, CALL)                    \
  switch (W) {                                   \
    case 1: CALL(1); break;                      \
    case 2: CALL(2); break;                      \
    case 4: CALL(4); break;                      \
    case 8: CALL(8); break;                      \
    case 16: CALL(16); break;                    \
    case 32: CALL(32); break;                    \
    default: CALL(64); break;                    \
  }
#define HCTR_BY_LPR(L, CALL)                     \
  switch (L) {                                   \
    case 4: CALL(4); break;                      \
    case 8: CALL(8); break;                      \
    case 16: CALL(16); break;                    \
    case 32: CALL(32); break;                    \
    default: CALL(64); break;                    \
  }

struct QueryArgs {
  const hctr_cache* c;
  const int64_t* keys;
  const int64_t* offsets;
  int64_t hotness;
  uint32_t n, n_bags;
  float* out;
  uint8_t* hit_mask;
  uint32_t* line_of;
  uint32_t* flag;   // nullptr when nothing will be inserted
  hipStream_t stream;
  u64* tags() const { return reinterpret_cast<u64*>(c->storage + c->off_tags); }
  uint32_t* stamps() const { return reinterpret_cast<uint32_t*>(c->storage + c->off_stamps); }
  float* data() const { return reinterpret_cast<float*>(c->storage + c->off_data); }
  CacheHeader* hdr() const { return reinterpret_cast<CacheHeader*>(c->storage); }
};

template <int WAYS>
static void launch_probe(const QueryArgs& a) {
  constexpr int KP = WAYS >= 8 ? 8 : WAYS;
  // at least one block: a call whose bags are all empty still counts as a call (the last block to
  // finish publishes the call count)
  const uint32_t blocks = (uint32_t)std::max<int64_t>(1, std::min<int64_t>(ceil_div(ceil_div((int64_t)a.n, KP) * WAYS, 256), 2048));
  hipLaunchKernelGGL((cache_probe<WAYS>), dim3(blocks), dim3(256), 0, a.stream, (const u64*)a.tags(), a.stamps(),
                     make_set_div(a.c->num_sets), a.c->host_rows, a.hdr(), a.keys, a.n, a.line_of, a.hit_mask,
                     a.flag);
}

template <int LPR, int MODE>
static void launch_gather(const QueryArgs& a, const float* staging) {
  dim3 grid((uint32_t)ceil_div(a.n_bags, 4), (uint32_t)ceil_div(a.c->dim, LPR * 4));
  hipLaunchKernelGGL((cache_gather<LPR, 4, MODE>), grid, dim3(256), 0, a.stream, (const float*)a.data(), staging,
                     a.c->host_table, a.c->host_rows, (int)a.c->dim, a.keys, (const uint32_t*)a.line_of,
                     a.offsets, a.hotness, a.n_bags, a.out);
}
template <int MODE>
static void dispatch_gather(int lpr, const QueryArgs& a, const float* staging) {
  switch (lpr) {
    case 4: launch_gather<4, MODE>(a, staging); break;
    case 8: launch_gather<8, MODE>(a, staging); break;
    case 16: launch_gather<16, MODE>(a, staging); break;
    case 32: launch_gather<32, MODE>(a, staging); break;
    default: launch_gather<64, MODE>(a, staging); break;
  }
}

template <int WAYS, int LPR, int MODE>
static void launch_query_small(const QueryArgs& a) {
  dim3 grid((uint32_t)ceil_div(a.n_bags, 4), 1);
  hipLaunchKernelGGL((cache_query_small<WAYS, LPR, MODE>), grid, dim3(256), 0, a.stream, (const u64*)a.tags(),
                     a.stamps(), make_set_div(a.c->num_sets), (const float*)a.data(), a.c->host_table, a.c->host_rows,
                     (int)a.c->dim, a.hdr(), a.keys, a.n, a.offsets, a.hotness, a.n_bags, a.line_of,
                     a.hit_mask, a.flag, a.out);
}

template <int WAYS, int MODE>
static void dispatch_query_small(int lpr, const QueryArgs& a) {
#define CALL(LL) launch_query_small<WAYS, LL, MODE>(a)
  HCTR_BY_LPR(lpr, CALL)
#undef CALL
}

template <int WAYS>
static void launch_insert_small(const QueryArgs& a) {
  hipLaunchKernelGGL((cache_insert_small<WAYS>), dim3(1), dim3(1024), 0, a.stream, a.tags(), a.stamps(), a.data(),
                     a.hdr(), a.c->host_table, (int)a.c->dim, make_set_div(a.c->num_sets), a.keys,
                     (const uint32_t*)a.flag, a.n);
}

template <int WAYS>
static void launch_place(const QueryArgs& a, const HashWsHeader* ws_hdr, const u64* skv, const u64* new_key,
                         uint32_t* dst) {
  // few blocks: each ends with three atomics on the same statistics words
  const uint32_t blocks = (uint32_t)std::min<int64_t>(ceil_div((int64_t)a.n * WAYS, 256), 512);
  hipLaunchKernelGGL((cache_place<WAYS>), dim3(blocks), dim3(256), 0,
                     a.stream, a.tags(), a.stamps(), a.hdr(), ws_hdr, skv, new_key, dst);
}

template <int LPR>
static void launch_fetch_fill(const QueryArgs& a, const HashWsHeader* ws_hdr, const u64* new_key,
                              float* staging, const uint32_t* dst, bool fill) {
  const uint32_t blocks = (uint32_t)std::min<int64_t>(ceil_div((int64_t)a.n * LPR, 256), 4096);
  if (!fill)
    hipLaunchKernelGGL((cache_fetch<LPR>), dim3(blocks), dim3(256), 0, a.stream, a.c->host_table, (int)a.c->dim,
                       ws_hdr, new_key, staging);
  else
    hipLaunchKernelGGL((cache_fill<LPR>), dim3(blocks), dim3(256), 0, a.stream, a.data(), (const float*)staging,
                       (int)a.c->dim, ws_hdr, dst);
}

}  // namespace hctr

using namespace hctr;

static void cache_offsets(int64_t num_sets, int32_t ways, int32_t dim, size_t* tags, size_t* stamps,
                          size_t* data, size_t* total) {
  const size_t lines = (size_t)num_sets * ways;
  size_t off = sizeof(CacheHeader);
  *tags = off; off = align_up(off + lines * 8);
  *stamps = off; off = align_up(off + lines * 4);
  *data = off; off = align_up(off + lines * dim * 4);
  *total = off;
}

static bool cache_shape_ok(int64_t num_sets, int32_t ways, int32_t dim) {
  if (num_sets < 1 || num_sets > 0x7FFFFFFFll) return false;
  if (ways < 1 || ways > 64 || (ways & (ways - 1)) != 0) return false;
  if (dim < 4 || dim % 4 != 0) return false;
  if ((uint64_t)num_sets * ways > 0x7FFFFFFFull) return false;   // line numbers keep their top bit free
  return true;
}

HCTR_API size_t hctr_cache_storage_bytes(int64_t num_sets, int32_t ways, int32_t dim) {
  if (!cache_shape_ok(num_sets, ways, dim)) return 0;
  size_t a, b, c, t;
  cache_offsets(num_sets, ways, dim, &a, &b, &c, &t);
  return t;
}

HCTR_API hctr_status hctr_cache_create(void* storage, size_t storage_bytes, int64_t num_sets, int32_t ways,
                                       int32_t dim, const float* host_table, int64_t host_rows,
                                       void* stream, hctr_cache** out) {
  if (!out) return fail(HCTR_E_NULL_PTR, "out is NULL");
  *out = nullptr;
  if (!storage || !host_table) return fail(HCTR_E_NULL_PTR, "storage / host_table is NULL");
  if (!cache_shape_ok(num_sets, ways, dim))
    return fail(HCTR_E_INVALID_ARG, "num_sets %lld / ways %d (power of two, 1..64) / dim %d (multiple of 4) invalid",
                (long long)num_sets, ways, dim);
  if (host_rows < 1) return fail(HCTR_E_INVALID_ARG, "host_rows %lld < 1", (long long)host_rows);
  if ((uintptr_t)storage % 256 != 0 || (uintptr_t)host_table % 16 != 0)
    return fail(HCTR_E_INVALID_ARG, "storage must be 256-byte and host_table 16-byte aligned");
  hctr_cache* c = new hctr_cache();
  size_t total;
  cache_offsets(num_sets, ways, dim, &c->off_tags, &c->off_stamps, &c->off_data, &total);
  if (storage_bytes < total) {
    delete c;
    return fail(HCTR_E_INVALID_ARG, "storage has %zu bytes, %zu needed", storage_bytes, total);
  }
  c->storage = static_cast<char*>(storage);
  c->num_sets = num_sets; c->ways = ways; c->dim = dim;
  c->host_table = host_table; c->host_rows = host_rows;
  c->epoch = 0;
  c->small_max_keys = kSmallMaxKeys;
  c->epoch_limit = 0xFFFFFF00u;
  const uint64_t lines = (uint64_t)num_sets * ways;
  hipLaunchKernelGGL(cache_clear, dim3((uint32_t)ceil_div((int64_t)(lines > 6 ? lines : 6), 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), reinterpret_cast<u64*>(c->storage + c->off_tags),
                     reinterpret_cast<uint32_t*>(c->storage + c->off_stamps), lines,
                     reinterpret_cast<CacheHeader*>(c->storage));
  hctr_status st = launch_status("cache_clear");
  if (st != HCTR_OK) { delete c; return st; }
  *out = c;
  return HCTR_OK;
}

HCTR_API hctr_status hctr_cache_set_epoch_limit(hctr_cache* c, int64_t limit) {
  if (!c) return fail(HCTR_E_NULL_PTR, "cache is NULL");
  if (limit < 2 || limit > 0xFFFFFF00ll)
    return fail(HCTR_E_INVALID_ARG, "limit %lld outside 2..2^32-256", (long long)limit);
  c->epoch_limit = (uint32_t)limit;
  return HCTR_OK;
}

HCTR_API hctr_status hctr_cache_set_small_call_limit(hctr_cache* c, int64_t max_keys) {
  if (!c) return fail(HCTR_E_NULL_PTR, "cache is NULL");
  if (max_keys < 0 || max_keys > kSmallMaxKeys)
    return fail(HCTR_E_INVALID_ARG, "limit %lld outside 0..%d", (long long)max_keys, kSmallMaxKeys);
  c->small_max_keys = max_keys;
  return HCTR_OK;
}

HCTR_API size_t hctr_cache_workspace_bytes(const hctr_cache* cache, int64_t nnz_max) {
  if (!cache || nnz_max < 0 || nnz_max >= (1ll << 31)) return 0;
  // sized for the general path, which needs the most; it then serves every call of up to nnz_max
  // keys whichever path that call takes
  hctr_cache general = *cache;
  general.small_max_keys = 0;
  return cache_ws_layout(&general, nnz_max).total;
}

// Which part of a query a call runs.  kWhole: classify, pool everything, insert.  kHitsPhase: classify
// and pool the hits only.  kMissPhase: what is left after kHitsPhase on the same keys and workspace
// (add the missing rows to the output, insert); it classifies nothing and starts no new call.
enum QueryPart { kWhole = 0, kHitsPhase = 1, kMissPhase = 2 };

// One query call.  out == nullptr pools nothing (insert-only); ready != nullptr is recorded on the
// stream as soon as out and hit_mask (and the miss list, if asked for) are complete, before any
// insertion work is enqueued.
static hctr_status cache_query_impl(hctr_cache* c, QueryPart part, int64_t batch, int32_t num_slots,
                                    const int64_t* keys, const int64_t* offsets, int64_t nnz,
                                    int32_t insert_missing, float* out, bool need_out, uint8_t* hit_mask,
                                    uint32_t* miss_list, uint32_t* n_missing, void* ws, size_t ws_bytes,
                                    void* stream_, hipEvent_t ready) {
  if (!c) return fail(HCTR_E_NULL_PTR, "cache is NULL");
  if (batch < 0 || num_slots < 1 || nnz < 0) return fail(HCTR_E_INVALID_ARG, "batch / num_slots / nnz invalid");
  const int64_t n_bags = batch * num_slots;
  if (n_bags >= (1ll << 31) || nnz >= (1ll << 31)) return fail(HCTR_E_UNSUPPORTED, "more than 2^31-1 bags or keys");
  int64_t hotness = 0;
  if (!offsets) {
    if (n_bags == 0 ? nnz != 0 : nnz % n_bags != 0)
      return fail(HCTR_E_INVALID_ARG, "offsets == NULL needs nnz (%lld) divisible by the %lld bags",
                  (long long)nnz, (long long)n_bags);
    hotness = n_bags ? nnz / n_bags : 0;
  }
  if ((miss_list == nullptr) != (n_missing == nullptr))
    return fail(HCTR_E_NULL_PTR, "miss_positions and n_missing go together");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // A new call: the count goes up by one (on the device, when the call's first kernel ends), after
  // the stamps have been lowered if it is about to run out.
  auto begin_call = [&]() -> hctr_status {
    if (c->epoch >= c->epoch_limit) {   // the count is about to run out: lower it and every stamp
      const uint32_t by = c->epoch_limit / 2;
      const uint64_t lines = (uint64_t)c->num_sets * c->ways;
      hipLaunchKernelGGL(cache_lower_stamps, dim3((uint32_t)ceil_div((int64_t)lines, 256)), dim3(256), 0, stream,
                         reinterpret_cast<uint32_t*>(c->storage + c->off_stamps), lines, by,
                         reinterpret_cast<CacheHeader*>(c->storage));
      HCTR_TRY(launch_status("cache_lower_stamps"));
      c->epoch -= by;
    }
    c->epoch += 1;
    return HCTR_OK;
  };
  if (n_bags == 0) {
    // No bags: nothing to read or write, no workspace needed, but it is a call like any other for the
    // replacement order (the simulation counts every call): one block of the probe publishes the count.
    if (nnz != 0) return fail(HCTR_E_INVALID_ARG, "nnz must be 0 when there are no bags");
    if (part != kMissPhase) {
      HCTR_TRY(begin_call());
      QueryArgs e{c, nullptr, nullptr, 0, 0u, 0u, nullptr, nullptr, nullptr, nullptr, stream};
#define CALL(W) launch_probe<W>(e)
      HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
      if (n_missing) hipLaunchKernelGGL(cache_store_u32, dim3(1), dim3(64), 0, stream, n_missing, 0u);
      if (ready) HCTR_TRY_HIP(hipEventRecord(ready, stream));
    }
    return launch_status("hctr_cache_query");
  }
  if (!out && need_out) return fail(HCTR_E_NULL_PTR, "out is NULL");
  if (nnz > 0 && !keys) return fail(HCTR_E_NULL_PTR, "keys is NULL");
  if (nnz == 0) insert_missing = 0;   // bags without keys: zeros in the output, one more call counted, nothing to insert
  if (out && (uintptr_t)out % 16 != 0) return fail(HCTR_E_INVALID_ARG, "out must be 16-byte aligned");
  const CacheWsLayout L = cache_ws_layout(c, nnz);
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < L.total) return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L.total);

  char* w = static_cast<char*>(ws);
  HashWsHeader* ws_hdr = reinterpret_cast<HashWsHeader*>(w + L.header);
  if (part != kMissPhase) HCTR_TRY(begin_call());
  // the miss flags serve the insertion, the second phase and the miss list
  const bool want_flags = insert_missing || part != kWhole || miss_list != nullptr;
  QueryArgs a{c, keys, offsets, hotness, (uint32_t)nnz, (uint32_t)n_bags, out, hit_mask,
              reinterpret_cast<uint32_t*>(w + L.line_of),
              want_flags ? reinterpret_cast<uint32_t*>(w + L.flag) : nullptr, stream};
  int lpr = pow2_ceil((int)ceil_div(c->dim, 4));
  lpr = lpr < 4 ? 4 : (lpr > 64 ? 64 : lpr);
  const bool small = nnz <= c->small_max_keys && c->dim <= 256;

  // ---- classify and pool
  if (part != kMissPhase) {
    if (small) {
      if (part == kHitsPhase) {
#define CALL(W) dispatch_query_small<W, kPoolHits>(lpr, a)
        HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
      } else {
#define CALL(W) dispatch_query_small<W, kPoolAll>(lpr, a)
        HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
      }
    } else {
#define CALL(W) launch_probe<W>(a)
      HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
      if (part == kHitsPhase) {
        if (out) dispatch_gather<kPoolHits>(lpr, a, nullptr);
      } else if (!insert_missing) {
        if (out) dispatch_gather<kPoolAll>(lpr, a, nullptr);   // missing rows straight from the host table
      }
    }
    if (miss_list != nullptr && nnz == 0) {   // no keys, none missing (a fill kernel: a memset node may not be captured)
      hipLaunchKernelGGL(cache_store_u32, dim3(1), dim3(64), 0, stream, n_missing, 0u);
    }
    if (miss_list != nullptr && nnz > 0) {   // ascending positions of the missing keys inside the host table
      uint32_t* idx = reinterpret_cast<uint32_t*>(w + L.idx);
      HCTR_TRY(exclusive_scan_u32(a.flag, idx, a.n, reinterpret_cast<uint32_t*>(w + L.scan_tmp), n_missing, stream));
      hipLaunchKernelGGL(cache_list_missing, dim3((uint32_t)ceil_div(a.n, 256)), dim3(256), 0, stream,
                         (const uint32_t*)a.flag, (const uint32_t*)idx, a.n, miss_list);
    }
    // out and hit_mask are complete here on every path but the general one-call path with insertion,
    // which pools after the missing rows have been staged (below)
    const bool pooled_later = part == kWhole && !small && insert_missing;
    if (ready && !pooled_later) HCTR_TRY_HIP(hipEventRecord(ready, stream));
    if (part == kHitsPhase) return launch_status("hctr_cache_query_hits");
  }

  // ---- missing rows into the output (second phase) and insertion
  if (small) {
    if (part == kMissPhase && out) dispatch_gather<kAddMisses>(lpr, a, nullptr);   // straight from the host table
    if (insert_missing && nnz > 0) {
#define CALL(W) launch_insert_small<W>(a)
      HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
    }
    return launch_status("hctr_cache_query");
  }
  if (!insert_missing) {
    if (part == kMissPhase && out) dispatch_gather<kAddMisses>(lpr, a, nullptr);
    return launch_status("hctr_cache_query");
  }
  DedupBuffers B{a.flag,
                 reinterpret_cast<uint32_t*>(w + L.idx),
                 reinterpret_cast<uint32_t*>(w + L.miss_pos),
                 reinterpret_cast<uint32_t*>(w + L.scr_slot),
                 reinterpret_cast<uint32_t*>(w + L.first),
                 reinterpret_cast<uint32_t*>(w + L.rank),
                 reinterpret_cast<uint32_t*>(w + L.scan_tmp),
                 reinterpret_cast<uint32_t*>(w + L.scratch),
                 L.scratch_cap_max,
                 &ws_hdr->n_miss,
                 &ws_hdr->n_new,
                 nullptr};
  HCTR_TRY(dedup_first_appearance(keys, a.n, B, a.stream));
  u64* new_key = reinterpret_cast<u64*>(w + L.new_key);
  u64* kv[2] = {reinterpret_cast<u64*>(w + L.kv0), reinterpret_cast<u64*>(w + L.kv1)};
  uint32_t* dst = reinterpret_cast<uint32_t*>(w + L.dst);
  float* staging = reinterpret_cast<float*>(w + L.staging);
  const uint32_t nb = (uint32_t)ceil_div(a.n, 256);
  hipLaunchKernelGGL(cache_list_new, dim3(nb), dim3(256), 0, a.stream, (const HashWsHeader*)ws_hdr, keys,
                     (const uint32_t*)B.miss_pos, (const uint32_t*)B.scr_slot, (const uint32_t*)B.first,
                     (const uint32_t*)B.rank, make_set_div(c->num_sets), B.scratch, new_key, kv[0]);
  hipLaunchKernelGGL(cache_mark_staged, dim3(nb), dim3(256), 0, a.stream, (const HashWsHeader*)ws_hdr,
                     (const uint32_t*)B.miss_pos, (const uint32_t*)B.scr_slot, (const uint32_t*)B.scratch, a.line_of);
#define CALL(LL) launch_fetch_fill<LL>(a, ws_hdr, new_key, staging, dst, false)
  HCTR_BY_LPR(lpr, CALL)
#undef CALL
  if (out) {
    if (part == kMissPhase) dispatch_gather<kAddMisses>(lpr, a, staging);
    else dispatch_gather<kPoolAll>(lpr, a, staging);
  }
  if (ready && part == kWhole) HCTR_TRY_HIP(hipEventRecord(ready, a.stream));
  HCTR_TRY(radix_sort_u64(L.sort, &ws_hdr->n_new, reinterpret_cast<uint64_t*>(kv[0]),
                          reinterpret_cast<uint64_t*>(kv[1]), reinterpret_cast<uint32_t*>(w + L.hist),
                          reinterpret_cast<uint32_t*>(w + L.aux), false, a.stream));
  const u64* skv = kv[L.sort.passes & 1];
#define CALL(W) launch_place<W>(a, ws_hdr, skv, new_key, dst)
  HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
#define CALL(LL) launch_fetch_fill<LL>(a, ws_hdr, new_key, staging, dst, true)
  HCTR_BY_LPR(lpr, CALL)
#undef CALL
  return launch_status("hctr_cache_query");
}

HCTR_API hctr_status hctr_cache_query(hctr_cache* c, int64_t batch, int32_t num_slots, const int64_t* keys,
                                      const int64_t* offsets, int64_t nnz, int32_t insert_missing,
                                      float* out, uint8_t* hit_mask, void* ws, size_t ws_bytes,
                                      void* stream) {
  return cache_query_impl(c, kWhole, batch, num_slots, keys, offsets, nnz, insert_missing, out, true, hit_mask,
                          nullptr, nullptr, ws, ws_bytes, stream, nullptr);
}

HCTR_API hctr_status hctr_cache_query_async(hctr_cache* c, int64_t batch, int32_t num_slots,
                                            const int64_t* keys, const int64_t* offsets, int64_t nnz,
                                            int32_t insert_missing, float* out, uint8_t* hit_mask, void* ws,
                                            size_t ws_bytes, void* stream, void* results_ready_event) {
  if (!results_ready_event) return fail(HCTR_E_NULL_PTR, "results_ready_event is NULL");
  return cache_query_impl(c, kWhole, batch, num_slots, keys, offsets, nnz, insert_missing, out, true, hit_mask,
                          nullptr, nullptr, ws, ws_bytes, stream, static_cast<hipEvent_t>(results_ready_event));
}

HCTR_API hctr_status hctr_cache_query_hits(hctr_cache* c, int64_t batch, int32_t num_slots, const int64_t* keys,
                                           const int64_t* offsets, int64_t nnz, float* out, uint8_t* hit_mask,
                                           uint32_t* miss_positions, uint32_t* n_missing, void* ws,
                                           size_t ws_bytes, void* stream, void* hits_ready_event) {
  return cache_query_impl(c, kHitsPhase, batch, num_slots, keys, offsets, nnz, 0, out, true, hit_mask,
                          miss_positions, n_missing, ws, ws_bytes, stream,
                          static_cast<hipEvent_t>(hits_ready_event));
}

HCTR_API hctr_status hctr_cache_query_complete(hctr_cache* c, int64_t batch, int32_t num_slots,
                                               const int64_t* keys, const int64_t* offsets, int64_t nnz,
                                               int32_t insert_missing, float* out, void* ws, size_t ws_bytes,
                                               void* stream) {
  return cache_query_impl(c, kMissPhase, batch, num_slots, keys, offsets, nnz, insert_missing, out, true, nullptr,
                          nullptr, nullptr, ws, ws_bytes, stream, nullptr);
}

HCTR_API hctr_status hctr_cache_insert(hctr_cache* c, const int64_t* keys, int64_t n, void* ws, size_t ws_bytes,
                                       void* stream) {
  return cache_query_impl(c, kWhole, n, 1, keys, nullptr, n, 1, nullptr, false, nullptr, nullptr, nullptr, ws,
                          ws_bytes, stream, nullptr);
}

HCTR_API hctr_status hctr_cache_update(hctr_cache* c, const int64_t* keys, const float* rows, int64_t n, void* ws,
                                       size_t ws_bytes, void* stream_) {
  if (!c) return fail(HCTR_E_NULL_PTR, "cache is NULL");
  if (n < 0 || n >= (1ll << 31)) return fail(HCTR_E_INVALID_ARG, "n %lld outside 0..2^31-1", (long long)n);
  if (n == 0) return HCTR_OK;
  if (!keys || !rows) return fail(HCTR_E_NULL_PTR, "keys / rows is NULL");
  if ((uintptr_t)rows % 16 != 0) return fail(HCTR_E_INVALID_ARG, "rows must be 16-byte aligned");
  hctr_cache general = *c;
  general.small_max_keys = 0;   // update always uses the general workspace layout
  const CacheWsLayout L = cache_ws_layout(&general, n);
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < L.total) return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L.total);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  char* w = static_cast<char*>(ws);
  HashWsHeader* ws_hdr = reinterpret_cast<HashWsHeader*>(w + L.header);
  uint32_t* line_of = reinterpret_cast<uint32_t*>(w + L.line_of);
  int64_t* keys_rev = reinterpret_cast<int64_t*>(w + L.new_key);
  DedupBuffers B{reinterpret_cast<uint32_t*>(w + L.flag),
                 reinterpret_cast<uint32_t*>(w + L.idx),
                 reinterpret_cast<uint32_t*>(w + L.miss_pos),
                 reinterpret_cast<uint32_t*>(w + L.scr_slot),
                 reinterpret_cast<uint32_t*>(w + L.first),
                 reinterpret_cast<uint32_t*>(w + L.rank),
                 reinterpret_cast<uint32_t*>(w + L.scan_tmp),
                 reinterpret_cast<uint32_t*>(w + L.scratch),
                 L.scratch_cap_max,
                 &ws_hdr->n_miss,
                 &ws_hdr->n_new,
                 nullptr};
  const uint32_t nn = (uint32_t)n;
  const u64* tags = reinterpret_cast<const u64*>(c->storage + c->off_tags);
  float* data = reinterpret_cast<float*>(c->storage + c->off_data);
#define CALL(W)                                                                                               \
  hipLaunchKernelGGL((cache_update_probe<W>),                                                                 \
                     dim3((uint32_t)std::min<int64_t>(ceil_div((int64_t)nn * W, 256), 2048)), dim3(256), 0,   \
                     stream, tags, make_set_div(c->num_sets), keys, nn, keys_rev, line_of, B.flag)
  HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
  HCTR_TRY(dedup_first_appearance(keys_rev, nn, B, stream));
  int lpr = pow2_ceil((int)ceil_div(c->dim, 4));
  lpr = lpr < 4 ? 4 : (lpr > 64 ? 64 : lpr);
#define CALL(LL)                                                                                              \
  hipLaunchKernelGGL((cache_update_copy<LL>),                                                                 \
                     dim3((uint32_t)std::min<int64_t>(ceil_div((int64_t)nn * LL, 256), 4096)), dim3(256), 0,  \
                     stream, data, (int)c->dim, (const HashWsHeader*)ws_hdr, (const uint32_t*)B.miss_pos,     \
                     (const uint32_t*)B.first, (const uint32_t*)line_of, rows, nn)
  HCTR_BY_LPR(lpr, CALL)
#undef CALL
  return launch_status("hctr_cache_update");
}

HCTR_API hctr_status hctr_cache_refresh(hctr_cache* c, void* stream) {
  if (!c) return fail(HCTR_E_NULL_PTR, "cache is NULL");
  const uint64_t lines = (uint64_t)c->num_sets * c->ways;
  int lpr = pow2_ceil((int)ceil_div(c->dim, 4));
  lpr = lpr < 4 ? 4 : (lpr > 64 ? 64 : lpr);
#define CALL(LL)                                                                                              \
  hipLaunchKernelGGL((cache_refresh_lines<LL>),                                                               \
                     dim3((uint32_t)std::min<int64_t>(ceil_div((int64_t)lines * LL, 256), 8192)), dim3(256),  \
                     0, static_cast<hipStream_t>(stream), reinterpret_cast<const u64*>(c->storage + c->off_tags), \
                     reinterpret_cast<float*>(c->storage + c->off_data), c->host_table, (int)c->dim, lines)
  HCTR_BY_LPR(lpr, CALL)
#undef CALL
  return launch_status("hctr_cache_refresh");
}

HCTR_API hctr_status hctr_cache_stats(hctr_cache* c, void* stream, int64_t stats[6]) {
  if (!c || !stats) return fail(HCTR_E_NULL_PTR, "NULL argument");
  int64_t head[7];   // the six statistics and the word that holds the call count
  HCTR_TRY_HIP(hipMemcpyAsync(head, c->storage, sizeof(head), hipMemcpyDeviceToHost,
                              static_cast<hipStream_t>(stream)));
  HCTR_TRY_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  for (int i = 0; i < 6; ++i) stats[i] = head[i];
  stats[2] = stats[0] - stats[1];   // every queried key is a hit or a miss
  c->epoch = (uint32_t)(uint64_t)head[6];   // replays of captured calls advance the device's count only
  return HCTR_OK;
}

HCTR_API hctr_status hctr_cache_state_view(hctr_cache* c, const uint64_t** tags, const uint32_t** stamps,
                                           const float** data) {
  if (!c) return fail(HCTR_E_NULL_PTR, "cache is NULL");
  if (tags) *tags = reinterpret_cast<const uint64_t*>(c->storage + c->off_tags);
  if (stamps) *stamps = reinterpret_cast<const uint32_t*>(c->storage + c->off_stamps);
  if (data) *data = reinterpret_cast<const float*>(c->storage + c->off_data);
  return HCTR_OK;
}

HCTR_API void hctr_cache_destroy(hctr_cache* c) { delete c; }
