// Embedding hash: open addressing over 128-byte buckets of eight {key, row} slots, probed by
// groups of eight lanes (one 16-byte slot per lane, one bucket per group per step, eight keys per
// wave in flight).  Linear probing over buckets; nothing is ever deleted, so an empty slot in a
// bucket ends a search.
//
// Insert-or-find keeps the table's contract "rows are handed out in order of first appearance in
// the call's key array" without any sequential step:
//   1. find every key; flag the misses and compact their positions (scan);
//   2. put the missed keys into a scratch table sized for this call: a slot holds only a position
//      of the call's key array (4 bytes; the key it stands for is keys[position]) and keeps the
//      smallest position of its key (atomicMin) = the key's first appearance;
//   3. flag the first appearances, scan them: rank = how many new keys appear earlier;
//   4. row = size + rank; keys whose row stays below max_rows claim a slot of the main table with a
//      64-bit compare-and-swap and publish the row, the others are rejected;
//   5. every other missed position copies the answer of its key's first appearance.
// The main table only ever holds published keys, so a later search never meets a half-made entry.
#include "hash_internal.h"

namespace hctr {

typedef unsigned long long u64;
typedef u64 u64x2 __attribute__((ext_vector_type(2)));

struct HashHeader {      // first 256 bytes of the hash storage
  u64 size;
  u64 pad[31];
};

__device__ __forceinline__ u64 mix_key(u64 x) {
  x ^= x >> 33;
  x *= 0xD6E8FEB86659FD93ull;
  x ^= x >> 29;
  x *= 0xA24BAED4963EE407ull;
  x ^= x >> 32;
  return x;
}
__device__ __forceinline__ uint32_t bucket_of(u64 key, uint32_t n_buckets) {
  return (uint32_t)(((mix_key(key) >> 32) * (u64)n_buckets) >> 32);
}
__device__ __forceinline__ uint32_t scratch_capacity(uint32_t n_miss) {  // power of two >= 2 * n_miss
  uint32_t want = n_miss < 32u ? 64u : 2u * n_miss;
  return 1u << (32 - __clz(want - 1u));
}
__device__ __forceinline__ uint32_t group_bits(uint64_t ballot) {  // this 8-lane group's votes
  return (uint32_t)(ballot >> (threadIdx.x & 56)) & 0xFFu;
}

__global__ __launch_bounds__(256) void hash_clear(u64x2* slots, uint64_t n_slots, HashHeader* hdr) {
  const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (i < n_slots) slots[i] = u64x2{kEmptyKey, kEmptyKey};
  if (i == 0) hdr->size = 0;
}

// An 8-lane group reads one bucket (8 slots of 16 bytes = one 128-byte line) per probe and works on
// kFindKeys keys at once, so that many independent bucket loads are in flight per wave: the search
// is bound by the latency of random lines, not by bandwidth.
constexpr int kFindKeys = 4;   // find-only call on 3.4 M keys, load 0.8: 0.277 / 0.236 / 0.227 ms with 1 / 2 / 4 (8 and 16: 30 % and 2.5 x slower)
__global__ __launch_bounds__(256) void hash_find(const u64x2* __restrict__ slots, uint32_t n_buckets,
                                                 const int64_t* __restrict__ keys, uint32_t n,
                                                 int64_t* __restrict__ rows,
                                                 uint32_t* __restrict__ miss_flag,
                                                 const HashHeader* __restrict__ table_hdr, int64_t max_rows,
                                                 HashWsHeader* ws_hdr) {
  // A table that already holds max_rows rows rejects every new key: nothing is flagged as missing
  // then, the scans are told to look at no position, and the insertion kernels that follow find an
  // empty list (row -1 is already the answer).
  const bool full = table_hdr != nullptr && table_hdr->size >= (u64)max_rows;
  if (ws_hdr != nullptr && blockIdx.x == 0 && threadIdx.x == 0) ws_hdr->n_scan = full ? 0u : n;
  const uint64_t i0 = (uint64_t)((blockIdx.x * 256u + threadIdx.x) >> 3) * kFindKeys;
  const int sub = threadIdx.x & 7;
  int64_t key[kFindKeys], row[kFindKeys];
  bool searching[kFindKeys];
  uint32_t b[kFindKeys];
#pragma unroll
  for (int u = 0; u < kFindKeys; ++u) {
    key[u] = i0 + u < n ? keys[i0 + u] : -1;
    searching[u] = key[u] >= 0;
    row[u] = -1;
    b[u] = searching[u] ? bucket_of((u64)key[u], n_buckets) : 0u;
  }
  for (uint32_t step = 0; step < n_buckets; ++step) {
    bool any = false;
#pragma unroll
    for (int u = 0; u < kFindKeys; ++u) any |= searching[u];
    if (__ballot(any) == 0) break;
    u64x2 s[kFindKeys];
#pragma unroll
    for (int u = 0; u < kFindKeys; ++u) {
      s[u] = u64x2{kEmptyKey, kEmptyKey};
      if (searching[u]) s[u] = slots[(uint64_t)b[u] * 8u + sub];
    }
#pragma unroll
    for (int u = 0; u < kFindKeys; ++u) {
      const uint32_t hit = group_bits(__ballot(searching[u] && s[u].x == (u64)key[u]));
      const uint32_t hole = group_bits(__ballot(searching[u] && s[u].x == kEmptyKey));
      if (searching[u]) {
        if (hit) {
          const int src = (threadIdx.x & 56) + (__ffs(hit) - 1);
          row[u] = (int64_t)__shfl((long long)s[u].y, src);
          searching[u] = false;
        } else if (hole) {
          searching[u] = false;
        } else {
          b[u] = (b[u] + 1 == n_buckets) ? 0u : b[u] + 1;
        }
      }
    }
  }
  if (sub == 0) {
#pragma unroll
    for (int u = 0; u < kFindKeys; ++u) {
      if (i0 + u < n) {
        rows[i0 + u] = row[u];
        if (miss_flag) miss_flag[i0 + u] = (key[u] >= 0 && row[u] < 0 && !full) ? 1u : 0u;
      }
    }
  }
}

__global__ __launch_bounds__(256) void hash_compact_misses(const uint32_t* __restrict__ flag,
                                                           const uint32_t* __restrict__ idx, uint32_t n,
                                                           uint32_t* __restrict__ miss_pos) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < n && flag[i]) miss_pos[idx[i]] = i;
}

constexpr uint32_t kNoPos = 0xFFFFFFFFu;   // empty scratch slot (positions stay below 2^31)

__global__ __launch_bounds__(256) void scratch_clear(uint32_t* scratch, const HashWsHeader* hdr) {
  const uint32_t cap = scratch_capacity(hdr->n_miss);
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (hdr->n_miss != 0 && i < cap) scratch[i] = kNoPos;
}

// One missed key per lane: claim or join the key's scratch slot, keep the smallest position.  A slot
// holds a position p and stands for the key keys[p]; once claimed it only ever moves to smaller
// positions of the same key, so "keys[slot] == my key" stays true or stays false.
__global__ __launch_bounds__(256) void scratch_insert(uint32_t* scratch, const HashWsHeader* hdr,
                                                      const int64_t* __restrict__ keys,
                                                      const uint32_t* __restrict__ miss_pos,
                                                      uint32_t* __restrict__ scr_slot) {
  const uint32_t m = blockIdx.x * 256u + threadIdx.x;
  const uint32_t n_miss = hdr->n_miss;
  if (m >= n_miss) return;
  const uint32_t cap = scratch_capacity(n_miss);
  const uint32_t pos = miss_pos[m];
  const u64 key = (u64)keys[pos];
  uint32_t s = (uint32_t)(mix_key(key ^ 0x5851F42D4C957F2Dull) >> 16) & (cap - 1);
  for (uint32_t step = 0; step < cap; ++step) {
    // A plain look first: a view (possibly stale) that already shows this key with a position
    // <= pos settles the matter without an atomic.  A hot key repeated a million times would
    // otherwise queue a million atomics on one address (measured: 22 ms for 11.5 M keys of a Zipf
    // pass, under 1 ms with the look).  A new key costs one load and one compare-and-swap.
    uint32_t seen = scratch[s];
    if (seen == kNoPos) {
      seen = atomicCAS(&scratch[s], kNoPos, pos);
      if (seen == kNoPos) { scr_slot[m] = s; return; }   // claimed
    }
    if ((u64)keys[seen] == key) {
      if (seen > pos) atomicMin(&scratch[s], pos);
      scr_slot[m] = s;
      return;
    }
    s = (s + 1) & (cap - 1);
  }
  scr_slot[m] = 0xFFFFFFFFu;  // cannot happen: at most cap/2 distinct keys
}

__global__ __launch_bounds__(256) void first_flags(const uint32_t* __restrict__ scratch,
                                                   const HashWsHeader* hdr,
                                                   const uint32_t* __restrict__ miss_pos,
                                                   const uint32_t* __restrict__ scr_slot, uint32_t n,
                                                   uint32_t* __restrict__ first) {
  const uint32_t m = blockIdx.x * 256u + threadIdx.x;
  if (m >= n || m >= hdr->n_miss) return;   // first[] is read (and scanned) for m < n_miss only
  const uint32_t s = scr_slot[m];
  first[m] = (s != 0xFFFFFFFFu && scratch[s] == miss_pos[m]) ? 1u : 0u;
}

// One new key per lane: assign the row, claim a slot in the main table, publish.  The key is known to
// be absent, so the lane only needs an empty slot: it reads the 8 keys of the bucket, tries the
// holes in slot order (a CAS that fails means another new key took the hole: next hole) and moves
// on to the next bucket when none is left.  (A group of 8 lanes per key, as in the search, made
// this kernel latency-bound: eight times the waves for the same dependent load -> CAS -> store.)
__global__ __launch_bounds__(256) void hash_insert_new(u64* slots /* {key,row} pairs */,
                                                       uint32_t n_buckets, const HashHeader* table_hdr,
                                                       int64_t max_rows, int64_t* __restrict__ rows,
                                                       const HashWsHeader* hdr,
                                                       const int64_t* __restrict__ keys,
                                                       const uint32_t* __restrict__ miss_pos,
                                                       const uint32_t* __restrict__ first,
                                                       const uint32_t* __restrict__ rank) {
  const uint32_t m = blockIdx.x * 256u + threadIdx.x;
  if (m >= hdr->n_miss || first[m] == 0) return;
  const u64 key = (u64)keys[miss_pos[m]];
  int64_t row = (int64_t)table_hdr->size + (int64_t)rank[m];
  bool placed = false;
  if (row < max_rows) {
    uint32_t b = bucket_of(key, n_buckets);
    for (uint32_t step = 0; step < n_buckets && !placed; ++step) {   // ends: the table keeps 20 % of its slots empty
      const u64x2* line = reinterpret_cast<const u64x2*>(slots) + (uint64_t)b * 8u;
      u64 seen[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) seen[j] = line[j].x;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (!placed && seen[j] == kEmptyKey) {
          u64* slot = &slots[2ull * ((uint64_t)b * 8u + j)];
          if (atomicCAS(slot, kEmptyKey, key) == kEmptyKey) {
            slot[1] = (u64)row;
            placed = true;
          }
        }
      }
      b = (b + 1 == n_buckets) ? 0u : b + 1;
    }
  }
  rows[miss_pos[m]] = placed ? row : -1;   // the answer, read by the key's other positions afterwards
}

// Every missed position that is not its key's first appearance copies the answer of the first one
// (the scratch slot still holds that position; first appearances were answered by hash_insert_new
// and are not written here, so the reads and writes of this kernel never meet).
__global__ __launch_bounds__(256) void hash_resolve(const uint32_t* __restrict__ scratch, HashWsHeader* hdr,
                                                    HashHeader* table_hdr, int64_t max_rows,
                                                    const uint32_t* __restrict__ miss_pos,
                                                    const uint32_t* __restrict__ scr_slot,
                                                    const uint32_t* __restrict__ first,
                                                    int64_t* rows) {
  const uint32_t m = blockIdx.x * 256u + threadIdx.x;
  if (m < hdr->n_miss && !first[m]) {
    const uint32_t s = scr_slot[m];
    rows[miss_pos[m]] = s != 0xFFFFFFFFu ? rows[scratch[s]] : -1;
  }
  if (m == 0) {
    const u64 grown = table_hdr->size + hdr->n_new;
    table_hdr->size = grown < (u64)max_rows ? grown : (u64)max_rows;
  }
}


// Steps 1b-3 above, shared with the cache's insertion path: from per-position miss flags to, per
// missed position m (in position order), the scratch slot of its key, whether it is the key's first
// appearance, and the rank of that first appearance among all first appearances.
hctr_status dedup_first_appearance(const int64_t* keys, uint32_t n, const DedupBuffers& B,
                                   hipStream_t stream) {
  const uint32_t nb = (uint32_t)ceil_div(n, 256);
  const HashWsHeader* hdr = reinterpret_cast<const HashWsHeader*>(B.n_miss);
  HCTR_TRY(exclusive_scan_u32(B.flag, B.idx, n, B.scan_tmp, B.n_miss, stream, B.n_scan));
  hipLaunchKernelGGL(hash_compact_misses, dim3(nb), dim3(256), 0, stream, (const uint32_t*)B.flag,
                     (const uint32_t*)B.idx, n, B.miss_pos);
  hipLaunchKernelGGL(scratch_clear, dim3((uint32_t)ceil_div(B.scratch_cap_max, 256)), dim3(256), 0, stream,
                     B.scratch, hdr);
  hipLaunchKernelGGL(scratch_insert, dim3(nb), dim3(256), 0, stream, B.scratch, hdr, keys,
                     (const uint32_t*)B.miss_pos, B.scr_slot);
  hipLaunchKernelGGL(first_flags, dim3(nb), dim3(256), 0, stream, (const uint32_t*)B.scratch, hdr,
                     (const uint32_t*)B.miss_pos, (const uint32_t*)B.scr_slot, n, B.first);
  HCTR_TRY(exclusive_scan_u32(B.first, B.rank, n, B.scan_tmp, B.n_new, stream, B.n_miss));   // first[m] is used for m < n_miss only
  return launch_status("dedup_first_appearance");
}

uint32_t dedup_scratch_capacity(uint32_t n_max) {
  uint64_t cap = 64;
  while (cap < 2ull * (n_max > 0 ? n_max : 1)) cap <<= 1;
  return (uint32_t)cap;
}

struct HashWsLayout {
  size_t header, flag, idx, miss_pos, scr_slot, first, rank, scan_tmp, scratch, total;
  uint32_t scratch_cap_max;
};

static HashWsLayout hash_ws_layout(int64_t n_max) {
  HashWsLayout L{};
  const size_t n = (size_t)(n_max > 0 ? n_max : 1);
  Carver c(nullptr);
  auto at = [&](size_t bytes) { size_t o = c.off; c.take<char>(bytes); return o; };
  L.header = at(sizeof(HashWsHeader));
  L.flag = at(n * 4); L.idx = at(n * 4); L.miss_pos = at(n * 4); L.scr_slot = at(n * 4);
  L.first = at(n * 4); L.rank = at(n * 4);
  L.scan_tmp = at(scan_tmp_count((uint32_t)n) * 4);
  L.scratch_cap_max = dedup_scratch_capacity((uint32_t)n);
  L.scratch = at((size_t)L.scratch_cap_max * 4);
  L.total = c.off;
  return L;
}

size_t hash_ws_bytes(int64_t n_max) { return hash_ws_layout(n_max).total; }

hctr_status hash_lookup(hctr_hash* h, const int64_t* keys, int64_t n64, int insert, int64_t* rows,
                        void* ws, size_t ws_bytes, hipStream_t stream) {
  if (n64 == 0) return HCTR_OK;
  const uint32_t n = (uint32_t)n64;
  const u64x2* slots = reinterpret_cast<const u64x2*>(h->slots);
  const uint32_t find_blocks = (uint32_t)ceil_div(ceil_div((int64_t)n, kFindKeys) * 8, 256);
  if (!insert) {
    hipLaunchKernelGGL(hash_find, dim3(find_blocks), dim3(256), 0, stream, slots, h->n_buckets, keys, n,
                       rows, (uint32_t*)nullptr, (const HashHeader*)nullptr, (int64_t)0, (HashWsHeader*)nullptr);
    return launch_status("hash_find");
  }
  const HashWsLayout L = hash_ws_layout(n64);
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < L.total) return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L.total);
  char* w = static_cast<char*>(ws);
  HashWsHeader* hdr = reinterpret_cast<HashWsHeader*>(w + L.header);
  HashHeader* thdr = reinterpret_cast<HashHeader*>(reinterpret_cast<char*>(h->slots) - sizeof(HashHeader));
  uint32_t* flag = reinterpret_cast<uint32_t*>(w + L.flag);
  uint32_t* idx = reinterpret_cast<uint32_t*>(w + L.idx);
  uint32_t* miss_pos = reinterpret_cast<uint32_t*>(w + L.miss_pos);
  uint32_t* scr_slot = reinterpret_cast<uint32_t*>(w + L.scr_slot);
  uint32_t* first = reinterpret_cast<uint32_t*>(w + L.first);
  uint32_t* rank = reinterpret_cast<uint32_t*>(w + L.rank);
  uint32_t* scan_tmp = reinterpret_cast<uint32_t*>(w + L.scan_tmp);
  uint32_t* scratch = reinterpret_cast<uint32_t*>(w + L.scratch);
  const uint32_t nb = (uint32_t)ceil_div(n, 256);

  hipLaunchKernelGGL(hash_find, dim3(find_blocks), dim3(256), 0, stream, slots, h->n_buckets, keys, n, rows, flag,
                     (const HashHeader*)thdr, h->max_rows, hdr);
  DedupBuffers B{flag, idx, miss_pos, scr_slot, first, rank, scan_tmp, scratch, L.scratch_cap_max,
                 &hdr->n_miss, &hdr->n_new, &hdr->n_scan};
  HCTR_TRY(dedup_first_appearance(keys, n, B, stream));
  hipLaunchKernelGGL(hash_insert_new, dim3(nb), dim3(256), 0, stream, h->slots, h->n_buckets,
                     (const HashHeader*)thdr, h->max_rows, rows, (const HashWsHeader*)hdr, keys,
                     (const uint32_t*)miss_pos, (const uint32_t*)first, (const uint32_t*)rank);
  hipLaunchKernelGGL(hash_resolve, dim3(nb), dim3(256), 0, stream, (const uint32_t*)scratch, hdr, thdr,
                     h->max_rows, (const uint32_t*)miss_pos, (const uint32_t*)scr_slot, (const uint32_t*)first, rows);
  return launch_status("hash_lookup");
}

}  // namespace hctr

using namespace hctr;

static uint32_t buckets_for(int64_t capacity) { return (uint32_t)ceil_div(capacity, 8); }

HCTR_API size_t hctr_hash_storage_bytes(int64_t capacity) {
  if (capacity < 64 || capacity > (1ll << 34)) return 0;
  return sizeof(HashHeader) + (size_t)buckets_for(capacity) * 128;
}

HCTR_API hctr_status hctr_hash_create(void* storage, size_t storage_bytes, int64_t capacity,
                                      int64_t max_rows, void* stream, hctr_hash** out) {
  if (!out) return fail(HCTR_E_NULL_PTR, "out is NULL");
  *out = nullptr;
  if (!storage) return fail(HCTR_E_NULL_PTR, "storage is NULL");
  if (capacity < 64 || capacity > (1ll << 34)) return fail(HCTR_E_INVALID_ARG, "capacity %lld outside 64..2^34", (long long)capacity);
  if (max_rows < 1 || (double)max_rows > 0.8 * (double)capacity)
    return fail(HCTR_E_INVALID_ARG, "max_rows %lld outside 1..0.8*capacity", (long long)max_rows);
  if ((uintptr_t)storage % 256 != 0) return fail(HCTR_E_INVALID_ARG, "storage must be 256-byte aligned");
  if (storage_bytes < hctr_hash_storage_bytes(capacity))
    return fail(HCTR_E_INVALID_ARG, "storage has %zu bytes, %zu needed", storage_bytes, hctr_hash_storage_bytes(capacity));
  hctr_hash* h = new hctr_hash();
  h->n_buckets = buckets_for(capacity);
  h->capacity = capacity;
  h->max_rows = max_rows;
  h->size = reinterpret_cast<unsigned long long*>(storage);
  h->slots = reinterpret_cast<unsigned long long*>(static_cast<char*>(storage) + sizeof(HashHeader));
  const uint64_t n_slots = (uint64_t)h->n_buckets * 8;
  hipLaunchKernelGGL(hash_clear, dim3((uint32_t)ceil_div((int64_t)n_slots, 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), reinterpret_cast<u64x2*>(h->slots), n_slots,
                     reinterpret_cast<HashHeader*>(storage));
  hctr_status st = launch_status("hash_clear");
  if (st != HCTR_OK) { delete h; return st; }
  *out = h;
  return HCTR_OK;
}

HCTR_API hctr_status hctr_hash_clear(hctr_hash* hash, void* stream) {
  if (!hash) return fail(HCTR_E_NULL_PTR, "hash is NULL");
  const uint64_t n_slots = (uint64_t)hash->n_buckets * 8;
  hipLaunchKernelGGL(hash_clear, dim3((uint32_t)ceil_div((int64_t)n_slots, 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), reinterpret_cast<u64x2*>(hash->slots), n_slots,
                     reinterpret_cast<HashHeader*>(hash->size));
  return launch_status("hash_clear");
}

HCTR_API size_t hctr_hash_workspace_bytes(int64_t n_max) {
  if (n_max < 0 || n_max >= (1ll << 31)) return 0;
  return hash_ws_bytes(n_max);
}

HCTR_API hctr_status hctr_hash_insert_or_find(hctr_hash* hash, const int64_t* keys, int64_t n,
                                              int32_t insert, int64_t* rows, void* ws, size_t ws_bytes,
                                              void* stream) {
  if (!hash) return fail(HCTR_E_NULL_PTR, "hash is NULL");
  if (n < 0 || n >= (1ll << 31)) return fail(HCTR_E_INVALID_ARG, "n %lld outside 0..2^31-1", (long long)n);
  if (n == 0) return HCTR_OK;
  if (!keys || !rows) return fail(HCTR_E_NULL_PTR, "keys / rows is NULL");
  return hash_lookup(hash, keys, n, insert, rows, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

HCTR_API hctr_status hctr_hash_size(hctr_hash* hash, void* stream, int64_t* size) {
  if (!hash || !size) return fail(HCTR_E_NULL_PTR, "NULL argument");
  unsigned long long v = 0;
  HCTR_TRY_HIP(hipMemcpyAsync(&v, hash->size, sizeof(v), hipMemcpyDeviceToHost, static_cast<hipStream_t>(stream)));
  HCTR_TRY_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  *size = (int64_t)v;
  return HCTR_OK;
}

HCTR_API void hctr_hash_destroy(hctr_hash* hash) { delete hash; }
