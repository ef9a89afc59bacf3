// Inference embedding cache: set-associative tags probed by groups of `ways` lanes, pooled gather
// that reads hits from HBM and misses straight from the pinned host table, and a fully parallel
// insertion that reproduces "insert distinct missing keys in first-appearance order, LRU victim per
// set at call granularity".
//
// Insertion without a sequential pass: the victims a set can give up in one call are a fixed list
// once the call's hits are stamped (empty ways by index, then untouched ways by (stamp, way)),
// because an inserted way is stamped with the current epoch and cannot be chosen again.  So the
// k-th distinct missing key of a set (in first-appearance order) takes the k-th entry of that
// list, or is skipped when the list is shorter.  The per-set order comes from a stable radix sort
// of (set, first-appearance index) pairs.
#include "common.h"
#include "rowvec.h"
#include "hash_internal.h"

struct hctr_cache {
  char* storage;
  int64_t num_sets;
  int32_t ways, dim;
  const float* host_table;
  int64_t host_rows;
  size_t off_tags, off_stamps, off_data;
};

namespace hctr {

typedef unsigned long long u64;
constexpr uint32_t kNoLine = 0xFFFFFFFFu;

struct CacheHeader {  // first 256 bytes of the cache storage
  u64 stats[6];       // queries, hits, (misses = queries - hits, filled in on the host), inserts, evictions, skipped inserts
  uint32_t epoch;
  uint32_t pad[51];
};
static_assert(sizeof(CacheHeader) == 256, "header is one 256-byte block");

__device__ __forceinline__ u64 set_of(u64 key, u64 num_sets) {
  u64 x = key * 0x9E3779B97F4A7C15ull;
  x ^= x >> 32;
  return x % num_sets;
}

__global__ __launch_bounds__(256) void cache_clear(u64* tags, uint32_t* stamps, uint64_t n_lines,
                                                   CacheHeader* hdr) {
  const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (i < n_lines) { tags[i] = kEmptyKey; stamps[i] = 0u; }
  if (i < 6) hdr->stats[i] = 0;
  if (i == 0) hdr->epoch = 0;
}

__global__ void cache_begin(CacheHeader* hdr, HashWsHeader* ws_hdr, u64 nnz) {
  if (threadIdx.x == 0) {
    hdr->epoch += 1;
    hdr->stats[0] += nnz;
    ws_hdr->n_miss = 0;
    ws_hdr->n_new = 0;
  }
}

// Classify every key against the tags as they stand (nothing writes tags in this kernel).  A group
// of WAYS lanes compares one tag per lane; each group takes kProbeKeys consecutive keys so that
// their tag loads are in flight together, and a block reports its hits with a single atomic
// (one atomic per wave on one address would serialise hundreds of thousands of them).
constexpr int kProbeKeys = 8;

template <int WAYS>
__global__ __launch_bounds__(256) void cache_probe(const u64* __restrict__ tags,
                                                   uint32_t* __restrict__ stamps, u64 num_sets,
                                                   int64_t host_rows, CacheHeader* hdr,
                                                   const int64_t* __restrict__ keys, uint32_t nnz,
                                                   uint32_t* __restrict__ line_of,
                                                   uint8_t* __restrict__ hit_mask,
                                                   uint32_t* __restrict__ miss_flag) {
  __shared__ uint32_t block_hits;
  if (threadIdx.x == 0) block_hits = 0;
  __syncthreads();
  const uint32_t group = (blockIdx.x * 256u + threadIdx.x) / WAYS;
  const int way = threadIdx.x % WAYS;
  const int lane = threadIdx.x & 63;
  constexpr uint64_t kGroupOnes = WAYS == 64 ? ~0ull : ((1ull << (WAYS & 63)) - 1ull);
  const uint64_t gmask = kGroupOnes << (lane - way);
  const uint32_t epoch = hdr->epoch;
  const uint32_t i0 = group * kProbeKeys;

  int64_t key[kProbeKeys];
  u64 tag[kProbeKeys];
  u64 slot[kProbeKeys];
#pragma unroll
  for (int j = 0; j < kProbeKeys; ++j) key[j] = (i0 + j < nnz) ? keys[i0 + j] : -1;
#pragma unroll
  for (int j = 0; j < kProbeKeys; ++j) {
    slot[j] = key[j] >= 0 ? set_of((u64)key[j], num_sets) * WAYS + way : 0;
    tag[j] = key[j] >= 0 ? tags[slot[j]] : kEmptyKey;
  }
  uint32_t hits = 0;
#pragma unroll
  for (int j = 0; j < kProbeKeys; ++j) {
    const bool match = key[j] >= 0 && tag[j] == (u64)key[j];
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
  if (hits) atomicAdd(&block_hits, hits);
  __syncthreads();
  if (threadIdx.x == 0 && block_hits) atomicAdd(&hdr->stats[1], (u64)block_hits);
}

// Pooled gather, one wave per bag: hits from the cache lines in HBM, misses from the host table.
template <int LPR, int U>
__global__ __launch_bounds__(256) void cache_gather(const float* __restrict__ data,
                                                    const float* __restrict__ host_table,
                                                    int64_t host_rows, int D,
                                                    const int64_t* __restrict__ keys,
                                                    const uint32_t* __restrict__ line_of,
                                                    const int64_t* __restrict__ offsets, int64_t hotness,
                                                    uint32_t n_bags, float* __restrict__ out) {
  constexpr int G = 64 / LPR;
  __shared__ float part[4][(G > 1 ? (G - 1) : 1) * LPR * 4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane / LPR, sub = lane % LPR;
  const int col = blockIdx.y * (LPR * 4) + sub * 4;
  const bool active = col < D;
  const uint32_t bag = blockIdx.x * 4u + wave;
  const bool live = bag < n_bags;
  int64_t b0 = 0, b1 = 0;
  if (live) {
    b0 = offsets ? offsets[bag] : (int64_t)bag * hotness;
    b1 = offsets ? offsets[bag + 1] : (int64_t)(bag + 1) * hotness;
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int64_t j = b0 + g; j < b1; j += G * U) {
    const float* src[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t jj = j + u * G;
      src[u] = nullptr;
      if (jj < b1) {
        const uint32_t line = line_of[jj];
        if (line != kNoLine) {
          src[u] = data + (int64_t)line * D;
        } else {
          const int64_t k = keys[jj];
          if (k >= 0 && k < host_rows) src[u] = host_table + k * D;
        }
      }
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
      float* p = &part[wave][((g - 1) * LPR + sub) * 4];
      p[0] = acc.x; p[1] = acc.y; p[2] = acc.z; p[3] = acc.w;
    }
    __syncthreads();
    if (g == 0) {
#pragma unroll
      for (int gg = 1; gg < G; ++gg) {
        const float* p = &part[wave][((gg - 1) * LPR + sub) * 4];
        acc.x += p[0]; acc.y += p[1]; acc.z += p[2]; acc.w += p[3];
      }
    }
  }
  if (live && g == 0 && active) {
    const float v[4] = {acc.x, acc.y, acc.z, acc.w};
    store_stream<4>(out + (int64_t)bag * D + col, v);
  }
}

// Distinct missing keys, in first-appearance order q = 0..n_new-1: key, and (set, q) sort pairs.
__global__ __launch_bounds__(256) void cache_list_new(const HashWsHeader* hdr,
                                                      const int64_t* __restrict__ keys,
                                                      const uint32_t* __restrict__ miss_pos,
                                                      const uint32_t* __restrict__ first,
                                                      const uint32_t* __restrict__ rank, u64 num_sets,
                                                      u64* __restrict__ new_key,
                                                      u64* __restrict__ sort_kv) {
  const uint32_t m = blockIdx.x * 256u + threadIdx.x;
  if (m >= hdr->n_miss || !first[m]) return;
  const uint32_t q = rank[m];
  const u64 key = (u64)keys[miss_pos[m]];
  new_key[q] = key;
  sort_kv[q] = (set_of(key, num_sets) << 32) | (u64)q;   // sorted by set, payload = first-appearance index
}

// One group of WAYS lanes per sorted position; the group at the start of a set's run places the
// whole run.  dst[q] = cache line that key q goes to, or kNoLine when its insert is skipped.
template <int WAYS>
__global__ __launch_bounds__(256) void cache_place(u64* __restrict__ tags, uint32_t* __restrict__ stamps,
                                                   CacheHeader* hdr, const HashWsHeader* ws_hdr,
                                                   const u64* __restrict__ skv,
                                                   const u64* __restrict__ new_key,
                                                   uint32_t* __restrict__ dst) {
  __shared__ uint32_t blk_stats[3];
  if (threadIdx.x < 3) blk_stats[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t j = (blockIdx.x * 256u + threadIdx.x) / WAYS;
  const int way = threadIdx.x % WAYS;
  const uint32_t n_new = ws_hdr->n_new;
  const uint32_t set = j < n_new ? (uint32_t)(skv[j] >> 32) : 0u;
  const bool leader = j < n_new && !(j > 0 && (uint32_t)(skv[j - 1] >> 32) == set);  // first of its set
  if (leader) {
    const uint32_t epoch = hdr->epoch;
    const uint64_t line = (uint64_t)set * WAYS + way;
    const u64 tag = tags[line];
    const uint32_t stamp = stamps[line];
    // order key of this way in the set's victim list; ways used in this call are not in the list
    const bool empty = tag == kEmptyKey;
    const bool eligible = empty || stamp < epoch;
    const u64 okey = !eligible ? ~0ull : (empty ? (u64)way : (((u64)stamp + 1ull) << 8) | (u64)way);
    uint32_t pos = 0, n_elig = 0;
  #pragma unroll
    for (int w = 0; w < WAYS; ++w) {
      const u64 other = (u64)__shfl((long long)okey, w, WAYS);
      pos += other < okey ? 1u : 0u;
      n_elig += other != ~0ull ? 1u : 0u;
    }
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
    // evicted is per lane; add it up over the group
  #pragma unroll
    for (int d = WAYS / 2; d >= 1; d >>= 1) evicted += __shfl_xor(evicted, d, WAYS);
    if (way == 0) {
      if (inserted) atomicAdd(&blk_stats[0], inserted);
      if (evicted) atomicAdd(&blk_stats[1], evicted);
      if (skipped) atomicAdd(&blk_stats[2], skipped);
    }
  }
  __syncthreads();
  if (threadIdx.x < 3 && blk_stats[threadIdx.x]) atomicAdd(&hdr->stats[3 + threadIdx.x], (u64)blk_stats[threadIdx.x]);
}

// Copy the rows of the placed keys from the host table into their cache lines.
template <int LPR>
__global__ __launch_bounds__(256) void cache_fill(float* __restrict__ data,
                                                  const float* __restrict__ host_table, int D,
                                                  const HashWsHeader* ws_hdr,
                                                  const u64* __restrict__ new_key,
                                                  const uint32_t* __restrict__ dst) {
  const uint32_t q = (blockIdx.x * 256u + threadIdx.x) / LPR;
  const int sub = threadIdx.x % LPR;
  if (q >= ws_hdr->n_new) return;
  const uint32_t line = dst[q];
  if (line == kNoLine) return;
  const float* src = host_table + (int64_t)new_key[q] * D;
  float* to = data + (int64_t)line * D;
  for (int col = sub * 4; col < D; col += LPR * 4) store4(to + col, load4(src + col));
}

struct CacheWsLayout {
  size_t header, line_of, flag, idx, miss_pos, scr_slot, first, rank, scan_tmp, scratch, new_key, kv0, kv1,
      hist, aux, dst, total;
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
  L.line_of = at(n * 4); L.flag = at(n * 4); L.idx = at(n * 4); L.miss_pos = at(n * 4);
  L.scr_slot = at(n * 4); L.first = at(n * 4); L.rank = at(n * 4);
  L.scan_tmp = at(scan_tmp_count((uint32_t)n) * 4);
  L.scratch_cap_max = dedup_scratch_capacity((uint32_t)n);
  L.scratch = at((size_t)L.scratch_cap_max * 16);
  L.new_key = at(n * 8);
  L.kv0 = at(n * 8); L.kv1 = at(n * 8);
  L.hist = at(L.sort.hist_count * 4);
  L.aux = at(L.sort.aux_count * 4);
  L.dst = at(n * 4);
  L.total = cv.off;
  return L;
}

template <int WAYS>
static void launch_probe(const hctr_cache* c, const int64_t* keys, uint32_t nnz, uint32_t* line_of,
                         uint8_t* hit_mask, uint32_t* miss_flag, hipStream_t stream) {
  hipLaunchKernelGGL((cache_probe<WAYS>), dim3((uint32_t)ceil_div(ceil_div((int64_t)nnz, kProbeKeys) * WAYS, 256)), dim3(256), 0,
                     stream, reinterpret_cast<const u64*>(c->storage + c->off_tags),
                     reinterpret_cast<uint32_t*>(c->storage + c->off_stamps), (u64)c->num_sets,
                     c->host_rows, reinterpret_cast<CacheHeader*>(c->storage), keys, nnz, line_of,
                     hit_mask, miss_flag);
}

template <int WAYS>
static void launch_place(const hctr_cache* c, const HashWsHeader* ws_hdr, uint32_t n_max,
                         const u64* skv, const u64* new_key, uint32_t* dst, hipStream_t stream) {
  hipLaunchKernelGGL((cache_place<WAYS>), dim3((uint32_t)ceil_div((int64_t)n_max * WAYS, 256)), dim3(256),
                     0, stream, reinterpret_cast<u64*>(c->storage + c->off_tags),
                     reinterpret_cast<uint32_t*>(c->storage + c->off_stamps),
                     reinterpret_cast<CacheHeader*>(c->storage), ws_hdr, skv, new_key, dst);
}

template <int LPR>
static void launch_gather(const hctr_cache* c, const int64_t* keys, const uint32_t* line_of,
                          const int64_t* offsets, int64_t hotness, uint32_t n_bags, float* out,
                          hipStream_t stream) {
  dim3 grid((uint32_t)ceil_div(n_bags, 4), (uint32_t)ceil_div(c->dim, LPR * 4));
  hipLaunchKernelGGL((cache_gather<LPR, 4>), grid, dim3(256), 0, stream,
                     reinterpret_cast<const float*>(c->storage + c->off_data), c->host_table, c->host_rows,
                     (int)c->dim, keys, line_of, offsets, hotness, n_bags, out);
}

template <int LPR>
static void launch_fill(const hctr_cache* c, const HashWsHeader* ws_hdr, uint32_t n_max, const u64* new_key,
                        const uint32_t* dst, hipStream_t stream) {
  hipLaunchKernelGGL((cache_fill<LPR>), dim3((uint32_t)ceil_div((int64_t)n_max * LPR, 256)), dim3(256), 0,
                     stream, reinterpret_cast<float*>(c->storage + c->off_data), c->host_table, (int)c->dim,
                     ws_hdr, new_key, dst);
}

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
  if ((uint64_t)num_sets * ways > 0xFFFFFFFEull) return false;
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

HCTR_API size_t hctr_cache_workspace_bytes(const hctr_cache* cache, int64_t nnz_max) {
  if (!cache || nnz_max < 0 || nnz_max >= (1ll << 31)) return 0;
  return cache_ws_layout(cache, nnz_max).total;
}

HCTR_API hctr_status hctr_cache_query(hctr_cache* c, int64_t batch, int32_t num_slots, const int64_t* keys,
                                      const int64_t* offsets, int64_t nnz, int32_t insert_missing,
                                      float* out, uint8_t* hit_mask, void* ws, size_t ws_bytes,
                                      void* stream_) {
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
  if (n_bags == 0) {
    if (nnz != 0) return fail(HCTR_E_INVALID_ARG, "nnz must be 0 when there are no bags");
    return HCTR_OK;
  }
  if (!out) return fail(HCTR_E_NULL_PTR, "out is NULL");
  if (nnz > 0 && !keys) return fail(HCTR_E_NULL_PTR, "keys is NULL");
  if ((uintptr_t)out % 16 != 0) return fail(HCTR_E_INVALID_ARG, "out must be 16-byte aligned");
  const CacheWsLayout L = cache_ws_layout(c, nnz);
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < L.total) return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L.total);

  hipStream_t stream = static_cast<hipStream_t>(stream_);
  char* w = static_cast<char*>(ws);
  HashWsHeader* ws_hdr = reinterpret_cast<HashWsHeader*>(w + L.header);
  uint32_t* line_of = reinterpret_cast<uint32_t*>(w + L.line_of);
  uint32_t* flag = reinterpret_cast<uint32_t*>(w + L.flag);
  const uint32_t n = (uint32_t)nnz;

  hipLaunchKernelGGL(cache_begin, dim3(1), dim3(64), 0, stream, reinterpret_cast<CacheHeader*>(c->storage), ws_hdr, (u64)nnz);
  if (n > 0) {
#define CALL(W) launch_probe<W>(c, keys, n, line_of, hit_mask, insert_missing ? flag : nullptr, stream)
    HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
  }
  int lpr = pow2_ceil((int)ceil_div(c->dim, 4));
  lpr = lpr < 4 ? 4 : (lpr > 64 ? 64 : lpr);
#define CALL(LL) launch_gather<LL>(c, keys, line_of, offsets, hotness, (uint32_t)n_bags, out, stream)
  HCTR_BY_LPR(lpr, CALL)
#undef CALL
  if (insert_missing && n > 0) {
    DedupBuffers B{flag,
                   reinterpret_cast<uint32_t*>(w + L.idx),
                   reinterpret_cast<uint32_t*>(w + L.miss_pos),
                   reinterpret_cast<uint32_t*>(w + L.scr_slot),
                   reinterpret_cast<uint32_t*>(w + L.first),
                   reinterpret_cast<uint32_t*>(w + L.rank),
                   reinterpret_cast<uint32_t*>(w + L.scan_tmp),
                   reinterpret_cast<u64*>(w + L.scratch),
                   L.scratch_cap_max,
                   &ws_hdr->n_miss,
                   &ws_hdr->n_new};
    HCTR_TRY(dedup_first_appearance(keys, n, B, stream));
    u64* new_key = reinterpret_cast<u64*>(w + L.new_key);
    u64* kv[2] = {reinterpret_cast<u64*>(w + L.kv0), reinterpret_cast<u64*>(w + L.kv1)};
    uint32_t* dst = reinterpret_cast<uint32_t*>(w + L.dst);
    hipLaunchKernelGGL(cache_list_new, dim3((uint32_t)ceil_div(n, 256)), dim3(256), 0, stream,
                       (const HashWsHeader*)ws_hdr, keys, (const uint32_t*)B.miss_pos,
                       (const uint32_t*)B.first, (const uint32_t*)B.rank, (u64)c->num_sets, new_key, kv[0]);
    HCTR_TRY(radix_sort_u64(L.sort, &ws_hdr->n_new, reinterpret_cast<uint64_t*>(kv[0]),
                            reinterpret_cast<uint64_t*>(kv[1]), reinterpret_cast<uint32_t*>(w + L.hist),
                            reinterpret_cast<uint32_t*>(w + L.aux), false, stream));
    const u64* skv = kv[L.sort.passes & 1];
#define CALL(W) launch_place<W>(c, ws_hdr, n, skv, new_key, dst, stream)
    HCTR_BY_WAYS(c->ways, CALL)
#undef CALL
#define CALL(LL) launch_fill<LL>(c, ws_hdr, n, new_key, dst, stream)
    HCTR_BY_LPR(lpr, CALL)
#undef CALL
  }
  return launch_status("hctr_cache_query");
}

HCTR_API hctr_status hctr_cache_stats(hctr_cache* c, void* stream, int64_t stats[6]) {
  if (!c || !stats) return fail(HCTR_E_NULL_PTR, "NULL argument");
  HCTR_TRY_HIP(hipMemcpyAsync(stats, c->storage, 6 * sizeof(int64_t), hipMemcpyDeviceToHost,
                              static_cast<hipStream_t>(stream)));
  HCTR_TRY_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  stats[2] = stats[0] - stats[1];   // every queried key is a hit or a miss
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
