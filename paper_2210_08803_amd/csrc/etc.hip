// Embedding training cache staged in host memory: the whole table lives in pinned host memory, the
// rows a training pass needs are loaded on demand into a working table in HBM (addressed through
// the embedding hash), trained there, and written back.  The host link is crossed once per loaded
// row and once per dumped row, by kernels that read / write the pinned memory directly.
#include "common.h"
#include "rowvec.h"
#include "hash_internal.h"

struct hctr_etc {
  hctr_hash* hash;
  float* table;       // device [max_rows, dim]
  float* host;        // pinned host [host_rows, dim]
  int64_t host_rows;
  int32_t dim;
  void* storage;      // device: EtcHeader, then row_keys [max_rows]
};

namespace hctr {

struct EtcHeader {   // first 256 bytes of the storage
  unsigned long long old_size;   // resident keys when the current load call began
  unsigned long long loaded;     // rows loaded, running total
  unsigned long long rejected;   // key occurrences that found no room, running total
  unsigned long long outside;    // key occurrences outside the host table, running total
  unsigned long long pad[28];
};
static_assert(sizeof(EtcHeader) == 256, "header is one 256-byte block");

// Keys outside the host table become -1 (the hash never stores negative keys); remembers how many
// keys were resident before the call.
__global__ __launch_bounds__(256) void etc_filter(const int64_t* __restrict__ keys, uint32_t n, int64_t host_rows,
                                                  int64_t* __restrict__ filtered, EtcHeader* hdr,
                                                  const unsigned long long* size) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i == 0) hdr->old_size = *size;
  bool bad = false;
  if (i < n) {
    const int64_t k = keys[i];
    bad = k < 0 || k >= host_rows;
    filtered[i] = bad ? (int64_t)-1 : k;
  }
  const uint64_t m = __ballot(bad);
  if (m != 0 && (threadIdx.x & 63) == 0) atomicAdd(&hdr->outside, (unsigned long long)__popcll(m));
}

// After the insert: the positions whose key got one of this call's new rows record the key of the
// row (every occurrence of a key writes the same value); rejected occurrences are counted.
__global__ __launch_bounds__(256) void etc_note(const int64_t* __restrict__ filtered, const int64_t* __restrict__ rows,
                                                uint32_t n, EtcHeader* hdr, int64_t* __restrict__ row_keys) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  bool rejected = false;
  if (i < n) {
    const int64_t k = filtered[i], r = rows[i];
    if (r >= (int64_t)hdr->old_size) row_keys[r] = k;
    rejected = k >= 0 && r < 0;
  }
  const uint64_t m = __ballot(rejected);
  if (m != 0 && (threadIdx.x & 63) == 0) atomicAdd(&hdr->rejected, (unsigned long long)__popcll(m));
}

// One new row per group of LPR lanes: host row -> working row.
template <int LPR>
__global__ __launch_bounds__(256) void etc_fetch(const float* __restrict__ host, float* __restrict__ table, int D,
                                                 EtcHeader* hdr, const unsigned long long* size,
                                                 const int64_t* __restrict__ row_keys) {
  const int sub = threadIdx.x % LPR;
  const uint64_t r0 = hdr->old_size, r1 = *size;
  if (blockIdx.x == 0 && threadIdx.x == 0 && r1 > r0) atomicAdd(&hdr->loaded, (unsigned long long)(r1 - r0));
  for (uint64_t r = r0 + (blockIdx.x * 256u + threadIdx.x) / LPR; r < r1; r += (uint64_t)gridDim.x * (256u / LPR)) {
    const float* src = host + row_keys[r] * D;
    float* to = table + r * D;
    for (int col = sub * 4; col < D; col += LPR * 4) store4(to + col, load4(src + col));
  }
}

// One resident row per group of LPR lanes: working row -> host row.
template <int LPR>
__global__ __launch_bounds__(256) void etc_dump(float* __restrict__ host, const float* __restrict__ table, int D,
                                                const unsigned long long* size, const int64_t* __restrict__ row_keys) {
  const int sub = threadIdx.x % LPR;
  const uint64_t r1 = *size;
  for (uint64_t r = (blockIdx.x * 256u + threadIdx.x) / LPR; r < r1; r += (uint64_t)gridDim.x * (256u / LPR)) {
    float* to = host + row_keys[r] * D;
    const float* src = table + r * D;
    for (int col = sub * 4; col < D; col += LPR * 4) store4(to + col, load4(src + col));
  }
}

__global__ void etc_init(EtcHeader* hdr) {
  if (threadIdx.x == 0) { hdr->old_size = 0; hdr->loaded = 0; hdr->rejected = 0; hdr->outside = 0; }
}

static int etc_lpr(int dim) {
  int l = pow2_ceil((int)ceil_div(dim, 4));
  return l < 4 ? 4 : (l > 64 ? 64 : l);
}

template <int LPR>
static void etc_copy(bool dump, const hctr_etc* e, EtcHeader* hdr, const int64_t* row_keys, int64_t rows_hint,
                     hipStream_t stream) {
  const uint32_t blocks = (uint32_t)std::min<int64_t>(std::max<int64_t>(ceil_div(rows_hint * LPR, 256), 1), 4096);
  if (dump)
    hipLaunchKernelGGL((etc_dump<LPR>), dim3(blocks), dim3(256), 0, stream, e->host, (const float*)e->table,
                       (int)e->dim, (const unsigned long long*)e->hash->size, row_keys);
  else
    hipLaunchKernelGGL((etc_fetch<LPR>), dim3(blocks), dim3(256), 0, stream, (const float*)e->host, e->table,
                       (int)e->dim, hdr, (const unsigned long long*)e->hash->size, row_keys);
}

static void etc_copy_dispatch(bool dump, const hctr_etc* e, EtcHeader* hdr, const int64_t* row_keys,
                              int64_t rows_hint, hipStream_t stream) {
  switch (etc_lpr(e->dim)) {
    case 4: etc_copy<4>(dump, e, hdr, row_keys, rows_hint, stream); break;
    case 8: etc_copy<8>(dump, e, hdr, row_keys, rows_hint, stream); break;
    case 16: etc_copy<16>(dump, e, hdr, row_keys, rows_hint, stream); break;
    case 32: etc_copy<32>(dump, e, hdr, row_keys, rows_hint, stream); break;
    default: etc_copy<64>(dump, e, hdr, row_keys, rows_hint, stream); break;
  }
}

}  // namespace hctr

using namespace hctr;

HCTR_API size_t hctr_etc_storage_bytes(int64_t max_rows) {
  if (max_rows < 1 || max_rows > (1ll << 34)) return 0;
  return align_up(sizeof(EtcHeader) + (size_t)max_rows * 8);
}

HCTR_API size_t hctr_etc_workspace_bytes(int64_t n_max) {
  if (n_max < 0 || n_max >= (1ll << 31)) return 0;
  const size_t n = (size_t)(n_max > 0 ? n_max : 1);
  return align_up(n * 8) + align_up(n * 8) + hash_ws_bytes(n_max);   // filtered keys, rows, hash workspace
}

HCTR_API hctr_status hctr_etc_create(hctr_hash* hash, void* table, int32_t dim, float* host_table,
                                     int64_t host_rows, void* storage, size_t storage_bytes, void* stream,
                                     hctr_etc** out) {
  if (!out) return fail(HCTR_E_NULL_PTR, "out is NULL");
  *out = nullptr;
  if (!hash || !table || !host_table || !storage) return fail(HCTR_E_NULL_PTR, "NULL argument");
  if (dim < 4 || dim % 4 != 0) return fail(HCTR_E_INVALID_ARG, "dim %d must be a positive multiple of 4", dim);
  if (host_rows < 1) return fail(HCTR_E_INVALID_ARG, "host_rows %lld < 1", (long long)host_rows);
  if ((uintptr_t)table % 16 != 0 || (uintptr_t)host_table % 16 != 0)
    return fail(HCTR_E_INVALID_ARG, "table and host_table must be 16-byte aligned");
  if ((uintptr_t)storage % 256 != 0) return fail(HCTR_E_INVALID_ARG, "storage must be 256-byte aligned");
  if (storage_bytes < hctr_etc_storage_bytes(hash->max_rows))
    return fail(HCTR_E_INVALID_ARG, "storage has %zu bytes, %zu needed", storage_bytes,
                hctr_etc_storage_bytes(hash->max_rows));
  hipLaunchKernelGGL(etc_init, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                     static_cast<EtcHeader*>(storage));
  HCTR_TRY(launch_status("etc_init"));
  hctr_etc* e = new hctr_etc();
  e->hash = hash; e->table = static_cast<float*>(table); e->host = host_table; e->host_rows = host_rows;
  e->dim = dim; e->storage = storage;
  *out = e;
  return HCTR_OK;
}

HCTR_API void hctr_etc_destroy(hctr_etc* etc) { delete etc; }

HCTR_API hctr_status hctr_etc_load(hctr_etc* etc, const int64_t* keys, int64_t n, int64_t* rows, void* ws,
                                   size_t ws_bytes, void* stream_) {
  if (!etc) return fail(HCTR_E_NULL_PTR, "etc is NULL");
  if (n < 0 || n >= (1ll << 31)) return fail(HCTR_E_INVALID_ARG, "n %lld outside 0..2^31-1", (long long)n);
  if (n == 0) return HCTR_OK;
  if (!keys) return fail(HCTR_E_NULL_PTR, "keys is NULL");
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < hctr_etc_workspace_bytes(n))
    return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, hctr_etc_workspace_bytes(n));
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  char* w = static_cast<char*>(ws);
  int64_t* filtered = reinterpret_cast<int64_t*>(w);
  int64_t* own_rows = reinterpret_cast<int64_t*>(w + align_up((size_t)n * 8));
  char* hash_ws = w + 2 * align_up((size_t)n * 8);
  if (!rows) rows = own_rows;
  EtcHeader* hdr = static_cast<EtcHeader*>(etc->storage);
  int64_t* row_keys = reinterpret_cast<int64_t*>(static_cast<char*>(etc->storage) + sizeof(EtcHeader));
  const uint32_t nb = (uint32_t)ceil_div(n, 256);
  hipLaunchKernelGGL(etc_filter, dim3(nb), dim3(256), 0, stream, keys, (uint32_t)n, etc->host_rows, filtered, hdr,
                     (const unsigned long long*)etc->hash->size);
  HCTR_TRY(hash_lookup(etc->hash, filtered, n, 1, rows, hash_ws, ws_bytes - 2 * align_up((size_t)n * 8), stream));
  hipLaunchKernelGGL(etc_note, dim3(nb), dim3(256), 0, stream, (const int64_t*)filtered, (const int64_t*)rows,
                     (uint32_t)n, hdr, row_keys);
  etc_copy_dispatch(false, etc, hdr, row_keys, n, stream);
  return launch_status("hctr_etc_load");
}

HCTR_API hctr_status hctr_etc_dump(hctr_etc* etc, int32_t evict, void* stream_) {
  if (!etc) return fail(HCTR_E_NULL_PTR, "etc is NULL");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  EtcHeader* hdr = static_cast<EtcHeader*>(etc->storage);
  const int64_t* row_keys = reinterpret_cast<const int64_t*>(static_cast<char*>(etc->storage) + sizeof(EtcHeader));
  etc_copy_dispatch(true, etc, hdr, row_keys, etc->hash->max_rows, stream);
  HCTR_TRY(launch_status("etc_dump"));
  if (evict) return hctr_hash_clear(etc->hash, stream_);
  return HCTR_OK;
}

HCTR_API hctr_status hctr_etc_stats(hctr_etc* etc, void* stream_, int64_t* stats) {
  if (!etc || !stats) return fail(HCTR_E_NULL_PTR, "NULL argument");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  EtcHeader h;
  unsigned long long size = 0;
  HCTR_TRY_HIP(hipMemcpyAsync(&h, etc->storage, sizeof(h), hipMemcpyDeviceToHost, stream));
  HCTR_TRY_HIP(hipMemcpyAsync(&size, etc->hash->size, sizeof(size), hipMemcpyDeviceToHost, stream));
  HCTR_TRY_HIP(hipStreamSynchronize(stream));
  stats[0] = (int64_t)size; stats[1] = (int64_t)h.loaded; stats[2] = (int64_t)h.rejected; stats[3] = (int64_t)h.outside;
  return HCTR_OK;
}
