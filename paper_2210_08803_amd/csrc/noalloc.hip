// Cache query for callers that cannot allocate device memory (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): the work arrays that hctr_cache_query takes as
// its `ws` argument live in a file-scope device array of this library instead.  Every GPU the
// library runs on holds its own copy of the array until the process ends.
#include <mutex>

#include "common.h"

namespace {

// line_of / miss flags of a call (8 bytes per key) and, on the general path, the work arrays of the
// first-appearance dedup, the (set, index) sort and the staging rows (dim * 4 bytes per key).
static __device__ __align__(256) unsigned char scratch[HCTR_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once asked for

// `scratch` is a host-side stand-in in host code; the memory behind it on the current device is what
// hipGetSymbolAddress returns, asked for once per device and kept.
hctr_status scratch_of_current_device(void** out) {
  int dev = -1;
  HCTR_TRY_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return hctr::fail(HCTR_E_UNSUPPORTED, "device %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_ptr[dev] == nullptr) {
    void* p = nullptr;
    HCTR_TRY_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return hctr::fail(HCTR_E_DEVICE, "hipGetSymbolAddress gave no address for the scratch array");
    g_ptr[dev] = p;
  }
  *out = g_ptr[dev];
  return HCTR_OK;
}

}  // namespace

HCTR_API hctr_status hctr_cache_query_static(hctr_cache* cache, int64_t batch, int32_t num_slots,
                                             const int64_t* keys, const int64_t* offsets, int64_t nnz,
                                             int32_t insert_missing, float* out, uint8_t* hit_mask,
                                             void* stream) {
  if (!cache) return hctr::fail(HCTR_E_NULL_PTR, "cache is NULL");
  if (nnz < 0) return hctr::fail(HCTR_E_INVALID_ARG, "nnz %lld negative", (long long)nnz);
  if (nnz > HCTR_STATIC_MAX_KEYS)
    return hctr::fail(HCTR_E_UNSUPPORTED, "hctr_cache_query_static takes at most %d keys per call, got %lld",
                      HCTR_STATIC_MAX_KEYS, (long long)nnz);
  const size_t need = hctr::cache_call_ws_bytes(cache, nnz);
  if (need > (size_t)HCTR_STATIC_SCRATCH_BYTES)
    return hctr::fail(HCTR_E_UNSUPPORTED,
                      "this call needs %zu bytes of work arrays, the static scratch has %zu (rows too wide for "
                      "the general path at this key count)", need, (size_t)HCTR_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  HCTR_TRY(scratch_of_current_device(&ws));
  return hctr_cache_query(cache, batch, num_slots, keys, offsets, nnz, insert_missing, out, hit_mask, ws,
                          (size_t)HCTR_STATIC_SCRATCH_BYTES, stream);
}
