// Internal helpers shared by the HIP translation units of libhctr (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>

#include "hctr.h"

#define HCTR_API extern "C" __attribute__((visibility("default")))

namespace hctr {

constexpr int kWave = 64;
constexpr uint32_t kNoRow = 0xFFFFFFFFu;          // 32-bit global row id meaning "key has no row"
constexpr uint64_t kEmptyKey = ~0ull;             // empty hash slot / empty cache tag

// Error text of the last failing call on this thread.
void set_error(const char* fmt, ...);
hctr_status fail(hctr_status st, const char* fmt, ...);
hctr_status check_hip(hipError_t e, const char* what);

#define HCTR_TRY_HIP(expr)                                        \
  do {                                                            \
    hipError_t e_ = (expr);                                       \
    if (e_ != hipSuccess) return ::hctr::check_hip(e_, #expr);    \
  } while (0)

#define HCTR_TRY(expr)                         \
  do {                                         \
    hctr_status s_ = (expr);                   \
    if (s_ != HCTR_OK) return s_;              \
  } while (0)

inline hctr_status launch_status(const char* what) { return check_hip(hipGetLastError(), what); }

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int ceil_log2(uint64_t x) {  // smallest b with 2^b >= x
  int b = 0;
  while (b < 64 && (1ull << b) < x) ++b;
  return b;
}
inline int pow2_ceil(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}

// Carves a workspace into 256-byte aligned pieces; with base == nullptr it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t count) {
    size_t at = off;
    off = align_up(off + count * sizeof(T));
    return base ? reinterpret_cast<T*>(base + at) : nullptr;
  }
};

// ---- device-side scan and sort primitives (primitives.hip) -------------------------------------

// Exclusive prefix sum of uint32 in[0..n) into out (may alias in).  tmp holds scan_tmp_count(n)
// uint32.  If total != nullptr the grand total is written there (uint32).  With n_dev != nullptr
// only the first min(*n_dev, n) items are scanned (a count known on the device only, read when the
// kernels run); items past it are neither read nor written, and total covers the scanned ones.
size_t scan_tmp_count(uint32_t n);
hctr_status exclusive_scan_u32(const uint32_t* in, uint32_t* out, uint32_t n, uint32_t* tmp,
                               uint32_t* total, hipStream_t stream, const uint32_t* n_dev = nullptr);

// Stable LSD radix sort of packed words (key << 32 | value) on the low `bits` bits of the key, in
// ceil(bits / 10) passes of evenly sized digits.  The element count is *n_dev if n_dev != nullptr
// (must be <= n_max), else n_max.  buf0 holds the input; the result lands in buf[passes & 1].
// hist holds plan.hist_count words; aux holds plan.aux_count words that must be zero on entry
// (aux_is_zero = false makes the sort clear them itself with one more launch).
constexpr uint32_t kSortTile = 4096;
constexpr uint32_t kSortSuper = 16;   // tiles per group with a shared running sum
constexpr int kSortMaxDigitBits = 10;
struct SortPlan {
  uint32_t n_max = 0;
  uint32_t n_blocks = 0;   // tiles of kSortTile words
  uint32_t n_super = 0;    // groups of kSortSuper tiles
  uint32_t max_bins = 0;
  size_t hist_count = 0;   // max_bins * n_blocks
  size_t aux_count = 0;    // passes * (1 + n_super) * max_bins
  int passes = 0;
  int digit_bits[4] = {0, 0, 0, 0};
};
SortPlan sort_plan(uint32_t n_max, int bits);
// Per pass p the aux area holds tot[max_bins] followed by sup[n_super][max_bins].
constexpr uint32_t kSortWideMaxTiles = 1024;  // up to this many tiles the sort uses 1024-thread blocks
constexpr uint32_t kSortDirectSuperMax = 48;  // above this many groups the group sums get their own scan
inline uint32_t* sort_aux_tot(const SortPlan& plan, uint32_t* aux, int p) {
  return aux + (size_t)p * (1 + plan.n_super) * plan.max_bins;
}
inline uint32_t* sort_aux_sup(const SortPlan& plan, uint32_t* aux, int p) {
  return sort_aux_tot(plan, aux, p) + plan.max_bins;
}
// Above kSortDirectSuperMax groups the group sums are built from the tile histograms and scanned by
// kernels of their own; the histogram kernels then add nothing to sup (pass NULL).
inline bool sort_scans_groups(const SortPlan& plan) { return plan.n_super > kSortDirectSuperMax; }
// first_hist_done: the caller has already filled hist[tile][digit] (and, unless
// sort_scans_groups(plan), added it to sup) for pass 0 (digit = low digit_bits[0] bits of the key)
// while producing buf0.
hctr_status radix_sort_u64(const SortPlan& plan, const uint32_t* n_dev, uint64_t* buf0, uint64_t* buf1,
                           uint32_t* hist, uint32_t* aux, bool aux_is_zero, hipStream_t stream,
                           bool first_hist_done = false);

// Bytes of work arrays that one hctr_cache_query call with nnz keys uses, on the path that call
// takes (cache.hip).
size_t cache_call_ws_bytes(const hctr_cache* c, int64_t nnz);

}  // namespace hctr
