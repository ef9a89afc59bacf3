// Device-wide exclusive scan and stable LSD radix sort for wave64 / gfx950.
//
// Both are three-phase, barrier-only designs (no spin waits, no look-back): every kernel finishes
// on its own, the stream orders the phases.  They serve the dedup step of the embedding backward
// pass (sort (row, bag) pairs by row, then mark run boundaries) and the per-set ordering of cache
// insertions.
#include "common.h"
#include "blockscan.h"

namespace hctr {

// ------------------------------------------------------------------------------------------------
// Exclusive scan
// ------------------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr uint32_t kScanTile = kScanThreads * kScanItems;  // 4096

__global__ __launch_bounds__(kScanThreads) void scan_tile_sums(const uint32_t* __restrict__ in,
                                                               uint32_t n, uint32_t* __restrict__ sums) {
  __shared__ uint32_t lds[kScanThreads / 64 + 1];
  const uint32_t base = blockIdx.x * kScanTile;
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    uint32_t idx = base + i * kScanThreads + threadIdx.x;
    if (idx < n) s += in[idx];
  }
  uint32_t total;
  block_exclusive_scan<kScanThreads>(s, lds, &total);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// One block scans the tile sums in place (exclusive), chunk by chunk with a running carry.
__global__ __launch_bounds__(1024) void scan_sums_inplace(uint32_t* __restrict__ sums, uint32_t nb,
                                                          uint32_t* __restrict__ total_out) {
  __shared__ uint32_t lds[1024 / 64 + 1];
  uint32_t carry = 0;
  for (uint32_t c0 = 0; c0 < nb; c0 += 1024) {
    uint32_t idx = c0 + threadIdx.x;
    uint32_t v = idx < nb ? sums[idx] : 0u;
    uint32_t tot;
    uint32_t ex = block_exclusive_scan<1024>(v, lds, &tot);
    if (idx < nb) sums[idx] = ex + carry;
    carry += tot;
  }
  if (total_out != nullptr && threadIdx.x == 0) *total_out = carry;
}

// in and out may be the same array: a thread reads all of its items before it writes any.
__global__ __launch_bounds__(kScanThreads) void scan_apply(const uint32_t* in, uint32_t* out, uint32_t n,
                                                           const uint32_t* __restrict__ sums,
                                                           uint32_t* __restrict__ total_out) {
  __shared__ uint32_t lds[kScanThreads / 64 + 1];
  const uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  uint32_t v[kScanItems];
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    v[i] = (base + i < n) ? in[base + i] : 0u;
    s += v[i];
  }
  uint32_t total;
  uint32_t run = block_exclusive_scan<kScanThreads>(s, lds, &total);
  run += sums ? sums[blockIdx.x] : 0u;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    if (base + i < n) out[base + i] = run;
    run += v[i];
  }
  if (sums == nullptr && total_out != nullptr && threadIdx.x == 0) *total_out = total;
}

size_t scan_tmp_count(uint32_t n) { return (size_t)ceil_div(n > 0 ? n : 1, kScanTile); }

hctr_status exclusive_scan_u32(const uint32_t* in, uint32_t* out, uint32_t n, uint32_t* tmp,
                               uint32_t* total, hipStream_t stream) {
  const uint32_t nb = (uint32_t)ceil_div(n > 0 ? n : 1, kScanTile);
  if (nb == 1) {
    hipLaunchKernelGGL(scan_apply, dim3(1), dim3(kScanThreads), 0, stream, in, out, n,
                       (const uint32_t*)nullptr, total);
    return launch_status("scan_apply");
  }
  hipLaunchKernelGGL(scan_tile_sums, dim3(nb), dim3(kScanThreads), 0, stream, in, n, tmp);
  hipLaunchKernelGGL(scan_sums_inplace, dim3(1), dim3(1024), 0, stream, tmp, nb, total);
  hipLaunchKernelGGL(scan_apply, dim3(nb), dim3(kScanThreads), 0, stream, in, out, n,
                     (const uint32_t*)tmp, (uint32_t*)nullptr);
  return launch_status("exclusive_scan_u32");
}

// ------------------------------------------------------------------------------------------------
// Radix sort: digits of up to 10 bits (so 28-bit row ids take 3 passes), tiles of 4096 keys per
// 256-thread block.  Each of the block's four waves owns 1024 consecutive keys and ranks them 64 at
// a time with ballot-based digit matching, so equal digits keep their input order (stable).
// ------------------------------------------------------------------------------------------------
constexpr int kSortThreads = 256;
constexpr int kSortRounds = kSortTile / kSortThreads;  // 16 rounds of 64 keys per wave
constexpr int kMaxBins = 1 << kSortMaxDigitBits;

__global__ __launch_bounds__(kSortThreads) void sort_hist(const uint32_t* __restrict__ keys,
                                                          uint32_t n_host,
                                                          const uint32_t* __restrict__ n_dev, int shift,
                                                          uint32_t bins, uint32_t nblk,
                                                          uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[kMaxBins];
  const uint32_t n = n_dev ? *n_dev : n_host;
  const uint32_t mask = bins - 1;
  for (uint32_t d = threadIdx.x; d < bins; d += kSortThreads) h[d] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * kSortTile;
  if (base < n) {
#pragma unroll 4
    for (int i = 0; i < kSortRounds; ++i) {
      uint32_t idx = base + i * kSortThreads + threadIdx.x;
      if (idx < n) atomicAdd(&h[(keys[idx] >> shift) & mask], 1u);
    }
  }
  __syncthreads();
  for (uint32_t d = threadIdx.x; d < bins; d += kSortThreads)
    hist[d * nblk + blockIdx.x] = h[d];  // digit-major for the scan
}

template <int DBITS>
__global__ __launch_bounds__(kSortThreads) void sort_scatter(
    const uint32_t* __restrict__ kin, const uint32_t* __restrict__ vin, uint32_t* __restrict__ kout,
    uint32_t* __restrict__ vout, uint32_t n_host, const uint32_t* __restrict__ n_dev, int shift,
    uint32_t bins, uint32_t nblk, const uint32_t* __restrict__ hist_scanned) {
  constexpr int BINS_MAX = 1 << DBITS;
  __shared__ uint32_t cnt[kSortThreads / 64][BINS_MAX];
  const uint32_t n = n_dev ? *n_dev : n_host;
  const uint32_t mask = bins - 1;
  const uint32_t base = blockIdx.x * kSortTile;
  if (base >= n) return;  // whole block leaves together
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (uint32_t d = threadIdx.x; d < bins; d += kSortThreads) {
#pragma unroll
    for (int w = 0; w < kSortThreads / 64; ++w) cnt[w][d] = 0;
  }
  __syncthreads();

  const uint32_t wbase = base + wave * (kSortTile / 4);
  const uint64_t below = (1ull << lane) - 1ull;
  uint32_t key[kSortRounds], rank[kSortRounds];
#pragma unroll
  for (int r = 0; r < kSortRounds; ++r) {
    const uint32_t idx = wbase + r * 64 + lane;
    key[r] = idx < n ? kin[idx] : 0xFFFFFFFFu;
  }
#pragma unroll
  for (int r = 0; r < kSortRounds; ++r) {
    const uint32_t idx = wbase + r * 64 + lane;
    const bool valid = idx < n;
    const uint32_t d = (key[r] >> shift) & mask;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < DBITS; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t vote = __ballot(bit);
      peers &= bit ? vote : ~vote;
    }
    const uint64_t lower = peers & below;
    uint32_t old = 0;
    if (valid && lower == 0) old = atomicAdd(&cnt[wave][d], (uint32_t)__popcll(peers));
    const int leader = valid ? (__ffsll((unsigned long long)peers) - 1) : lane;
    old = __shfl(old, leader);
    rank[r] = old + (uint32_t)__popcll(lower);
  }
  __syncthreads();
  for (uint32_t d = threadIdx.x; d < bins; d += kSortThreads) {
    uint32_t run = hist_scanned[d * nblk + blockIdx.x];
#pragma unroll
    for (int w = 0; w < kSortThreads / 64; ++w) {
      uint32_t c = cnt[w][d];
      cnt[w][d] = run;
      run += c;
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kSortRounds; ++r) {
    const uint32_t idx = wbase + r * 64 + lane;
    if (idx < n) {
      const uint32_t d = (key[r] >> shift) & mask;
      const uint32_t pos = cnt[wave][d] + rank[r];
      kout[pos] = key[r];
      vout[pos] = vin[idx];
    }
  }
}

SortPlan sort_plan(uint32_t n_max, int bits) {
  SortPlan p;
  if (bits < 1) bits = 1;
  p.n_max = n_max;
  p.n_blocks = (uint32_t)ceil_div(n_max > 0 ? n_max : 1, kSortTile);
  p.passes = (bits + kSortMaxDigitBits - 1) / kSortMaxDigitBits;
  uint32_t max_bins = 0;
  for (int i = 0; i < p.passes; ++i) {  // spread the bits evenly: 28 -> 10, 9, 9
    p.digit_bits[i] = bits / p.passes + (i < bits % p.passes ? 1 : 0);
    if ((1u << p.digit_bits[i]) > max_bins) max_bins = 1u << p.digit_bits[i];
  }
  p.hist_count = max_bins * p.n_blocks;
  return p;
}

hctr_status radix_sort_pairs(const SortPlan& plan, const uint32_t* n_dev, uint32_t* keys0,
                             uint32_t* vals0, uint32_t* keys1, uint32_t* vals1, uint32_t* hist,
                             uint32_t* scan_tmp, hipStream_t stream) {
  uint32_t* k[2] = {keys0, keys1};
  uint32_t* v[2] = {vals0, vals1};
  int shift = 0;
  for (int p = 0; p < plan.passes; ++p) {
    const int db = plan.digit_bits[p];
    const uint32_t bins = 1u << db;
    const int src = p & 1, dst = src ^ 1;
    hipLaunchKernelGGL(sort_hist, dim3(plan.n_blocks), dim3(kSortThreads), 0, stream,
                       (const uint32_t*)k[src], plan.n_max, n_dev, shift, bins, plan.n_blocks, hist);
    HCTR_TRY(exclusive_scan_u32(hist, hist, bins * plan.n_blocks, scan_tmp, nullptr, stream));
    if (db <= 8)
      hipLaunchKernelGGL((sort_scatter<8>), dim3(plan.n_blocks), dim3(kSortThreads), 0, stream,
                         (const uint32_t*)k[src], (const uint32_t*)v[src], k[dst], v[dst], plan.n_max,
                         n_dev, shift, bins, plan.n_blocks, (const uint32_t*)hist);
    else
      hipLaunchKernelGGL((sort_scatter<kSortMaxDigitBits>), dim3(plan.n_blocks), dim3(kSortThreads), 0,
                         stream, (const uint32_t*)k[src], (const uint32_t*)v[src], k[dst], v[dst],
                         plan.n_max, n_dev, shift, bins, plan.n_blocks, (const uint32_t*)hist);
    shift += db;
  }
  return launch_status("radix_sort_pairs");
}

}  // namespace hctr
