// Device-wide exclusive scan and stable LSD radix sort for wave64 / gfx950.
//
// Both are three-phase, barrier-only designs (no spin waits, no look-back): every kernel finishes
// on its own, the stream orders the phases.  They serve the dedup step of the embedding backward
// pass (sort (row, bag) pairs by row, then mark run boundaries) and the per-set ordering of cache
// insertions.
#include "common.h"

namespace hctr {

// ------------------------------------------------------------------------------------------------
// Exclusive scan
// ------------------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr uint32_t kScanTile = kScanThreads * kScanItems;  // 4096

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

// Exclusive scan of one value per thread over a block of NT threads; *block_total gets the sum.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* lds /*[NT/64 + 1]*/,
                                                         uint32_t* block_total) {
  constexpr int NW = NT / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = wave_inclusive_scan(v);
  if (lane == 63) lds[wave] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t run = 0;
    for (int w = 0; w < NW; ++w) {
      uint32_t t = lds[w];
      lds[w] = run;
      run += t;
    }
    lds[NW] = run;
  }
  __syncthreads();
  uint32_t res = inc - v + lds[wave];
  *block_total = lds[NW];
  __syncthreads();  // lds may be reused by the caller right away
  return res;
}

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
// Radix sort: 8-bit digits, tiles of 4096 keys per 256-thread block.  Each of the block's four
// waves owns 1024 consecutive keys and ranks them 64 at a time with ballot-based digit matching,
// so equal digits keep their input order (stable).
// ------------------------------------------------------------------------------------------------
constexpr int kSortThreads = 256;
constexpr int kSortRounds = kSortTile / kSortThreads;  // 16 rounds of 64 keys per wave

__global__ __launch_bounds__(kSortThreads) void sort_hist(const uint32_t* __restrict__ keys,
                                                          uint32_t n_host,
                                                          const uint32_t* __restrict__ n_dev, int shift,
                                                          uint32_t mask, uint32_t nblk,
                                                          uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[256];
  const uint32_t n = n_dev ? *n_dev : n_host;
  h[threadIdx.x] = 0;
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
  hist[threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];  // digit-major for the scan
}

__global__ __launch_bounds__(kSortThreads) void sort_scatter(
    const uint32_t* __restrict__ kin, const uint32_t* __restrict__ vin, uint32_t* __restrict__ kout,
    uint32_t* __restrict__ vout, uint32_t n_host, const uint32_t* __restrict__ n_dev, int shift,
    uint32_t mask, uint32_t nblk, const uint32_t* __restrict__ hist_scanned) {
  __shared__ uint32_t cnt[kSortThreads / 64][256];
  const uint32_t n = n_dev ? *n_dev : n_host;
  const uint32_t base = blockIdx.x * kSortTile;
  if (base >= n) return;  // whole block leaves together
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int w = 0; w < kSortThreads / 64; ++w) cnt[w][threadIdx.x] = 0;
  __syncthreads();

  const uint32_t wbase = base + wave * (kSortTile / 4);
  const uint64_t below = (1ull << lane) - 1ull;
  uint32_t key[kSortRounds], rank[kSortRounds];
#pragma unroll
  for (int r = 0; r < kSortRounds; ++r) {
    const uint32_t idx = wbase + r * 64 + lane;
    const bool valid = idx < n;
    const uint32_t k = valid ? kin[idx] : 0xFFFFFFFFu;
    key[r] = k;
    const uint32_t d = (k >> shift) & mask;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
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
  {
    const uint32_t d = threadIdx.x;
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
  p.n_max = n_max;
  p.n_blocks = (uint32_t)ceil_div(n_max > 0 ? n_max : 1, kSortTile);
  p.hist_count = 256u * p.n_blocks;
  p.passes = (bits + 7) / 8;
  return p;
}

hctr_status radix_sort_pairs(const SortPlan& plan, int bits, const uint32_t* n_dev, uint32_t* keys0,
                             uint32_t* vals0, uint32_t* keys1, uint32_t* vals1, uint32_t* hist,
                             uint32_t* scan_tmp, hipStream_t stream) {
  uint32_t* k[2] = {keys0, keys1};
  uint32_t* v[2] = {vals0, vals1};
  for (int p = 0; p < plan.passes; ++p) {
    const int shift = 8 * p;
    const int nb = bits - shift < 8 ? bits - shift : 8;
    const uint32_t mask = (1u << nb) - 1u;
    const int src = p & 1, dst = src ^ 1;
    hipLaunchKernelGGL(sort_hist, dim3(plan.n_blocks), dim3(kSortThreads), 0, stream,
                       (const uint32_t*)k[src], plan.n_max, n_dev, shift, mask, plan.n_blocks, hist);
    HCTR_TRY(exclusive_scan_u32(hist, hist, plan.hist_count, scan_tmp, nullptr, stream));
    hipLaunchKernelGGL(sort_scatter, dim3(plan.n_blocks), dim3(kSortThreads), 0, stream,
                       (const uint32_t*)k[src], (const uint32_t*)v[src], k[dst], v[dst], plan.n_max,
                       n_dev, shift, mask, plan.n_blocks, (const uint32_t*)hist);
  }
  return launch_status("radix_sort_pairs");
}

}  // namespace hctr
