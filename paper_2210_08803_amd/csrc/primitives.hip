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
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr uint32_t kScanTile = kScanThreads * kScanItems;  // 4096

// Length actually scanned: the first *n_dev items when a device-side count is given (never more
// than the host's n); items past it are neither read nor written.
__device__ __forceinline__ uint32_t scan_length(uint32_t n_host, const uint32_t* n_dev) {
  if (n_dev == nullptr) return n_host;
  const uint32_t nd = *n_dev;
  return nd < n_host ? nd : n_host;
}


__global__ __launch_bounds__(kScanThreads) void scan_tile_sums(const uint32_t* __restrict__ in,
                                                               uint32_t n_host,
                                                               const uint32_t* __restrict__ n_dev,
                                                               uint32_t* __restrict__ sums) {
  __shared__ uint32_t lds[kScanThreads / 64 + 1];
  const uint32_t n = scan_length(n_host, n_dev);
  const uint32_t base = blockIdx.x * kScanTile;
  uint32_t s = 0;
  if (base < n) {   // block-uniform; the items themselves without a branch (index clamped), all in flight
    uint32_t v[kScanItems];
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
      const uint32_t idx = base + i * kScanThreads + threadIdx.x;
      v[i] = in[idx < n ? idx : n - 1];
    }
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) s += base + i * kScanThreads + threadIdx.x < n ? v[i] : 0u;
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
__global__ __launch_bounds__(kScanThreads) void scan_apply(const uint32_t* in, uint32_t* out, uint32_t n_host,
                                                           const uint32_t* __restrict__ n_dev,
                                                           const uint32_t* __restrict__ sums,
                                                           uint32_t* __restrict__ total_out) {
  __shared__ uint32_t lds[kScanThreads / 64 + 1];
  const uint32_t n = scan_length(n_host, n_dev);
  const uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  uint32_t v[kScanItems];
  uint32_t s = 0;
  // a thread's 16 consecutive items as four 16-byte accesses when they all exist and the arrays
  // allow it (word by word, a wave's load touches 64 separate 64-byte pieces)
  const bool whole = (uint64_t)base + kScanItems <= n &&
                     ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15u) == 0;
  if (whole) {
#pragma unroll
    for (int i = 0; i < kScanItems; i += 4) {
      const u32x4v q = *reinterpret_cast<const u32x4v*>(in + base + i);
      v[i] = q.x; v[i + 1] = q.y; v[i + 2] = q.z; v[i + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) v[i] = (base + i < n) ? in[base + i] : 0u;
  }
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) s += v[i];
  uint32_t total;
  uint32_t run = block_exclusive_scan<kScanThreads>(s, lds, &total);
  run += sums ? sums[blockIdx.x] : 0u;
  if (whole) {
#pragma unroll
    for (int i = 0; i < kScanItems; i += 4) {
      u32x4v q;
      q.x = run; run += v[i];
      q.y = run; run += v[i + 1];
      q.z = run; run += v[i + 2];
      q.w = run; run += v[i + 3];
      *reinterpret_cast<u32x4v*>(out + base + i) = q;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
      if (base + i < n) out[base + i] = run;
      run += v[i];
    }
  }
  if (sums == nullptr && total_out != nullptr && threadIdx.x == 0) *total_out = total;
}

size_t scan_tmp_count(uint32_t n) { return (size_t)ceil_div(n > 0 ? n : 1, kScanTile); }

hctr_status exclusive_scan_u32(const uint32_t* in, uint32_t* out, uint32_t n, uint32_t* tmp,
                               uint32_t* total, hipStream_t stream, const uint32_t* n_dev) {
  const uint32_t nb = (uint32_t)ceil_div(n > 0 ? n : 1, kScanTile);
  if (nb == 1) {
    hipLaunchKernelGGL(scan_apply, dim3(1), dim3(kScanThreads), 0, stream, in, out, n, n_dev,
                       (const uint32_t*)nullptr, total);
    return launch_status("scan_apply");
  }
  hipLaunchKernelGGL(scan_tile_sums, dim3(nb), dim3(kScanThreads), 0, stream, in, n, n_dev, tmp);
  hipLaunchKernelGGL(scan_sums_inplace, dim3(1), dim3(1024), 0, stream, tmp, nb, total);
  hipLaunchKernelGGL(scan_apply, dim3(nb), dim3(kScanThreads), 0, stream, in, out, n, n_dev,
                     (const uint32_t*)tmp, (uint32_t*)nullptr);
  return launch_status("exclusive_scan_u32");
}

// ------------------------------------------------------------------------------------------------
// Radix sort of packed (key << 32 | value) words by the key's low `bits` bits: LSD, digits of up
// to 10 bits (28-bit row ids take 3 passes), tiles of 4096 words per block, two kernels per pass
// up to 48 groups of 16 tiles (about 3 M words) and no device-wide scan kernel in between:
//   sort_hist     counts the tile's digits into hist[tile][digit] (block-major, coalesced) and adds
//                 them to sup[tile / 16][digit] (sums over groups of 16 tiles);
//   sort_scatter  derives the tile's global offsets on its own - digit totals = sum of all sup
//                 rows, scanned in LDS, plus the sup rows of earlier groups, plus the hist rows of
//                 earlier tiles of its group (at most n_tiles/16 + 15 coalesced row reads) - then
//                 ranks and scatters.
// Beyond that, two kernels between them prepare the offsets: sort_sum_groups builds the group sums
// and turns the hist rows of a group into running sums within the group, sort_scan_groups scans the
// group sums; a scatter block then reads three rows (digit totals, its group's, its tile's).
// Each wave of a block owns a run of consecutive words and ranks them 64 at a time with ballot-based
// digit matching, so equal digits keep their input order (stable).  Blocks have 256 threads (waves
// own 1024 words) when there are tiles enough to fill the chip several times over, else 1024
// threads for the counting kernel: with about one tile per compute unit it is bound by the length
// of a thread's serial loop, not by bandwidth (the scatter measured faster with 256 threads).
// ------------------------------------------------------------------------------------------------
constexpr int kSortThreads = 256;
constexpr int kSortWideThreads = 1024;
constexpr int kMaxBins = 1 << kSortMaxDigitBits;

__global__ __launch_bounds__(256) void sort_zero_aux(uint32_t* __restrict__ aux, uint32_t count) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < count) aux[i] = 0u;
}

template <int NT>
__global__ __launch_bounds__(NT) void sort_hist(const uint64_t* __restrict__ kv, uint32_t n_host,
                                                const uint32_t* __restrict__ n_dev, int shift,
                                                uint32_t bins, uint32_t* __restrict__ hist,
                                                uint32_t* __restrict__ sup) {
  // Four copies of the counters, lane l adds to copy l mod 4: with skewed digits (the top bits of the
  // rows) many lanes of a wave hold the same digit and their adds to one LDS address queue up (that
  // pass took 274 us against 181 us for a spread digit on 86 M words).  A copy is one word longer
  // than the bins so that a digit's four counters sit in four different banks.
  constexpr int COPIES = 4;
  __shared__ uint32_t h[COPIES][kMaxBins + 1];
  const uint32_t n = n_dev ? *n_dev : n_host;
  const uint32_t base = blockIdx.x * kSortTile;
  if (base >= n) return;  // nobody reads the rows of tiles past the end
  const uint32_t mask = bins - 1;
  for (uint32_t d = threadIdx.x; d < bins; d += NT) {
#pragma unroll
    for (int c = 0; c < COPIES; ++c) h[c][d] = 0;
  }
  __syncthreads();
  // all of the thread's words first, index clamped instead of a branch (a load under a branch is
  // waited for before the next one is issued)
  constexpr int PER = (int)(kSortTile / NT);
  uint64_t w[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const uint32_t idx = base + i * NT + threadIdx.x;
    w[i] = kv[idx < n ? idx : n - 1];
  }
  __builtin_amdgcn_sched_barrier(0);   // every load above is issued before the first use below
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const uint32_t idx = base + i * NT + threadIdx.x;
    if (idx < n) atomicAdd(&h[threadIdx.x & (COPIES - 1)][(uint32_t)(w[i] >> (32 + shift)) & mask], 1u);
  }
  __syncthreads();
  uint32_t* row = hist + (uint64_t)blockIdx.x * bins;
  uint32_t* srow = sup + (uint64_t)(blockIdx.x / kSortSuper) * bins;
  for (uint32_t d = threadIdx.x; d < bins; d += NT) {
    const uint32_t c = h[0][d] + h[1][d] + h[2][d] + h[3][d];
    row[d] = c;
    if (c && sup) atomicAdd(&srow[d], c);
  }
}

// For many tiles the group sums get kernels of their own, so that a scatter block reads one row
// instead of one per earlier group.  sort_sum_groups: one block per group adds the histograms of
// its (at most 16) tiles and leaves in each tile's row the sum of the rows before it in the group
// (the 16 tiles of a group run on 8 dies, so every scatter block adding up the rows before its
// own fetched them from memory again: 1.31 GB read per pass for 0.69 GB of words).
// sort_scan_groups: a block of 1024 threads owns 32 digits; its threads
// form 32 chunks of consecutive groups x 32 digits, sum their chunk, combine the chunk sums through
// LDS and then turn their chunk into running sums (sup[g][d] = count of digit d in all earlier
// groups) - every load of a chunk is independent of the others, where one thread per digit walking
// all groups took 88 us per pass for 1,300 groups.
__global__ __launch_bounds__(256) void sort_sum_groups(uint32_t* __restrict__ hist, uint32_t n_host,
                                                       const uint32_t* __restrict__ n_dev, uint32_t bins,
                                                       uint32_t* __restrict__ sup) {
  const uint32_t n = n_dev ? *n_dev : n_host;
  const uint32_t n_tiles = (uint32_t)(((uint64_t)n + kSortTile - 1) / kSortTile);
  const uint32_t g = blockIdx.x;
  const uint32_t d0 = threadIdx.x * 4;
  if (d0 >= bins) return;
  u32x4v acc = {0, 0, 0, 0}, v[kSortSuper];
#pragma unroll
  for (uint32_t k = 0; k < kSortSuper; ++k) {
    const uint32_t t = g * kSortSuper + k;
    v[k] = t < n_tiles ? *reinterpret_cast<const u32x4v*>(hist + (uint64_t)t * bins + d0) : u32x4v{0, 0, 0, 0};
  }
#pragma unroll
  for (uint32_t k = 0; k < kSortSuper; ++k) {
    const uint32_t t = g * kSortSuper + k;
    if (t < n_tiles) *reinterpret_cast<u32x4v*>(hist + (uint64_t)t * bins + d0) = acc;
    acc += v[k];
  }
  *reinterpret_cast<u32x4v*>(sup + (uint64_t)g * bins + d0) = acc;
}

__global__ __launch_bounds__(1024) void sort_scan_groups(uint32_t* __restrict__ sup, uint32_t* __restrict__ tot,
                                                         uint32_t bins, uint32_t n_super) {
  __shared__ uint32_t part[32][33];
  const uint32_t dd = threadIdx.x & 31, c = threadIdx.x >> 5;
  const uint32_t d = blockIdx.x * 32 + dd;   // bins is a multiple of 4 and may be below 32: guard below
  const uint32_t per = (n_super + 31) / 32;
  const uint32_t g0 = c * per, g1 = (g0 + per < n_super) ? g0 + per : n_super;
  uint32_t sum = 0;
  if (d < bins) {
    for (uint32_t g = g0; g < g1; g += 8) {
      uint32_t v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = g + k < g1 ? sup[(uint64_t)(g + k) * bins + d] : 0u;
#pragma unroll
      for (int k = 0; k < 8; ++k) sum += v[k];
    }
  }
  part[c][dd] = sum;
  __syncthreads();
  uint32_t run = 0, all = 0;
  for (uint32_t cc = 0; cc < 32; ++cc) {
    const uint32_t p = part[cc][dd];
    if (cc < c) run += p;
    all += p;
  }
  if (d < bins) {
    if (c == 0) tot[d] = all;
    for (uint32_t g = g0; g < g1; g += 8) {
      uint32_t v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = g + k < g1 ? sup[(uint64_t)(g + k) * bins + d] : 0u;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (g + k < g1) sup[(uint64_t)(g + k) * bins + d] = run;
        run += v[k];
      }
    }
  }
}

template <int DBITS, int NT, bool SCANNED>
__global__ __launch_bounds__(NT) void sort_scatter(
    const uint64_t* __restrict__ in, uint64_t* __restrict__ out, uint32_t n_host,
    const uint32_t* __restrict__ n_dev, int shift, uint32_t bins, const uint32_t* __restrict__ hist,
    const uint32_t* __restrict__ tot, const uint32_t* __restrict__ sup, uint32_t n_super) {
  constexpr int BINS_MAX = 1 << DBITS;
  __shared__ uint32_t cnt[NT / 64][BINS_MAX];
  __shared__ uint32_t gbase[BINS_MAX];
  __shared__ uint32_t scan_lds[NT / 64 + 1];
  const uint32_t n = n_dev ? *n_dev : n_host;
  const uint32_t mask = bins - 1;
  // Workgroups go to the chip's 8 dies in turn, each with an L2 of its own.  Die x takes the x-th
  // eighth of the input, so that the blocks resident on a die hold neighbouring tiles: their runs of
  // one digit are adjacent in the output and leave that L2 as whole lines instead of pieces.
  const uint32_t gq = gridDim.x >> 3, gr = gridDim.x & 7u, die = blockIdx.x & 7u;
  const uint32_t blk = die * gq + (die < gr ? die : gr) + (blockIdx.x >> 3);   // tile of this block
  const uint32_t base = blk * kSortTile;
  if (base >= n) return;  // whole block leaves together
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // The tile's words first: their latency hides behind the offset computation below.
  constexpr int ROUNDS = kSortTile / NT;   // rounds of 64 words per wave
  const uint32_t wbase = base + wave * (ROUNDS * 64);
  uint64_t word[ROUNDS];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {   // index clamped instead of a branch: all loads leave together
    const uint32_t idx = wbase + r * 64 + lane;
    word[r] = in[idx < n ? idx : n - 1];
  }

  // Global offset of each digit for this tile: thread t owns digits 4t .. 4t+3.
  {
    const uint32_t d0 = threadIdx.x * 4;
    u32x4v t4 = {0, 0, 0, 0}, pre = {0, 0, 0, 0};
    if (d0 < bins) {
      const uint32_t g = blk / kSortSuper;
      if (SCANNED) {   // sort_sum_groups left the running sums within the group in hist
        t4 = *reinterpret_cast<const u32x4v*>(tot + d0);
        pre = *reinterpret_cast<const u32x4v*>(sup + (uint64_t)g * bins + d0);
        pre += *reinterpret_cast<const u32x4v*>(hist + (uint64_t)blk * bins + d0);
      } else {
        const uint32_t b_begin = g * kSortSuper;   // at most kSortSuper - 1 = 15 rows of this group
        u32x4v hrow[kSortSuper - 1];
#pragma unroll
        for (uint32_t k = 0; k < kSortSuper - 1; ++k)   // requested first: in flight while the group sums arrive
          hrow[k] = b_begin + k < blk ? *reinterpret_cast<const u32x4v*>(hist + (uint64_t)(b_begin + k) * bins + d0)
                                        : u32x4v{0, 0, 0, 0};
        // rows are fetched twelve at a time so the loads overlap instead of queueing behind each other
        constexpr uint32_t kBatch = 12;
        for (uint32_t sb0 = 0; sb0 < n_super; sb0 += kBatch) {
          u32x4v v[kBatch];
#pragma unroll
          for (uint32_t k = 0; k < kBatch; ++k)
            v[k] = sb0 + k < n_super ? *reinterpret_cast<const u32x4v*>(sup + (uint64_t)(sb0 + k) * bins + d0)
                                     : u32x4v{0, 0, 0, 0};
#pragma unroll
          for (uint32_t k = 0; k < kBatch; ++k) {
            t4 += v[k];
            if (sb0 + k < g) pre += v[k];
          }
        }
#pragma unroll
        for (uint32_t k = 0; k < kSortSuper - 1; ++k) pre += hrow[k];
      }
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan<NT>(t4.x + t4.y + t4.z + t4.w, scan_lds, &total);
    if (d0 < bins) {
      gbase[d0] = run + pre.x; run += t4.x;
      gbase[d0 + 1] = run + pre.y; run += t4.y;
      gbase[d0 + 2] = run + pre.z; run += t4.z;
      gbase[d0 + 3] = run + pre.w;
    }
  }
  for (uint32_t d = threadIdx.x; d < bins; d += NT) {
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) cnt[w][d] = 0;
  }
  __syncthreads();

  const uint64_t below = (1ull << lane) - 1ull;
  uint32_t rank[ROUNDS];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const uint32_t idx = wbase + r * 64 + lane;
    const bool valid = idx < n;
    const uint32_t d = (uint32_t)(word[r] >> (32 + shift)) & mask;
    // peers = the valid lanes whose digit equals this lane's.  Per bit: m = the lane's bit spread over
    // a word (0 or ~0), vote ^ m = the lanes whose bit differs; those are collected over all bits
    // and struck out at the end (four vector instructions per bit, where a select between vote and
    // ~vote took nine - the ranking is bound by them).
    uint32_t differs_lo = 0, differs_hi = 0;
#pragma unroll
    for (int b = 0; b < DBITS; ++b) {
      const uint32_t m = (uint32_t)((int32_t)(d << (31 - b)) >> 31);
      const uint64_t vote = __ballot(m != 0u);
      differs_lo |= (uint32_t)vote ^ m;
      differs_hi |= (uint32_t)(vote >> 32) ^ m;
    }
    const uint64_t peers = __ballot(valid) & ~(((uint64_t)differs_hi << 32) | differs_lo);
    const uint64_t lower = peers & below;
    uint32_t old = 0;
    if (valid && lower == 0) old = atomicAdd(&cnt[wave][d], (uint32_t)__popcll(peers));
    const int leader = valid ? (__ffsll((unsigned long long)peers) - 1) : lane;
    old = __shfl(old, leader);
    rank[r] = old + (uint32_t)__popcll(lower);
  }
  __syncthreads();
  if constexpr (SCANNED) {
    // Many tiles: the stores are what counts.  Written straight from the registers, neighbouring
    // lanes hold words of different digits and a wave's store goes to 64 places, 8 bytes each.
    // The tile is sorted within LDS first (a word's place in the tile = words of smaller digits +
    // words of its digit in earlier waves + its rank), then written out in that order: neighbouring
    // lanes hold neighbouring words of a digit's run, and a store touches as few lines as the runs allow.
    __shared__ uint64_t stage[kSortTile];
    const uint32_t d0 = threadIdx.x * 4;   // thread t owns digits 4t .. 4t+3, as above
    uint32_t c[4][NT / 64], tile_cnt[4] = {0, 0, 0, 0};
    if (d0 < bins) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) {
          c[k][w] = cnt[w][d0 + k];
          tile_cnt[k] += c[k][w];
        }
      }
    }
    uint32_t total;
    uint32_t local = block_exclusive_scan<NT>(tile_cnt[0] + tile_cnt[1] + tile_cnt[2] + tile_cnt[3], scan_lds, &total);
    if (d0 < bins) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        gbase[d0 + k] -= local;   // place in the output = place in the tile + this difference
        uint32_t run = local;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) {
          cnt[w][d0 + k] = run;
          run += c[k][w];
        }
        local += tile_cnt[k];
      }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const uint32_t idx = wbase + r * 64 + lane;
      if (idx < n) {
        const uint32_t d = (uint32_t)(word[r] >> (32 + shift)) & mask;
        stage[cnt[wave][d] + rank[r]] = word[r];
      }
    }
    __syncthreads();
    const uint32_t held = n - base < kSortTile ? n - base : kSortTile;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const uint32_t j = r * NT + threadIdx.x;
      if (j < held) {
        const uint64_t w = stage[j];
        const uint32_t d = (uint32_t)(w >> (32 + shift)) & mask;
        out[gbase[d] + j] = w;
      }
    }
  } else {
    for (uint32_t d = threadIdx.x; d < bins; d += NT) {
      uint32_t run = gbase[d];
#pragma unroll
      for (int w = 0; w < NT / 64; ++w) {
        const uint32_t c = cnt[w][d];
        cnt[w][d] = run;
        run += c;
      }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const uint32_t idx = wbase + r * 64 + lane;
      if (idx < n) {
        const uint32_t d = (uint32_t)(word[r] >> (32 + shift)) & mask;
        out[cnt[wave][d] + rank[r]] = word[r];
      }
    }
  }
}

SortPlan sort_plan(uint32_t n_max, int bits) {
  SortPlan p;
  if (bits < 1) bits = 1;
  if (bits > 32) bits = 32;
  p.n_max = n_max;
  p.n_blocks = (uint32_t)ceil_div(n_max > 0 ? n_max : 1, kSortTile);
  p.n_super = (uint32_t)ceil_div(p.n_blocks, kSortSuper);
  p.passes = (bits + kSortMaxDigitBits - 1) / kSortMaxDigitBits;
  p.max_bins = 4;
  for (int i = 0; i < p.passes; ++i) {  // spread the bits evenly: 28 -> 10, 9, 9
    p.digit_bits[i] = bits / p.passes + (i < bits % p.passes ? 1 : 0);
    if (p.digit_bits[i] < 2) p.digit_bits[i] = 2;   // rows are read four digits at a time
    if ((1u << p.digit_bits[i]) > p.max_bins) p.max_bins = 1u << p.digit_bits[i];
  }
  p.hist_count = (size_t)p.max_bins * p.n_blocks;
  p.aux_count = (size_t)p.passes * (1 + p.n_super) * p.max_bins;
  return p;
}

hctr_status radix_sort_u64(const SortPlan& plan, const uint32_t* n_dev, uint64_t* buf0, uint64_t* buf1,
                           uint32_t* hist, uint32_t* aux, bool aux_is_zero, hipStream_t stream,
                           bool first_hist_done) {
  uint64_t* buf[2] = {buf0, buf1};
  if (!aux_is_zero)
    hipLaunchKernelGGL(sort_zero_aux, dim3((uint32_t)ceil_div((int64_t)plan.aux_count, 256)), dim3(256), 0,
                       stream, aux, (uint32_t)plan.aux_count);
  const int scan_sup = sort_scans_groups(plan) ? 1 : 0;
  const bool wide = plan.n_blocks <= kSortWideMaxTiles;
  int shift = 0;
  for (int p = 0; p < plan.passes; ++p) {
    const int db = plan.digit_bits[p];
    const uint32_t bins = 1u << db;
    uint32_t* tot = sort_aux_tot(plan, aux, p);
    uint32_t* sup = sort_aux_sup(plan, aux, p);
    const int src = p & 1, dst = src ^ 1;
    const uint64_t* in = buf[src];
    const uint32_t* chist = hist;
    const uint32_t* ctot = tot;
    const uint32_t* csup = sup;
    uint32_t* hist_sup = scan_sup ? nullptr : sup;   // the scanned path builds sup from the histograms
    if (!(p == 0 && first_hist_done)) {
      if (wide)
        hipLaunchKernelGGL((sort_hist<kSortWideThreads>), dim3(plan.n_blocks), dim3(kSortWideThreads), 0, stream,
                           in, plan.n_max, n_dev, shift, bins, hist, hist_sup);
      else
        hipLaunchKernelGGL((sort_hist<kSortThreads>), dim3(plan.n_blocks), dim3(kSortThreads), 0, stream, in,
                           plan.n_max, n_dev, shift, bins, hist, hist_sup);
    }
    if (scan_sup) {
      hipLaunchKernelGGL(sort_sum_groups, dim3(plan.n_super), dim3(256), 0, stream, hist, plan.n_max, n_dev, bins,
                         sup);
      hipLaunchKernelGGL(sort_scan_groups, dim3((uint32_t)ceil_div(bins, 32)), dim3(1024), 0, stream, sup, tot,
                         bins, plan.n_super);
    }
#define HCTR_SCATTER(DB, NT, SC)                                                                         \
  hipLaunchKernelGGL((sort_scatter<DB, NT, SC>), dim3(plan.n_blocks), dim3(NT), 0, stream, in, buf[dst], \
                     plan.n_max, n_dev, shift, bins, chist, ctot, csup, plan.n_super)
    if (scan_sup) {   // an instantiation of its own: without the rows of the other scheme it needs fewer registers
      if (db <= 8) HCTR_SCATTER(8, kSortThreads, true);
      else HCTR_SCATTER(kSortMaxDigitBits, kSortThreads, true);
    } else if (db <= 8) HCTR_SCATTER(8, kSortThreads, false);   // the scatter measured faster with 256 threads
    else HCTR_SCATTER(kSortMaxDigitBits, kSortThreads, false);  // at every size
#undef HCTR_SCATTER
    shift += db;
  }
  return launch_status("radix_sort_u64");
}

}  // namespace hctr
