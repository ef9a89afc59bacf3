// Embedding layer forward (key -> row, gather, pool) and backward (dedup, segmented reduce, SGD)
// for gfx950.  Bandwidth-bound work: every lane moves 16 bytes per load, a table row is covered
// by a group of LPR adjacent lanes (LPR * 16 bytes >= row bytes), and several independent row
// loads are in flight per lane before the first use.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "rowvec.h"
#include "blockscan.h"
#include "hash_internal.h"

namespace hctr {

// Per-slot row ranges, passed by value in the kernel argument segment (2 KB).
struct SlotTable {
  int64_t base[HCTR_MAX_SLOTS];
  int64_t num[HCTR_MAX_SLOTS];
};

// The count of keys without a row is kept in kInvalidParts partial counters behind the header (a
// wave adds to the counter picked by its block index): thousands of waves adding to ONE address
// queue up behind each other (about 10 ns each), which cost milliseconds when a third of a batch's
// keys had no row.  The reader sums the parts.
constexpr uint32_t kInvalidParts = 1024;

// First 256 bytes of an embedding workspace; kInvalidParts 8-byte counters follow.
struct EmbHeader {
  unsigned long long mark;     // kEmbMark once hctr_emb_workspace_init has run on this memory
  long long num_unique;        // U of the last backward
  uint32_t n_valid;            // sorted positions holding a real row
  uint32_t n_long;             // rows whose carry is left to whole blocks (0 between backward calls)
  uint32_t carry_done;         // blocks of the carry kernel that have finished (0 between calls)
  uint32_t pad[57];
};
static_assert(sizeof(EmbHeader) == 256, "header is one 256-byte block");
constexpr size_t kEmbHeadBytes = sizeof(EmbHeader) + kInvalidParts * 8;
constexpr unsigned long long kEmbMark = 0x57424d4552544348ull;   // "HCTREMBW"

// Adds a wave's count of keys without a row (call with the wave's total in every lane).
__device__ __forceinline__ void add_invalid(EmbHeader* hdr, uint32_t wave_total) {
  if ((threadIdx.x & 63) == 0 && wave_total != 0)
    atomicAdd(reinterpret_cast<unsigned long long*>(hdr + 1) + (blockIdx.x & (kInvalidParts - 1)),
              (unsigned long long)wave_total);
}

// Resets the dedup part of the header and clears the counters that later kernels add to.
__global__ __launch_bounds__(256) void emb_init_header(EmbHeader* hdr, uint32_t* seg_off, int reset_invalid,
                                                       uint32_t* zero, uint32_t zero_count) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (reset_invalid && i < kInvalidParts) reinterpret_cast<unsigned long long*>(hdr + 1)[i] = 0;
  if (i == 0) {
    if (reset_invalid) hdr->mark = kEmbMark;
    hdr->num_unique = 0;
    hdr->n_valid = 0;
    hdr->n_long = 0;
    hdr->carry_done = 0;
    if (seg_off) seg_off[0] = 0;
  }
  if (i < zero_count) zero[i] = 0u;
}

// Order in which the forward kernels walk the bags.  n_samples == 0: in memory order (bag = sample *
// S + slot).  n_samples == batch: slot by slot (all samples of slot 0, then slot 1, ...): the chip
// then works on one table at a time and that table's hot rows stay in the 4 MB L2 of every XCD
// instead of sharing it with the other slots' (headline forward 226 -> 205 us, multi-hot forward
// 3.30 -> 2.85 ms).  The price is that consecutive work items write output rows S rows apart, so the
// host asks for it only from a certain size of the output row on: 256 bytes with one key per bag
// (fp16 rows of 128 columns: forward 0.113 -> 0.106-0.110 ms), 128 bytes with several keys per bag,
// where many rows are read per row written (the same rows pooled into an fp16 output: 1.47 -> 1.25 ms).
constexpr size_t kSlotMajorMinRowBytes = 256;
constexpr size_t kSlotMajorMinRowBytesCsr = 128;
__device__ __forceinline__ uint32_t walk_to_bag(uint32_t v, uint32_t n_bags, uint32_t S, uint32_t n_samples) {
  if (n_samples == 0 || v >= n_bags) return v;
  return (v % n_samples) * S + v / n_samples;
}

// ------------------------------------------------------------------------------------------------
// Forward, one key per bag: a group of LPR lanes copies U rows (U independent 16-byte loads per
// lane in flight), so a wave covers 64/LPR * U bags.  Measured on the 26-table workload of 512-byte
// rows, same buffers: 1 / 2 / 4 / 8 / 16 / 24 / 32 rows per group in blocks of 256 threads 253 /
// 205 / 191 / 188 / 184 / 194 / 214 us; 4 / 8 / 12 / 16 rows in blocks of 512 threads 188 / 185 /
// 184 / 197 us; 16 rows in blocks of 64 / 128 threads 194 / 192 us.  (A plain copy of the same size
// behaves the other way round: the fewer loads a thread has under way, the faster.  What the gather
// needs to hide is the chain key -> row address -> row.)
// ------------------------------------------------------------------------------------------------
constexpr int kOneHotRows = 16;          // U of the launch below
constexpr uint32_t kOneHotThreads = 256;
template <typename T, typename OutT, int LPR, int U, bool HASHED>
__global__ __launch_bounds__(kOneHotThreads) void fwd_onehot(const T* __restrict__ table, int D,
                                                  int64_t total_rows, const int64_t* __restrict__ keys,
                                                  const int64_t* __restrict__ rows64, uint32_t n_bags,
                                                  uint32_t S, uint32_t n_samples, const SlotTable slots,
                                                  OutT* __restrict__ out, EmbHeader* hdr) {
  constexpr int VEC = RowVec<T>::VEC;
  constexpr uint32_t kThreads = kOneHotThreads;
  const int sub = threadIdx.x % LPR;
  const uint32_t group0 = (blockIdx.x * kThreads + threadIdx.x) / LPR;
  const uint32_t n_groups = gridDim.x * (kThreads / LPR);
  const int col = blockIdx.y * (LPR * VEC) + sub * VEC;
  const bool active = col < D;
  uint32_t nbad = 0;  // counted by the first lane of each group
  __shared__ int64_t s_base[HCTR_MAX_SLOTS], s_num[HCTR_MAX_SLOTS];
  if (!HASHED) {   // slot ranges by LDS: a per-lane index into the kernel arguments would be a global load
    if (threadIdx.x < S) {
      s_base[threadIdx.x] = slots.base[threadIdx.x];
      s_num[threadIdx.x] = slots.num[threadIdx.x];
    }
    __syncthreads();
  }
  for (uint64_t bag0_64 = (uint64_t)group0 * U; bag0_64 < n_bags; bag0_64 += (uint64_t)n_groups * U) {
    const uint32_t bag0 = (uint32_t)bag0_64;
    int64_t row[U], in[U];
    uint32_t bags[U];
    // The U keys (hashed mode: rows) first, index clamped instead of a branch: a load whose value is
    // used under the same branch is waited for before the next one is issued, which put four key
    // latencies in a row ahead of the row loads.
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t bag = bags[u] = walk_to_bag(bag0 + u, n_bags, S, n_samples);
      const uint32_t bc = bag < n_bags ? bag : n_bags - 1;
      in[u] = HASHED ? rows64[bc] : keys[bc];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t bag = bags[u];
      const uint32_t s = (bag < n_bags ? bag : n_bags - 1) % S;
      const int64_t lim = HASHED ? total_rows : s_num[s];
      const int64_t add = HASHED ? 0 : s_base[s];
      const bool ok = bag < n_bags && in[u] >= 0 && in[u] < lim;
      row[u] = ok ? add + in[u] : -1;
      nbad += (sub == 0 && bag < n_bags && !ok) ? 1u : 0u;
    }
    // the U row pieces without a branch (a bag without a row, or a lane past the row's end, reads
    // the start of row 0 and is zeroed below), widened only after all of them are under way
    typename RowVec<T>::Raw raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      raw[u] = RowVec<T>::load_raw(table + ((row[u] >= 0 && active) ? row[u] * D + col : (int64_t)0));
    if constexpr (sizeof(T) == 2 && sizeof(OutT) == 2) {
      // fp16 rows into an fp16 output: the pieces go out as they came in (widening and rounding
      // back gives the same bits at sixteen conversions per piece)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        typename RowVec<T>::Raw x = raw[u];
        if (!(row[u] >= 0 && active)) x = typename RowVec<T>::Raw{0u, 0u, 0u, 0u};
        const uint32_t bag = bags[u];
        if (bag < n_bags && active)
          __builtin_nontemporal_store(x, reinterpret_cast<typename RowVec<T>::Raw*>(out + (int64_t)bag * D + col));
      }
    } else {
      float v[U][VEC];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        RowVec<T>::widen(raw[u], v[u]);
        if (!(row[u] >= 0 && active)) {
#pragma unroll
          for (int i = 0; i < VEC; ++i) v[u][i] = 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t bag = bags[u];
        if (bag < n_bags && active) {
          store_stream<VEC>(out + (int64_t)bag * D + col, v[u]);
        }
      }
    }
  }
  if (blockIdx.y == 0 && __ballot(nbad != 0) != 0) {  // rare: add the groups' counts across the wave
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) nbad += __shfl_xor(nbad, d);
    add_invalid(hdr, nbad);
  }
}

// ------------------------------------------------------------------------------------------------
// Forward, CSR bags: one wave per bag.  The wave's 64/LPR lane groups take the bag's keys round
// robin, U keys each per step; the groups' partial sums are staged in LDS and added in group order
// by group 0, which scales (mean) and writes the pooled row.
//
// With every row served by the caches the kernel takes 85 % of the time it takes on real keys: what
// bounds it is the number of vector instructions it issues, not memory.  So everything that is the
// same for the whole wave (bag, slot, offsets, loop bounds) is derived from scalar registers - the
// slot comes from blockIdx.z when the bags are walked slot by slot, which also spares two integer
// divisions per wave - and the steps in which every lane has a row to fetch, nearly all of them,
// take a path without per-row tests: the row id by one ds_bpermute at a precomputed index, the
// address by one 32 x 32 -> 64 bit multiply-add, then the adds.  Nothing crosses waves, so a wave
// past the end leaves at once and no wave waits for the longest bag of its block.
// ------------------------------------------------------------------------------------------------
template <typename T, typename OutT, int LPR, int U, bool HASHED>
__global__ __launch_bounds__(256) void fwd_csr(const T* __restrict__ table, int D, int64_t total_rows,
                                               const int64_t* __restrict__ keys,
                                               const int64_t* __restrict__ rows64,
                                               const int64_t* __restrict__ offsets, uint32_t n_bags,
                                               uint32_t S, uint32_t n_samples, const SlotTable slots, int mean,
                                               OutT* __restrict__ out, EmbHeader* hdr) {
  constexpr int VEC = RowVec<T>::VEC;
  constexpr int G = 64 / LPR;
  constexpr int STEP = G * U;   // keys of one step of the wave (a power of two)
  __shared__ float part[4][(G > 1 ? (G - 1) : 1) * LPR * VEC];
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane / LPR, sub = lane % LPR;
  const int col = blockIdx.y * (LPR * VEC) + sub * VEC;
  const bool active = col < D;
  const bool all_active = (int)((blockIdx.y + 1u) * (uint32_t)(LPR * VEC)) <= D;   // the whole wave holds columns
  uint32_t bag, s;
  if (n_samples != 0) {   // slot by slot: grid z is the slot, x the sample
    const uint32_t sample = blockIdx.x * 4u + wave;
    if (sample >= n_samples) return;
    s = blockIdx.z;
    bag = sample * S + s;
  } else {
    bag = blockIdx.x * 4u + wave;
    if (bag >= n_bags) return;
    s = bag % S;
  }
  const int64_t b0 = offsets[bag], b1 = offsets[bag + 1];
  int64_t base = 0, num = 0;
  if (!HASHED) {
    base = slots.base[s];
    num = slots.num[s];
  }
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  // 1.0f that the compiler cannot see through: acc + x written as fma(x, one, acc) is the same sum
  // bit for bit, and with fp16 rows the conversion rides along in the one instruction
  // (v_fma_mix_f32) instead of taking one of its own.
  const float one = D > 0 ? 1.0f : 0.0f;
  const char* lane_base = reinterpret_cast<const char*>(table) + (int64_t)col * (int64_t)sizeof(T);
  const uint32_t row_bytes = (uint32_t)D * (uint32_t)sizeof(T);
  uint32_t nbad = 0;
  // 64 keys at a time: one coalesced key load and one row computation per lane, then the groups
  // pick their rows from the lanes by shuffle, U row loads each in flight.
  for (int64_t c0 = b0; c0 < b1; c0 += 64) {
    const int cnt = b1 - c0 < 64 ? (int)(b1 - c0) : 64;
    uint32_t myrow = kNoRow;
    if (lane < cnt) {
      if (HASHED) {
        const int64_t r = rows64[c0 + lane];
        if (r >= 0 && r < total_rows) myrow = (uint32_t)r;
      } else {
        const int64_t k = keys[c0 + lane];
        if (k >= 0 && k < num) myrow = (uint32_t)(base + k);
      }
      nbad += myrow == kNoRow ? 1u : 0u;
    }
    int j0 = 0;
    if (all_active && __ballot(lane < cnt && myrow == kNoRow) == 0) {
      // whole steps: lane group g takes keys j0 + g, j0 + g + G, ... of the chunk, all of them there
      const int full = cnt & ~(STEP - 1);
      for (; j0 < full; j0 += STEP) {
        typename RowVec<T>::Raw raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t r = (uint32_t)__builtin_amdgcn_ds_bpermute((j0 + g + u * G) << 2, (int)myrow);
          raw[u] = RowVec<T>::load_raw(reinterpret_cast<const T*>(lane_base + (uint64_t)r * row_bytes));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float v[VEC];
          RowVec<T>::widen(raw[u], v);
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[i] = __builtin_fmaf(v[i], one, acc[i]);
        }
      }
      if (j0 < cnt) {
        // the chunk's last, partial step: the lanes past the chunk's end hold kNoRow, so a group
        // whose turn lies past the end picks that up, fetches the start of row 0 and leaves it out
        typename RowVec<T>::Raw raw[U];
        bool there[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t r = (uint32_t)__builtin_amdgcn_ds_bpermute((j0 + g + u * G) << 2, (int)myrow);
          there[u] = r != kNoRow;
          raw[u] = RowVec<T>::load_raw(reinterpret_cast<const T*>(lane_base + (uint64_t)(there[u] ? r : 0u) * row_bytes));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float v[VEC];
          RowVec<T>::widen(raw[u], v);
          if (there[u]) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = __builtin_fmaf(v[i], one, acc[i]);
          }
        }
        j0 = cnt;
      }
    }
    for (; j0 < cnt; j0 += STEP) {   // same trip count for every lane: the shuffles need all lanes
      uint32_t row[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int jj = j0 + g + u * G;
        row[u] = __shfl(myrow, jj < cnt ? jj : lane);
        if (jj >= cnt) row[u] = kNoRow;
      }
      // the U row pieces without a branch (no row, or a lane past the row's end: the start of row 0,
      // left out of the sum below), widened only after all of them are under way
      typename RowVec<T>::Raw raw[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        raw[u] = RowVec<T>::load_raw(table + ((row[u] != kNoRow && active) ? (int64_t)row[u] * D + col : (int64_t)0));
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float v[VEC];
        RowVec<T>::widen(raw[u], v);
        if (row[u] != kNoRow && active) {
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[i] = __builtin_fmaf(v[i], one, acc[i]);
        }
      }
    }
  }
  if (G > 1) {
    // The groups' sums meet in LDS, within the wave: a wave's LDS accesses are carried out in the
    // order it issues them, and the fences keep the compiler from moving the reads above the writes.
    if (g > 0) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) part[wave][((g - 1) * LPR + sub) * VEC + i] = acc[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (g == 0) {
#pragma unroll
      for (int gg = 1; gg < G; ++gg)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += part[wave][((gg - 1) * LPR + sub) * VEC + i];
    }
  }
  if (g == 0 && active) {
    if (mean && b1 > b0) {
      const float w = 1.0f / (float)(b1 - b0);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] *= w;
    }
    store_stream<VEC>(out + (int64_t)bag * D + col, acc);
  }
  if (blockIdx.y == 0 && __ballot(nbad != 0) != 0) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) nbad += __shfl_xor(nbad, d);
    add_invalid(hdr, nbad);
  }
}

// Low half of a sorted (row, bag) word.  A mean needs 1 / (keys of the bag) for every occurrence,
// and fetching the bag's two bounds from the offsets at that point is a random read per occurrence
// (it cost a fifth of the multi-hot reduction).  The key -> row kernel walks the keys in bag order
// and has the bounds at hand, so when bag numbers leave bag_bits < 32 the count goes into the bits
// above the bag number; a count too large for them is stored as 0 = "look it up".  bag_bits == 32:
// the low half is the bag number alone.
struct BagWord {
  static __device__ __forceinline__ uint32_t pack(uint32_t bag, uint32_t count, uint32_t bag_bits) {
    const uint32_t room = 32u - bag_bits;   // 4..31
    return bag | ((count >> room) == 0 ? count << bag_bits : 0u);
  }
  static __device__ __forceinline__ uint32_t bag(uint32_t low, uint32_t bag_bits) {
    return bag_bits < 32u ? low & ((1u << bag_bits) - 1u) : low;
  }
  static __device__ __forceinline__ uint32_t count(uint32_t low, uint32_t bag_bits) {   // 0: not stored
    return bag_bits < 32u ? low >> bag_bits : 0u;
  }
};

// ------------------------------------------------------------------------------------------------
// Backward step 1: per key, the 32-bit global row (or kNoRow) and the bag it belongs to.
// ------------------------------------------------------------------------------------------------
// Bag of every key of one 4096-key tile of a CSR batch, into LDS (bag + 1; the tile starts at key
// k0).  Two binary searches find the bags of the tile's first and last key; every bag in between
// marks the position where it starts (atomicMax: of several bags starting at one position - empty
// ones - the last owns the key); a running maximum over the positions fills in the rest.
template <int NT>
__device__ __forceinline__ void tile_bags(const int64_t* __restrict__ offsets, uint32_t n_bags, uint32_t k0,
                                          uint32_t k1, uint32_t* bagof /*[kSortTile]*/,
                                          uint32_t* lds /*[NT / 64 + 2]*/) {
  constexpr int PER = kSortTile / NT;    // consecutive positions per thread in the running maximum
  constexpr int NW = NT / 64;
  const uint32_t tid = threadIdx.x;
  for (uint32_t i = tid; i < kSortTile; i += NT) bagof[i] = 0;
  if (tid < 128) {
    // The bag with offsets[bag] <= k < offsets[bag + 1] - the last bag that starts at or before k -
    // for k = k0 (wave 0) and k = k1 - 1 (wave 1).  A wave narrows the range 64-fold per step (each
    // lane tests one pivot): 4 dependent loads for a million bags where a binary search needs 20.
    const int64_t k = tid < 64 ? k0 : k1 - 1;
    const uint32_t ln = tid & 63;
    uint32_t lo = 0, hi = n_bags - 1;   // the answer lies in [lo, hi]; offsets[lo] <= k throughout
    while (lo < hi) {
      const uint32_t step = (hi - lo) / 64 + 1;
      const uint64_t p = (uint64_t)lo + (uint64_t)ln * step;
      const bool at_or_before = p <= hi && offsets[p] <= k;
      const uint32_t j = (uint32_t)__popcll(__ballot(at_or_before)) - 1u;   // lane 0 always votes yes
      const uint64_t top = (uint64_t)lo + (uint64_t)(j + 1) * step - 1;
      lo += j * step;
      hi = top < hi ? (uint32_t)top : hi;
    }
    if (ln == 0) lds[NW + (tid >> 6)] = lo;
  }
  __syncthreads();
  const uint32_t b_lo = lds[NW], b_hi = lds[NW + 1];
  if (tid == 0) atomicMax(&bagof[0], b_lo + 1);
  for (uint32_t bag = b_lo + 1 + tid; bag <= b_hi; bag += NT) {
    const int64_t start = offsets[bag];
    if (start >= (int64_t)k0 && start < (int64_t)k1) atomicMax(&bagof[(uint32_t)start - k0], bag + 1);
  }
  __syncthreads();
  // inclusive running maximum, PER consecutive positions per thread
  uint32_t v[PER], m = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    v[i] = bagof[tid * PER + i];
    m = v[i] > m ? v[i] : m;
    v[i] = m;
  }
  uint32_t inc = m;  // wave-level inclusive max-scan of the thread maxima
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(inc, d);
    if (lane >= d && t > inc) inc = t;
  }
  if (lane == 63) lds[wave] = inc;
  __syncthreads();
  uint32_t before = __shfl_up(inc, 1);
  if (lane == 0) before = 0;
  for (int w = 0; w < wave; ++w) before = lds[w] > before ? lds[w] : before;
#pragma unroll
  for (int i = 0; i < PER; ++i) bagof[tid * PER + i] = v[i] > before ? v[i] : before;
  __syncthreads();
}

// NT = 256, or 1024 when there is only about one tile per compute unit.  PACK: the number of keys of
// the bag rides in the word's spare bits (see BagWord; needs offsets and bag_bits < 32).  A template
// choice because the extra loads cost registers that the plain kernel should not pay for.
template <int NT, bool PACK>
__global__ __launch_bounds__(NT) void bwd_rows(const int64_t* __restrict__ keys,
                                               const int64_t* __restrict__ rows64,
                                               const int64_t* __restrict__ offsets, uint32_t nnz,
                                               uint32_t n_bags, uint32_t S, const SlotTable slots,
                                               int64_t total_rows, uint64_t* __restrict__ kv,
                                               EmbHeader* hdr, uint32_t bins,
                                               uint32_t* __restrict__ hist, uint32_t* __restrict__ sup,
                                               uint32_t bag_bits) {
  // One sort tile per block, so the block can also deliver the tile's histogram of the first sort
  // digit (the low bits of the row) and spare the sort its first counting pass.
  __shared__ uint32_t h[1 << kSortMaxDigitBits];   // (four copies as in sort_hist cost occupancy here: slower)
  __shared__ uint32_t bagof[kSortTile];
  __shared__ uint32_t small[NT / 64 + 2];
  const uint32_t mask = bins - 1;
  const uint32_t k0 = blockIdx.x * kSortTile;
  const uint32_t k1 = nnz - k0 < kSortTile ? nnz : k0 + kSortTile;
  for (uint32_t d = threadIdx.x; d < bins; d += NT) h[d] = 0;
  __shared__ int64_t s_base[HCTR_MAX_SLOTS], s_num[HCTR_MAX_SLOTS];   // see fwd_onehot
  if (rows64 == nullptr && threadIdx.x < S) {
    s_base[threadIdx.x] = slots.base[threadIdx.x];
    s_num[threadIdx.x] = slots.num[threadIdx.x];
  }
  if (offsets != nullptr) tile_bags<NT>(offsets, n_bags, k0, k1, bagof, small);
  else __syncthreads();
  uint32_t nbad = 0;
  // the thread's keys (or rows) first, index clamped instead of a branch: all loads leave together
  constexpr int PER = (int)(kSortTile / NT);
  const int64_t* src = rows64 != nullptr ? rows64 : keys;
  int64_t in[PER];
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const uint32_t i = k0 + it * (uint32_t)NT + threadIdx.x;
    in[it] = src[i < nnz ? i : nnz - 1];
  }
  // the bounds of each key's bag; their low halves are enough, a call has fewer than 2^31 keys
  uint32_t first[PACK ? PER : 1], past[PACK ? PER : 1];
  if constexpr (PACK) {
    const uint32_t* low = reinterpret_cast<const uint32_t*>(offsets);
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const uint32_t i = k0 + it * (uint32_t)NT + threadIdx.x;
      const uint32_t bag = bagof[(i < nnz ? i : nnz - 1) - k0] - 1u;
      first[it] = low[2 * (uint64_t)bag];
      past[it] = low[2 * (uint64_t)bag + 2];
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // every load above is issued before the first use below
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const uint32_t i = k0 + it * (uint32_t)NT + threadIdx.x;
    if (i < nnz) {
      const uint32_t bag = offsets != nullptr ? bagof[i - k0] - 1u : i;
      int64_t row = -1;
      if (rows64 != nullptr) {
        const int64_t r = in[it];
        if (r >= 0 && r < total_rows) row = r;
      } else {
        const int64_t k = in[it];
        const uint32_t s = bag % S;
        if (k >= 0 && k < s_num[s]) row = s_base[s] + k;
      }
      const uint32_t r32 = row < 0 ? kNoRow : (uint32_t)row;
      nbad += row < 0 ? 1u : 0u;
      uint32_t low = bag;
      if constexpr (PACK) low = BagWord::pack(bag, past[it] - first[it], bag_bits);
      kv[i] = ((uint64_t)r32 << 32) | low;
      atomicAdd(&h[r32 & mask], 1u);
    }
  }
  __syncthreads();
  uint32_t* hrow = hist + (uint64_t)blockIdx.x * bins;
  uint32_t* srow = sup + (uint64_t)(blockIdx.x / kSortSuper) * bins;
  for (uint32_t d = threadIdx.x; d < bins; d += NT) {
    const uint32_t c = h[d];
    hrow[d] = c;
    if (c && sup) atomicAdd(&srow[d], c);
  }
  if (__ballot(nbad != 0) != 0) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) nbad += __shfl_xor(nbad, d);
    add_invalid(hdr, nbad);
  }
}

// Backward step 3: run boundaries of the sorted rows = the distinct rows of the batch.  A position
// starts a segment if it holds a real row that differs from its left neighbour.  Two kernels over
// tiles of 4096 positions (a wave owns a run of consecutive ones and finds starts 64 at a time with a
// ballot): the first counts the starts per tile and adds them to a per-64-tiles sum; the second
// derives its tile's first segment number from those, then numbers the starts and writes the
// unique rows, the segment offsets and, per position, the number of starts before it.
constexpr uint32_t kSegTile = 4096;
constexpr uint32_t kSegSuper = 64;

// The rows of a wave's ROUNDS * 64 consecutive sorted words plus the row before the first and after
// the last of them, all requested at once and without a branch (indices clamped; a load under a
// branch is waited for before the next one is issued, which made these kernels latency-bound).
// Words past the end count as kNoRow.  rows[0] = the row before, rows[1 + r] = round r's.
template <int ROUNDS>
__device__ __forceinline__ void seg_load_rows(const uint64_t* __restrict__ skv, uint32_t wbase, uint32_t n,
                                              uint32_t* rows /*[ROUNDS + 2]*/) {
  const int lane = threadIdx.x & 63;
  const uint32_t last = n - 1;   // n >= 1
  uint64_t w[ROUNDS + 2];
  const uint32_t before = wbase > 0 ? wbase - 1 : 0;
  w[0] = skv[before < last ? before : last];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const uint32_t idx = wbase + r * 64 + lane;
    w[1 + r] = skv[idx < last ? idx : last];
  }
  const uint32_t after = wbase + ROUNDS * 64;
  w[ROUNDS + 1] = skv[after < last ? after : last];
  __builtin_amdgcn_sched_barrier(0);   // every load above is issued before the first use below
  rows[0] = (wbase > 0 && wbase - 1 < n) ? (uint32_t)(w[0] >> 32) : kNoRow;
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) rows[1 + r] = wbase + r * 64 + lane < n ? (uint32_t)(w[1 + r] >> 32) : kNoRow;
  rows[ROUNDS + 1] = after < n ? (uint32_t)(w[ROUNDS + 1] >> 32) : kNoRow;
}

// Lanes of round r whose word starts a run of equal rows; prev63 = the row of the word just before
// the round's first (the previous round's last lane, or the row before the wave's range).
__device__ __forceinline__ uint64_t seg_start_mask(uint32_t row, uint32_t prev63, uint32_t idx) {
  const int lane = threadIdx.x & 63;
  uint32_t prev = __shfl_up(row, 1);
  if (lane == 0) prev = prev63;
  return __ballot(row != kNoRow && (idx == 0 || prev != row));
}

template <int NT>
__global__ __launch_bounds__(NT) void seg_count(const uint64_t* __restrict__ skv, uint32_t n,
                                                uint32_t* __restrict__ counts, uint32_t* __restrict__ segsup) {
  constexpr int NW = NT / 64, ROUNDS = kSegTile / NT;
  __shared__ uint32_t wsum[NW];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t wbase = blockIdx.x * kSegTile + wave * (ROUNDS * 64u);
  uint32_t rows[ROUNDS + 2];
  seg_load_rows<ROUNDS>(skv, wbase, n, rows);
  uint32_t c = 0, prev63 = rows[0];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    c += (uint32_t)__popcll(seg_start_mask(rows[1 + r], prev63, wbase + r * 64 + lane));
    prev63 = __shfl(rows[1 + r], 63);
  }
  if (lane == 0) wsum[wave] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += wsum[w];
    counts[blockIdx.x] = t;
    if (t) atomicAdd(&segsup[blockIdx.x / kSegSuper], t);
  }
}

template <int NT>
__global__ __launch_bounds__(NT) void seg_write(const uint64_t* __restrict__ skv, uint32_t n,
                                                const uint32_t* __restrict__ counts,
                                                const uint32_t* __restrict__ segsup,
                                                uint32_t* __restrict__ starts_before, uint32_t W,
                                                uint32_t* __restrict__ uniq,
                                                uint32_t* __restrict__ seg_off, EmbHeader* hdr) {
  constexpr int NW = NT / 64, ROUNDS = kSegTile / NT;
  __shared__ uint32_t red[NW];
  __shared__ uint32_t wsum[NW];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t tile = blockIdx.x;
  const uint32_t g = tile / kSegSuper;
  const uint32_t wbase = tile * kSegTile + wave * (ROUNDS * 64u);
  uint32_t rows[ROUNDS + 2];
  seg_load_rows<ROUNDS>(skv, wbase, n, rows);   // requested before the sums below: both in flight together
  // number of starts in all earlier tiles
  uint32_t part = 0;
  for (uint32_t i = threadIdx.x; i < g; i += NT) part += segsup[i];
  if (threadIdx.x < kSegSuper && g * kSegSuper + threadIdx.x < tile) part += counts[g * kSegSuper + threadIdx.x];
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d);
  if (lane == 0) red[wave] = part;

  uint64_t m[ROUNDS];
  uint32_t c = 0, prev63 = rows[0];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    m[r] = seg_start_mask(rows[1 + r], prev63, wbase + r * 64 + lane);
    prev63 = __shfl(rows[1 + r], 63);
    c += (uint32_t)__popcll(m[r]);
  }
  if (lane == 0) wsum[wave] = c;
  __syncthreads();
  uint32_t run = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) run += red[w];
  for (int w = 0; w < wave; ++w) run += wsum[w];
  const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const uint32_t p = wbase + r * 64 + lane;
    const uint32_t row = rows[1 + r];
    // the row to the right: the neighbouring lane's, or the next round's first / the row after the range
    uint32_t next = __shfl_down(row, 1);
    const uint32_t next0 = __shfl(rows[2 + r], 0);   // rows[ROUNDS + 1] is the same in every lane
    if (lane == 63) next = next0;
    if (p < n) {
      const uint32_t before = run + (uint32_t)__popcll(m[r] & below);
      const bool start = (m[r] >> lane) & 1ull;
      // the reduction asks for this count only at the last position of a window (W is a power of two)
      if (((p + 1) & (W - 1)) == 0) starts_before[p / W] = before;
      if (start) {
        uniq[before] = row;
        seg_off[before] = p;
      }
      if (row != kNoRow && (p == n - 1 || next == kNoRow)) {
        const uint32_t U = before + (start ? 1u : 0u);  // last real row closes the last segment
        seg_off[U] = p + 1;
        hdr->n_valid = p + 1;
        hdr->num_unique = (long long)U;
      }
    }
    run += (uint32_t)__popcll(m[r]);
  }
}

// ------------------------------------------------------------------------------------------------
// Where the backward kernels find an occurrence's gradient row and a row's storage.  UniformView:
// one fused table, every bag D wide, dY is [n_bags, D].  GroupView: a fused group of lookups of
// different widths over separate tables; dY is [batch, width_total] with lookup l at column
// col[l]; bag = sample * L + l; rows are numbered over the concatenation of the tables.
// ------------------------------------------------------------------------------------------------
struct GroupLookup {
  void* table;        // the lookup's table (several lookups may name the same one)
  uint32_t row_base;  // first row number of that table
  uint32_t col;       // first output column
  uint32_t dim;       // row width
  uint32_t mean;      // 1: mean combiner
};
static_assert(sizeof(GroupLookup) == 24, "kernel-argument layout");

template <typename T, typename DyT>
struct UniformView {
  static constexpr int kLds = 1;
  static constexpr bool kUniform = true;   // one table, one row width, one combiner for all bags
  T* table;
  float* master;   // fp32 copy of an fp16 table that takes the update (the table row is its rounding), or NULL
  const DyT* dY;
  int D;
  int mean;
  __device__ __forceinline__ const GroupLookup* stage(GroupLookup*) const { return nullptr; }
  __device__ __forceinline__ int dmax() const { return D; }
  __device__ __forceinline__ bool is_mean(uint32_t, const GroupLookup*) const { return mean != 0; }
  __device__ __forceinline__ const DyT* grad(uint32_t bag, const GroupLookup*, int* width) const {
    *width = D;
    return dY + (int64_t)bag * D;
  }

  __device__ __forceinline__ int row_width(uint32_t, const GroupLookup*) const { return D; }
  // four weights of row r at column col, widened to fp32 / written back
  __device__ __forceinline__ f32x4 load_weights(uint32_t r, uint32_t, const GroupLookup*, int col) const {
    if (master) return load4(master + (int64_t)r * D + col);
    return load_row4(table + (int64_t)r * D + col);
  }
  // the same in two steps, so that the caller can have several rows under way before it widens any
  __device__ __forceinline__ Raw4 load_weights_raw(uint32_t r, uint32_t, const GroupLookup*, int col) const {
    if (master) return load_raw4(master + (int64_t)r * D + col);
    return load_raw4(table + (int64_t)r * D + col);
  }
  __device__ __forceinline__ f32x4 widen_weights(const Raw4& x) const {
    if (master) return widen4(x, static_cast<const float*>(nullptr));
    return widen4(x, static_cast<const T*>(nullptr));
  }
  __device__ __forceinline__ void store_weights(uint32_t r, uint32_t, const GroupLookup*, int col, f32x4 x) const {
    if (master) store4(master + (int64_t)r * D + col, x);
    store_row4(table + (int64_t)r * D + col, x);
  }
};

template <typename T>
struct GroupView {
  static constexpr int kLds = HCTR_MAX_GROUP_LOOKUPS;
  static constexpr bool kUniform = false;
  const float* dY;
  uint32_t L;
  uint32_t width_total;
  int dmax_;
  GroupLookup lk[HCTR_MAX_GROUP_LOOKUPS];
  // The lookups go to LDS first: indexing the kernel arguments per lane would be a global load.
  __device__ __forceinline__ const GroupLookup* stage(GroupLookup* lds) const {
    if (threadIdx.x < L) lds[threadIdx.x] = lk[threadIdx.x];
    __syncthreads();
    return lds;
  }
  __device__ __forceinline__ int dmax() const { return dmax_; }
  __device__ __forceinline__ bool is_mean(uint32_t bag, const GroupLookup* l) const { return l[bag % L].mean != 0; }
  __device__ __forceinline__ const float* grad(uint32_t bag, const GroupLookup* l, int* width) const {
    const GroupLookup& k = l[bag % L];
    *width = (int)k.dim;
    return dY + (int64_t)(bag / L) * width_total + k.col;
  }
  __device__ __forceinline__ int row_width(uint32_t bag, const GroupLookup* l) const { return (int)l[bag % L].dim; }
  __device__ __forceinline__ f32x4 load_weights(uint32_t r, uint32_t bag, const GroupLookup* l, int col) const {
    const GroupLookup& k = l[bag % L];
    return load_row4(static_cast<const T*>(k.table) + (int64_t)(r - k.row_base) * k.dim + col);
  }
  __device__ __forceinline__ Raw4 load_weights_raw(uint32_t r, uint32_t bag, const GroupLookup* l, int col) const {
    const GroupLookup& k = l[bag % L];
    return load_raw4(static_cast<const T*>(k.table) + (int64_t)(r - k.row_base) * k.dim + col);
  }
  __device__ __forceinline__ f32x4 widen_weights(const Raw4& x) const {
    return widen4(x, static_cast<const T*>(nullptr));
  }
  __device__ __forceinline__ void store_weights(uint32_t r, uint32_t bag, const GroupLookup* l, int col,
                                                f32x4 x) const {
    const GroupLookup& k = l[bag % L];
    store_row4(static_cast<T*>(k.table) + (int64_t)(r - k.row_base) * k.dim + col, x);
  }
};

// A row that crosses window borders is finished after the reduction (see bwd_carry): by a lane group
// when at most kCarryShort windows follow the one that owns it, by a whole block otherwise.
constexpr uint32_t kCarryShort = 8;

__device__ __forceinline__ void carry_extent(const uint64_t* __restrict__ skv,
                                             const uint32_t* __restrict__ starts_before,
                                             const uint32_t* __restrict__ seg_off, uint32_t win, uint32_t W,
                                             uint32_t bag_bits, uint32_t* row, uint32_t* bag, uint32_t* last) {
  // a tail exists only when the window is full and its last row continues into the next window
  const uint32_t p = win * W + W - 1;
  const uint64_t w64 = skv[p];
  const uint32_t r = (uint32_t)(w64 >> 32);
  const uint32_t u = starts_before[win] + ((p == 0 || (uint32_t)(skv[p - 1] >> 32) != r) ? 1u : 0u) - 1u;
  *row = r;
  *bag = BagWord::bag((uint32_t)w64, bag_bits);   // any occurrence of the row names its table
  *last = (seg_off[u + 1] - 1u) / W;   // last window holding a piece of the row
}

// ------------------------------------------------------------------------------------------------
// Backward steps 4+5.  The sorted occurrence list is cut into windows of W positions; a group of
// LPR lanes (4 dY columns per lane) walks one window.  A row whose occurrences all lie inside the
// window is reduced and updated on the spot.  A row that crosses window borders leaves one partial
// sum per window ("head" if the row began in an earlier window, else "tail"), and the second kernel
// adds a row's partials in window order and applies the update.  Order of additions is fixed by
// the sorted positions, so results do not vary from run to run.
// ------------------------------------------------------------------------------------------------
// ONCE: one key per bag, so every gradient row is read exactly once and is loaded with a streaming
// load that keeps the caches for what is reused.  With several keys per bag the rows ARE reused (a
// multi-hot backward ran 45 % slower with streaming loads), so they are read the ordinary way.
template <typename T, int LPR, typename View, bool ONCE>
__global__ __launch_bounds__(256) void bwd_reduce_windows(
    const View view, const uint64_t* __restrict__ skv, EmbHeader* hdr,
    const int64_t* __restrict__ offsets, float lr, float* __restrict__ head, float* __restrict__ tail,
    uint8_t* __restrict__ tail_flag, uint32_t W, uint32_t bag_bits,
    uint32_t* __restrict__ long_list) {
  __shared__ GroupLookup lds_lk[View::kLds];
  const GroupLookup* lk = view.stage(lds_lk);
  const int sub = threadIdx.x % LPR;
  const uint32_t win = (blockIdx.x * 256u + threadIdx.x) / LPR;
  const int col = blockIdx.y * (LPR * 4) + sub * 4;
  const int DM = view.dmax();
  const uint32_t n_valid = hdr->n_valid;
  const uint64_t start64 = (uint64_t)win * W;
  if (start64 >= n_valid) return;
  const uint32_t start = (uint32_t)start64;
  const uint32_t end = (n_valid - start < W) ? n_valid : start + W;

  // Asked for now, used at the very end: the row at the start of window win + kCarryShort + 1.  If
  // it is the row that leaves this window, that row goes on for more than kCarryShort windows.
  const uint64_t far = (uint64_t)(win + kCarryShort + 1u) * W;
  const uint32_t far_row = (uint32_t)(skv[far < n_valid ? far : n_valid - 1u] >> 32);
  // `before`: the row being summed began in an earlier window (only the window's first row can).
  bool before = start > 0 && (uint32_t)(skv[start - 1] >> 32) == (uint32_t)(skv[start] >> 32);
  bool wrote_tail = false;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  constexpr int UB = 4;   // occurrences per step: UB dY loads (+ the table rows that finish) in flight
  // for the steps that only add (uniform views): this lane's piece of gradient row 0, the bytes of a
  // gradient row, the first lane of the group, and whether every lane of the wave holds columns
  typedef typename std::remove_const<typename std::remove_pointer<decltype(view.dY)>::type>::type DyPiece;
  const char* dy_lane = reinterpret_cast<const char*>(view.dY) + (int64_t)col * (int64_t)sizeof(DyPiece);
  const uint32_t dy_row_bytes = (uint32_t)DM * (uint32_t)sizeof(DyPiece);
  const uint32_t grp_lane0 = (threadIdx.x & 63u) & ~(uint32_t)(LPR - 1);
  const bool all_cols = (int)((blockIdx.y + 1u) * (uint32_t)(LPR * 4)) <= DM;

  for (uint32_t p0 = start; p0 < end; p0 += LPR) {
    const int cnt = (end - p0 < (uint32_t)LPR) ? (int)(end - p0) : LPR;
    // one coalesced load of LPR (row, bag) words, and of each word's right neighbour: a row whose
    // neighbour differs ends here, so its table row can be requested together with the dY rows
    uint32_t myrow = kNoRow, mynext = kNoRow, mybag = 0;
    float myw = 1.f;
    if (sub < cnt) {
      const uint64_t w64 = skv[p0 + sub];
      myrow = (uint32_t)(w64 >> 32);
      mybag = BagWord::bag((uint32_t)w64, bag_bits);
      if (p0 + sub + 1 < n_valid) mynext = (uint32_t)(skv[p0 + sub + 1] >> 32);
      if (view.is_mean(mybag, lk)) {
        const uint32_t stored = BagWord::count((uint32_t)w64, bag_bits);
        myw = 1.0f / (stored ? (float)stored : (float)(offsets[mybag + 1] - offsets[mybag]));
      }
    }
    // Positions at which a step cannot simply add: a run of equal rows ends there, or the chunk does.
    const uint64_t stops = __ballot(sub >= cnt || mynext != myrow);
    for (int q0 = 0; q0 < cnt; q0 += UB) {
      if constexpr (View::kUniform && !ONCE) {
        // Most occurrences of a batch with several keys per bag lie inside long runs of one row,
        // and there the kernel is bound by the vector instructions it issues.  A step in which no
        // group of the wave meets a stop only adds: bag (and weight) by one ds_bpermute each at a
        // precomputed index, the address by one multiply-add, the load, four adds.
        const uint32_t q0u = __builtin_amdgcn_readfirstlane(q0);
        constexpr uint64_t kGroupBit0 = LPR == 64 ? 1ull : 0xFFFFFFFFFFFFFFFFull / ((1ull << (LPR & 63)) - 1ull);
        const uint64_t step = (kGroupBit0 * ((1ull << UB) - 1ull)) << q0u;
        if ((stops & step) == 0 && all_cols) {
          Raw4 vr[UB];
          float w[UB];
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int at = (int)((grp_lane0 + q0u + (uint32_t)u) << 2);
            const uint32_t bg = (uint32_t)__builtin_amdgcn_ds_bpermute(at, (int)mybag);
            w[u] = view.mean ? __int_as_float(__builtin_amdgcn_ds_bpermute(at, __float_as_int(myw))) : 1.f;
            const DyPiece* g = reinterpret_cast<const DyPiece*>(dy_lane + (uint64_t)bg * dy_row_bytes);
            if constexpr (ONCE) vr[u] = load_stream_raw4(g);
            else vr[u] = load_raw4(g);
          }
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const f32x4 v = widen4(vr[u], static_cast<const DyPiece*>(nullptr));
            acc.x += w[u] * v.x; acc.y += w[u] * v.y;
            acc.z += w[u] * v.z; acc.w += w[u] * v.w;
          }
          continue;
        }
      }
      // All loads of the step raw and first - the UB gradient pieces without a branch (a lane past
      // the row's width reads the row's first piece and leaves it out), the table rows that end
      // here under their branch but with nothing else in it - and widened only afterwards.
      uint32_t r[UB], b[UB];
      bool ends[UB], in_row[UB];
      float w[UB];
      Raw4 vr[UB], tr[UB];
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        const bool live = q0 + u < cnt;
        const int q = live ? q0 + u : q0;  // clamp: dead positions are ignored below
        r[u] = __shfl(myrow, q, LPR);
        ends[u] = live && __shfl(mynext, q, LPR) != r[u];
        b[u] = __shfl(mybag, q, LPR);
        w[u] = __shfl(myw, q, LPR);
        int width;
        const auto* g = view.grad(b[u], lk, &width);
        in_row[u] = col < width;
        if constexpr (ONCE) vr[u] = load_stream_raw4(g + (in_row[u] ? col : 0));
        else vr[u] = load_raw4(g + (in_row[u] ? col : 0));
      }
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        tr[u] = Raw4{u32x4{0u, 0u, 0u, 0u}};
        if (ends[u] && in_row[u]) tr[u] = view.load_weights_raw(r[u], b[u], lk, col);
      }
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        int width;
        const f32x4 v = widen4(vr[u], view.grad(b[u], lk, &width));   // the pointer only names the type
        if (q0 + u < cnt && in_row[u]) {
          acc.x += w[u] * v.x; acc.y += w[u] * v.y;
          acc.z += w[u] * v.z; acc.w += w[u] * v.w;
        }
        if (ends[u]) {
          if (in_row[u]) {
            if (before) {
              store4(head + (int64_t)win * DM + col, acc);
            } else {
              f32x4 t = view.widen_weights(tr[u]);
              t.x -= lr * acc.x; t.y -= lr * acc.y; t.z -= lr * acc.z; t.w -= lr * acc.w;
              view.store_weights(r[u], b[u], lk, col, t);
            }
          }
          acc = f32x4{0.f, 0.f, 0.f, 0.f};
          before = false;
        }
      }
    }
  }
  // the last row of the window continues in the next window
  const bool continues = end < n_valid && (uint32_t)(skv[end] >> 32) == (uint32_t)(skv[end - 1] >> 32);
  if (continues) {
    if (col < DM) store4((before ? head : tail) + (int64_t)win * DM + col, acc);
    wrote_tail = !before;
  }
  if (sub == 0 && blockIdx.y == 0) {
    tail_flag[win] = wrote_tail ? 1 : 0;
    // this window owns a row that goes on: list it if it goes on for long (the rows are sorted, so
    // it does exactly when it still is the row kCarryShort + 1 windows further on)
    if (wrote_tail && far < n_valid && far_row == (uint32_t)(skv[end - 1] >> 32))
      long_list[atomicAdd(&hdr->n_long, 1u)] = win;
  }
}

// Rows that cross window borders.  The window holding a row's first piece owns the row; its last
// window follows from seg_off.  One kernel, two kinds of blocks that do not depend on each other.
// Rows with more than kCarryShort following windows were listed by the reduction kernel; the first
// long_blocks blocks (first, so that they start at once: they run longest) give each of them a
// whole block: the lane groups each add a contiguous share of the partials, the shares are staged
// in LDS and added in group order.  The other blocks give every window a lane group: an owner with
// at most kCarryShort following windows adds their partials itself (all loads in flight at once)
// and updates the row.  Which row lands where in the list does not
// matter: every row's additions happen in an order fixed by its length alone.
template <typename View, int LPR>
__device__ __forceinline__ void carry_short_rows(const View& view, const GroupLookup* lk,
                                                 const uint64_t* __restrict__ skv,
                                                 const uint32_t* __restrict__ starts_before,
                                                 const uint32_t* __restrict__ seg_off, uint32_t n_valid, float lr,
                                                 const float* __restrict__ head, const float* __restrict__ tail,
                                                 const uint8_t* __restrict__ tail_flag, uint32_t W,
                                                 uint32_t bag_bits, uint32_t block) {
  const int sub = threadIdx.x % LPR;
  const uint32_t win = (block * 1024u + threadIdx.x) / LPR;
  const int col = blockIdx.y * (LPR * 4) + sub * 4;
  const int DM = view.dmax();
  if ((uint64_t)win * W >= n_valid) return;
  if (!tail_flag[win]) return;
  uint32_t r, bag, last;
  carry_extent(skv, starts_before, seg_off, win, W, bag_bits, &r, &bag, &last);
  const uint32_t cnt = last - win;   // following windows, each with a head partial
  if (cnt > kCarryShort) return;     // on the list of long rows
  const bool active = col < view.row_width(bag, lk);
  f32x4 h[kCarryShort];
#pragma unroll
  for (uint32_t k = 0; k < kCarryShort; ++k)
    h[k] = (active && k < cnt) ? load4(head + (int64_t)(win + 1 + k) * DM + col) : f32x4{0.f, 0.f, 0.f, 0.f};
  if (active) {
    f32x4 tot = load4(tail + (int64_t)win * DM + col);
#pragma unroll
    for (uint32_t k = 0; k < kCarryShort; ++k) { tot.x += h[k].x; tot.y += h[k].y; tot.z += h[k].z; tot.w += h[k].w; }
    f32x4 x = view.load_weights(r, bag, lk, col);
    x.x -= lr * tot.x; x.y -= lr * tot.y; x.z -= lr * tot.z; x.w -= lr * tot.w;
    view.store_weights(r, bag, lk, col, x);
  }
}

template <typename View, int LPR>
__device__ __forceinline__ void carry_long_rows(const View& view, const GroupLookup* lk,
                                                const uint64_t* __restrict__ skv,
                                                const uint32_t* __restrict__ starts_before,
                                                const uint32_t* __restrict__ seg_off, uint32_t n_long, float lr,
                                                const float* __restrict__ head, const float* __restrict__ tail,
                                                uint32_t W, const uint32_t* __restrict__ long_list,
                                                uint32_t bag_bits, uint32_t n_blocks,
                                                f32x4* part /*[1024], LDS*/) {
  constexpr int NG = 1024 / LPR;
  const int sub = threadIdx.x % LPR, g = threadIdx.x / LPR;
  const int col = blockIdx.y * (LPR * 4) + sub * 4;
  const int DM = view.dmax();
  for (uint32_t i = blockIdx.x; i < n_long; i += n_blocks) {   // block-uniform loop
    const uint32_t win = long_list[i];
    uint32_t r, bag, last;
    carry_extent(skv, starts_before, seg_off, win, W, bag_bits, &r, &bag, &last);
    const bool active = col < view.row_width(bag, lk);
    const uint32_t cnt = last - win;
    const uint32_t share = (cnt + NG - 1) / NG;
    const uint32_t f0 = win + 1 + g * share;
    const uint32_t f1 = (f0 + share < last + 1) ? f0 + share : last + 1;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t w2 = f0; w2 < f1; w2 += 8) {
      f32x4 h[8];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        h[k] = (active && w2 + k < f1) ? load4(head + (int64_t)(w2 + k) * DM + col) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < 8; ++k) { acc.x += h[k].x; acc.y += h[k].y; acc.z += h[k].z; acc.w += h[k].w; }
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    if (g == 0 && active) {
      f32x4 tot = load4(tail + (int64_t)win * DM + col);
#pragma unroll 8
      for (int gg = 0; gg < NG; ++gg) {
        const f32x4 q = part[gg * LPR + sub];
        tot.x += q.x; tot.y += q.y; tot.z += q.z; tot.w += q.w;
      }
      f32x4 x = view.load_weights(r, bag, lk, col);
      x.x -= lr * tot.x; x.y -= lr * tot.y; x.z -= lr * tot.z; x.w -= lr * tot.w;
      view.store_weights(r, bag, lk, col, x);
    }
    __syncthreads();   // part is reused by the next row
  }
}

template <typename T, int LPR, typename View>
__global__ __launch_bounds__(1024) void bwd_carry(
    const View view, const uint64_t* __restrict__ skv, const uint32_t* __restrict__ starts_before,
    const uint32_t* __restrict__ seg_off, EmbHeader* hdr, float lr, const float* __restrict__ head,
    const float* __restrict__ tail, const uint8_t* __restrict__ tail_flag, uint32_t W,
    const uint32_t* __restrict__ long_list, uint32_t bag_bits, uint32_t long_blocks) {
  __shared__ f32x4 part[1024];
  __shared__ GroupLookup lds_lk[View::kLds];
  const GroupLookup* lk = view.stage(lds_lk);
  if (blockIdx.x >= long_blocks) {
    carry_short_rows<View, LPR>(view, lk, skv, starts_before, seg_off, hdr->n_valid, lr, head, tail, tail_flag, W,
                                bag_bits, blockIdx.x - long_blocks);
    return;
  }
  carry_long_rows<View, LPR>(view, lk, skv, starts_before, seg_off, hdr->n_long, lr, head, tail, W, long_list,
                             bag_bits, long_blocks, part);
  // Only these blocks read the list's length, and past this barrier every thread of the block has:
  // the block that is counted last empties the list for the next call.
  __syncthreads();
  if (threadIdx.x == 0 && atomicAdd(&hdr->carry_done, 1u) == long_blocks * gridDim.y - 1u) {
    hdr->n_long = 0;
    hdr->carry_done = 0;
  }
}

// ------------------------------------------------------------------------------------------------
// Fused group of lookups over tables of different widths.  Forward: a thread owns four adjacent
// output columns of one sample (one lookup's quad), walks that bag's keys with four row loads in
// flight and writes its quad once; the lanes of a lookup read the same keys (one request per
// wave) and adjacent 16-byte pieces of the same rows, and a wave's stores are contiguous whatever
// the widths are.
// ------------------------------------------------------------------------------------------------
struct GroupFwdArgs {
  uint32_t L;
  uint32_t width_total;
  uint32_t per_sample;                          // dense input: keys per sample; 0 = CSR offsets are given
  GroupLookup lk[HCTR_MAX_GROUP_LOOKUPS];
  uint32_t num_rows[HCTR_MAX_GROUP_LOOKUPS];    // rows of the lookup's table
  uint32_t before[HCTR_MAX_GROUP_LOOKUPS];      // dense input: keys of a sample before lookup l
  uint32_t hot[HCTR_MAX_GROUP_LOOKUPS];         // dense input: keys of lookup l per sample
};

// A thread works on NQ quads at a time (the same columns of NQ samples a grid stride apart) and
// keeps one key and one row load per quad in flight; with dense input the bag bounds are computed,
// not loaded, so a one-hot lookup costs two dependent loads (key, row), NQ-fold overlapped.
// FIXED: the grid's thread count is a multiple of the quads of a sample, so a thread keeps its
// columns from one step to the next: which lookup owns them (a binary search), that lookup's table,
// width, row count and combiner are found once per thread instead of once per quad, and a step is
// left with the loads, the adds and three multiply-adds for its addresses.
template <typename T, int NQ, bool FIXED>
__global__ __launch_bounds__(256) void fwd_group(const GroupFwdArgs a, const int64_t* __restrict__ keys,
                                                 const int64_t* __restrict__ offsets, uint64_t n_quads,
                                                 float* __restrict__ out, EmbHeader* hdr) {
  __shared__ GroupLookup lk[HCTR_MAX_GROUP_LOOKUPS];
  __shared__ uint32_t nrows[HCTR_MAX_GROUP_LOOKUPS], before[HCTR_MAX_GROUP_LOOKUPS], hot[HCTR_MAX_GROUP_LOOKUPS];
  if (threadIdx.x < a.L) {
    lk[threadIdx.x] = a.lk[threadIdx.x];
    nrows[threadIdx.x] = a.num_rows[threadIdx.x];
    before[threadIdx.x] = a.before[threadIdx.x];
    hot[threadIdx.x] = a.hot[threadIdx.x];
  }
  __syncthreads();
  const uint32_t W4 = a.width_total / 4;
  const uint64_t n_threads = (uint64_t)gridDim.x * 256u;
  const bool dense = a.per_sample != 0;
  uint32_t nbad = 0;   // counted by the lane that owns a lookup's first quad
  // the lookup that owns column c: the last one starting at or before it
  auto owner = [&](uint32_t c) {
    int lo = 0, hi = (int)a.L - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (lk[mid].col <= c) lo = mid; else hi = mid - 1;
    }
    return lo;
  };
  if constexpr (FIXED) {
    const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    const uint32_t c = (uint32_t)(t % W4) * 4u;
    const uint32_t batch = (uint32_t)(n_quads / W4);
    const uint32_t bstride = (uint32_t)(n_threads / W4);
    const int lo = owner(c);
    const GroupLookup k = lk[lo];
    const T* tbl = static_cast<const T*>(k.table);
    const uint32_t cl = c - k.col, dim = k.dim;
    const int64_t nr = nrows[lo];
    const uint32_t bef = before[lo], hot_l = hot[lo];
    for (uint32_t b0 = (uint32_t)(t / W4); b0 < batch; b0 += bstride * NQ) {
      int64_t k0[NQ], k1[NQ];
      bool live[NQ];
      int64_t longest = 0;
#pragma unroll
      for (int u = 0; u < NQ; ++u) {
        const uint32_t b = b0 + (uint32_t)u * bstride;
        live[u] = b < batch;
        const uint32_t bb = live[u] ? b : b0;
        if (dense) {
          k0[u] = (int64_t)bb * a.per_sample + bef;
          k1[u] = k0[u] + hot_l;
        } else {
          const uint64_t bag = (uint64_t)bb * a.L + (uint32_t)lo;
          k0[u] = offsets[bag];
          k1[u] = offsets[bag + 1];
        }
        if (!live[u]) k1[u] = k0[u];   // nothing to read, nothing to write
        if (k1[u] - k0[u] > longest) longest = k1[u] - k0[u];
      }
      f32x4 acc[NQ];
#pragma unroll
      for (int u = 0; u < NQ; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int64_t j = 0; j < longest; ++j) {
        int64_t key[NQ];
#pragma unroll
        for (int u = 0; u < NQ; ++u) key[u] = k0[u] + j < k1[u] ? keys[k0[u] + j] : (int64_t)-1;
        Raw4 raw[NQ];
        bool ok[NQ];
#pragma unroll
        for (int u = 0; u < NQ; ++u) {
          ok[u] = key[u] >= 0 && key[u] < nr;
          raw[u] = load_raw4(tbl + (ok[u] ? key[u] : 0) * dim + cl);
        }
#pragma unroll
        for (int u = 0; u < NQ; ++u) {
          const f32x4 v = widen4(raw[u], tbl);
          nbad += (cl == 0 && k0[u] + j < k1[u] && !ok[u]) ? 1u : 0u;
          if (ok[u]) { acc[u].x += v.x; acc[u].y += v.y; acc[u].z += v.z; acc[u].w += v.w; }
        }
      }
#pragma unroll
      for (int u = 0; u < NQ; ++u) {
        if (live[u]) {
          if (k.mean && k1[u] > k0[u]) {
            const float w = 1.0f / (float)(k1[u] - k0[u]);
            acc[u].x *= w; acc[u].y *= w; acc[u].z *= w; acc[u].w *= w;
          }
          const uint32_t b = b0 + (uint32_t)u * bstride;
          __builtin_nontemporal_store(acc[u], reinterpret_cast<f32x4*>(out + (uint64_t)b * a.width_total + c));
        }
      }
    }
  } else {
  for (uint64_t q0 = (uint64_t)blockIdx.x * 256u + threadIdx.x; q0 < n_quads; q0 += n_threads * NQ) {
    const T* tbl[NQ];
    uint32_t cl[NQ], dim[NQ], mean[NQ];
    int64_t nr[NQ], k0[NQ], k1[NQ];
    uint64_t dst[NQ];
    int64_t longest = 0;
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
      const uint64_t q = q0 + (uint64_t)u * n_threads;
      const bool live = q < n_quads;
      const uint64_t qq = live ? q : q0;
      const uint32_t b = (uint32_t)(qq / W4);
      const uint32_t c = (uint32_t)(qq % W4) * 4u;
      const int lo = owner(c);
      const GroupLookup k = lk[lo];
      tbl[u] = static_cast<const T*>(k.table);
      cl[u] = c - k.col;
      dim[u] = k.dim;
      mean[u] = k.mean;
      nr[u] = nrows[lo];
      dst[u] = (uint64_t)b * a.width_total + c;
      if (dense) {
        k0[u] = (int64_t)b * a.per_sample + before[lo];
        k1[u] = k0[u] + hot[lo];
      } else {
        const uint64_t bag = (uint64_t)b * a.L + (uint32_t)lo;
        k0[u] = offsets[bag];
        k1[u] = offsets[bag + 1];
      }
      if (!live) k1[u] = k0[u];   // nothing to read, nothing to write
      if (k1[u] - k0[u] > longest) longest = k1[u] - k0[u];
    }
    f32x4 acc[NQ];
#pragma unroll
    for (int u = 0; u < NQ; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int64_t j = 0; j < longest; ++j) {
      int64_t key[NQ];
#pragma unroll
      for (int u = 0; u < NQ; ++u) key[u] = k0[u] + j < k1[u] ? keys[k0[u] + j] : (int64_t)-1;
      // the NQ row pieces raw and without a branch (a key with no row reads row 0 and is left out),
      // widened once all are under way: see RowVec
      Raw4 raw[NQ];
      bool ok[NQ];
#pragma unroll
      for (int u = 0; u < NQ; ++u) {
        ok[u] = key[u] >= 0 && key[u] < nr[u];
        raw[u] = load_raw4(tbl[u] + (ok[u] ? key[u] : 0) * dim[u] + cl[u]);
      }
#pragma unroll
      for (int u = 0; u < NQ; ++u) {
        const f32x4 v = widen4(raw[u], tbl[u]);
        nbad += (cl[u] == 0 && k0[u] + j < k1[u] && !ok[u]) ? 1u : 0u;
        if (ok[u]) { acc[u].x += v.x; acc[u].y += v.y; acc[u].z += v.z; acc[u].w += v.w; }
      }
    }
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
      if (q0 + (uint64_t)u * n_threads < n_quads) {
        if (mean[u] && k1[u] > k0[u]) {
          const float w = 1.0f / (float)(k1[u] - k0[u]);
          acc[u].x *= w; acc[u].y *= w; acc[u].z *= w; acc[u].w *= w;
        }
        __builtin_nontemporal_store(acc[u], reinterpret_cast<f32x4*>(out + dst[u]));
      }
    }
  }
  }
  if (__ballot(nbad != 0) != 0) {   // every lane of the wave is here: the loops above have no early exit
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) nbad += __shfl_xor(nbad, d);
    add_invalid(hdr, nbad);
  }
}

// Dense input: the CSR offsets of `batch` samples that each bring hot[l] keys for lookup l.
struct GroupHotness {
  uint32_t L;
  uint32_t per_sample;                            // sum of the hotness values
  uint32_t before[HCTR_MAX_GROUP_LOOKUPS];        // keys of a sample before lookup l
};
__global__ __launch_bounds__(256) void group_dense_offsets(const GroupHotness h, uint64_t n_bags,
                                                           int64_t* __restrict__ offsets) {
  __shared__ uint32_t before[HCTR_MAX_GROUP_LOOKUPS];
  if (threadIdx.x < h.L) before[threadIdx.x] = h.before[threadIdx.x];
  __syncthreads();
  const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (i < n_bags) offsets[i] = (int64_t)(i / h.L) * h.per_sample + before[i % h.L];
  if (i == n_bags) offsets[i] = (int64_t)(n_bags / h.L) * h.per_sample;
}

// Counts the violations of the CSR contract: offsets[0] = 0, offsets[n_bags] = nnz, non-decreasing.
__global__ __launch_bounds__(256) void check_offsets(const int64_t* __restrict__ offsets, uint64_t n_bags,
                                                     int64_t nnz, unsigned long long* bad) {
  __shared__ uint32_t blk;
  if (threadIdx.x == 0) blk = 0;
  __syncthreads();
  uint32_t mine = 0;
  for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i <= n_bags; i += (uint64_t)gridDim.x * 256u) {
    const int64_t o = offsets[i];
    if (i == 0 && o != 0) ++mine;
    if (i == n_bags && o != nnz) ++mine;
    if (i < n_bags && offsets[i + 1] < o) ++mine;
  }
  if (mine) atomicAdd(&blk, mine);
  __syncthreads();
  if (threadIdx.x == 0 && blk) atomicAdd(bad, (unsigned long long)blk);
}

// ------------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------------
struct EmbLayout {
  // byte offsets into the workspace (all multiples of 256)
  size_t header, kv0, kv1, hist, aux, seg_counts, flags, uniq, seg_off, long_list, head, tail,
      tail_flag, rows64, hash_ws, extra, total;
  uint32_t window, n_windows, seg_tiles, seg_super;
  int sort_bits;
  SortPlan sort;
};

constexpr int64_t kWindowSwitch = 8ll << 20;
static uint32_t pick_window(int64_t nnz) { return nnz <= kWindowSwitch ? 64u : 256u; }   // powers of two (seg_write)

// Workspace of a layer or a group: total_rows rows in all, widest row dmax, hashed = with the
// key -> row scratch of the hashed mode, extra = bytes appended for the caller (group: CSR offsets).
static EmbLayout emb_layout_raw(int64_t total_rows, int dmax, int64_t nnz_max, bool hashed, size_t extra) {
  EmbLayout L{};
  const size_t n = (size_t)(nnz_max > 0 ? nnz_max : 1);
  Carver c(nullptr);
  auto at = [&](size_t bytes) { size_t o = c.off; c.take<char>(bytes); return o; };
  L.sort_bits = ceil_log2((uint64_t)total_rows + 1);
  L.sort = sort_plan((uint32_t)n, L.sort_bits);
  L.window = pick_window(nnz_max);
  L.n_windows = (uint32_t)ceil_div((int64_t)n, L.window);
  L.header = at(kEmbHeadBytes);
  L.kv0 = at(n * 8); L.kv1 = at(n * 8);
  L.hist = at(L.sort.hist_count * 4);
  L.seg_tiles = (uint32_t)ceil_div((int64_t)n, kSegTile);
  L.seg_super = (uint32_t)ceil_div(L.seg_tiles, kSegSuper);
  L.aux = at((L.sort.aux_count + L.seg_super) * 4);   // sort sums, then the per-64-tiles start counts
  L.seg_counts = at((size_t)L.seg_tiles * 4);
  L.flags = at((size_t)L.n_windows * 4);   // per window: distinct rows that begin before its last position
  L.uniq = at(n * 4);
  L.seg_off = at((n + 1) * 4);
  L.long_list = at((size_t)L.n_windows * 4);
  L.head = at((size_t)L.n_windows * dmax * 4);
  L.tail = at((size_t)L.n_windows * dmax * 4);
  L.tail_flag = at(L.n_windows);
  if (hashed) {
    L.rows64 = at(n * 8);
    L.hash_ws = at(hash_ws_bytes((int64_t)n));
  }
  if (extra) L.extra = at(extra);
  L.total = c.off;
  return L;
}

static EmbLayout emb_layout(const hctr_emb_desc* d, int64_t nnz_max) {
  return emb_layout_raw(d->total_rows, d->dim, nnz_max, d->hash != nullptr, 0);
}

// Bytes that serve every call of up to nnz_max keys.  A call lays the workspace out from its own
// key count, and the layout grows with it except where the reduction window widens: a call just
// below that switch has four times the windows (and partial-sum rows) of a call just above it.
static size_t emb_bytes_upto(int64_t total_rows, int dmax, int64_t nnz_max, bool hashed, size_t extra) {
  size_t need = emb_layout_raw(total_rows, dmax, nnz_max, hashed, extra).total;
  if (nnz_max > kWindowSwitch) need = std::max(need, emb_layout_raw(total_rows, dmax, kWindowSwitch, hashed, extra).total);
  return need;
}

static hctr_status validate_desc(const hctr_emb_desc* d) {
  if (!d) return fail(HCTR_E_NULL_PTR, "desc is NULL");
  if (d->num_slots < 1 || d->num_slots > HCTR_MAX_SLOTS)
    return fail(HCTR_E_INVALID_ARG, "num_slots %d outside 1..%d", d->num_slots, HCTR_MAX_SLOTS);
  if (d->table_dtype != HCTR_F32 && d->table_dtype != HCTR_F16)
    return fail(HCTR_E_INVALID_ARG, "table_dtype %d unknown", d->table_dtype);
  const int mult = d->table_dtype == HCTR_F32 ? 4 : 8;
  if (d->dim <= 0 || d->dim % mult != 0)
    return fail(HCTR_E_INVALID_ARG, "dim %d must be a positive multiple of %d", d->dim, mult);
  if (d->combiner != HCTR_SUM && d->combiner != HCTR_MEAN)
    return fail(HCTR_E_INVALID_ARG, "combiner %d unknown", d->combiner);
  if (d->io_dtype != HCTR_F32 && d->io_dtype != HCTR_F16)
    return fail(HCTR_E_INVALID_ARG, "io_dtype %d unknown", d->io_dtype);
  if (d->master) {
    if (d->table_dtype != HCTR_F16) return fail(HCTR_E_INVALID_ARG, "master rows go with an fp16 table only");
    if ((uintptr_t)d->master % 16 != 0) return fail(HCTR_E_INVALID_ARG, "master must be 16-byte aligned");
  }
  if (!d->table) return fail(HCTR_E_NULL_PTR, "table is NULL");
  if ((uintptr_t)d->table % 16 != 0) return fail(HCTR_E_INVALID_ARG, "table must be 16-byte aligned");
  if (d->total_rows < 1 || d->total_rows > 0xFFFFFFFEll)
    return fail(HCTR_E_UNSUPPORTED, "total_rows %lld outside 1..2^32-2", (long long)d->total_rows);
  if (d->hash) {
    if (d->total_rows < d->hash->max_rows)
      return fail(HCTR_E_INVALID_ARG, "table has %lld rows, the hash can hand out %lld",
                  (long long)d->total_rows, (long long)d->hash->max_rows);
  } else {
    if (!d->slot_row_base || !d->slot_num_rows)
      return fail(HCTR_E_NULL_PTR, "slot_row_base / slot_num_rows is NULL in direct mode");
    for (int s = 0; s < d->num_slots; ++s) {
      if (d->slot_row_base[s] < 0 || d->slot_num_rows[s] < 0 ||
          d->slot_row_base[s] + d->slot_num_rows[s] > d->total_rows)
        return fail(HCTR_E_INVALID_ARG, "slot %d rows [%lld, +%lld) leave the table of %lld rows", s,
                    (long long)d->slot_row_base[s], (long long)d->slot_num_rows[s],
                    (long long)d->total_rows);
    }
  }
  return HCTR_OK;
}

static hctr_status validate_batch(const hctr_emb_desc* d, int64_t batch, const int64_t* keys,
                                  const int64_t* offsets, int64_t nnz, const void* io, void* ws,
                                  size_t ws_bytes, EmbLayout* L, bool need_io = true,
                                  bool need_keys = true) {
  HCTR_TRY(validate_desc(d));
  if (batch < 0 || nnz < 0) return fail(HCTR_E_INVALID_ARG, "batch %lld / nnz %lld negative",
                                        (long long)batch, (long long)nnz);
  const int64_t n_bags = batch * d->num_slots;
  if (n_bags >= (1ll << 31) || nnz >= (1ll << 31))
    return fail(HCTR_E_UNSUPPORTED, "more than 2^31-1 bags or keys in one call");
  if (!offsets && nnz != n_bags)
    return fail(HCTR_E_INVALID_ARG, "offsets == NULL needs nnz == batch*num_slots (%lld != %lld)",
                (long long)nnz, (long long)n_bags);
  if (batch == 0 && nnz != 0) return fail(HCTR_E_INVALID_ARG, "nnz must be 0 when batch is 0");
  if (nnz > 0 && !keys && need_keys) return fail(HCTR_E_NULL_PTR, "keys is NULL");
  if (n_bags > 0 && !io && need_io) return fail(HCTR_E_NULL_PTR, "out / dY is NULL");
  if (io && (uintptr_t)io % 16 != 0) return fail(HCTR_E_INVALID_ARG, "out / dY must be 16-byte aligned");
  *L = emb_layout(d, nnz);
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < L->total)
    return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L->total);
  return HCTR_OK;
}

static void fill_slots(const hctr_emb_desc* d, SlotTable* st) {
  for (int s = 0; s < HCTR_MAX_SLOTS; ++s) {
    st->base[s] = (!d->hash && s < d->num_slots) ? d->slot_row_base[s] : 0;
    st->num[s] = (!d->hash && s < d->num_slots) ? d->slot_num_rows[s] : 0;
  }
}

template <typename T>
static int lanes_per_row(int dim) {
  int l = pow2_ceil((int)ceil_div((int64_t)dim * (int64_t)sizeof(T), 16));
  return l < 4 ? 4 : (l > 64 ? 64 : l);
}

template <typename T, typename OutT, int LPR>
static void launch_forward(const hctr_emb_desc* d, const int64_t* keys, const int64_t* rows64,
                           const int64_t* offsets, uint32_t n_bags, const SlotTable& st, OutT* out,
                           EmbHeader* hdr, hipStream_t stream) {
  constexpr int VEC = RowVec<T>::VEC;
  const uint32_t ychunks = (uint32_t)ceil_div(d->dim, LPR * VEC);
  const T* table = static_cast<const T*>(d->table);
  // slot by slot when every slot has a table of its own and an output row fills four cache lines
  const uint32_t S = (uint32_t)d->num_slots;
  // (bags of several keys read many rows per row they write, so there the walk pays from one cache line on)
  const size_t min_row_bytes = offsets ? kSlotMajorMinRowBytesCsr : kSlotMajorMinRowBytes;
  const uint32_t n_samples = (!rows64 && S > 1 && (size_t)d->dim * sizeof(OutT) >= min_row_bytes) ? n_bags / S : 0u;
  if (!offsets) {
    constexpr int U = kOneHotRows;
    const uint32_t bags_per_block = (kOneHotThreads / LPR) * U;
    dim3 grid((uint32_t)ceil_div(n_bags, bags_per_block), ychunks);
    if (rows64)
      hipLaunchKernelGGL((fwd_onehot<T, OutT, LPR, U, true>), grid, dim3(kOneHotThreads), 0, stream, table, d->dim,
                         d->total_rows, keys, rows64, n_bags, S, n_samples, st, out, hdr);
    else
      hipLaunchKernelGGL((fwd_onehot<T, OutT, LPR, U, false>), grid, dim3(kOneHotThreads), 0, stream, table, d->dim,
                         d->total_rows, keys, rows64, n_bags, S, n_samples, st, out, hdr);
  } else {
    constexpr int U = 4;
    // four bags (waves) per block; slot by slot: x counts the samples, z the slots
    const dim3 grid = n_samples ? dim3((uint32_t)ceil_div(n_samples, 4), ychunks, S)
                                : dim3((uint32_t)ceil_div(n_bags, 4), ychunks, 1);
    const int mean = d->combiner == HCTR_MEAN;
    if (rows64)
      hipLaunchKernelGGL((fwd_csr<T, OutT, LPR, U, true>), grid, dim3(256), 0, stream, table, d->dim,
                         d->total_rows, keys, rows64, offsets, n_bags, S, n_samples, st, mean,
                         out, hdr);
    else
      hipLaunchKernelGGL((fwd_csr<T, OutT, LPR, U, false>), grid, dim3(256), 0, stream, table, d->dim,
                         d->total_rows, keys, rows64, offsets, n_bags, S, n_samples, st, mean,
                         out, hdr);
  }
}

template <typename T, typename OutT>
static void dispatch_forward(int lpr, const hctr_emb_desc* d, const int64_t* keys,
                             const int64_t* rows64, const int64_t* offsets, uint32_t n_bags,
                             const SlotTable& st, OutT* out, EmbHeader* hdr, hipStream_t stream) {
  switch (lpr) {
    case 4: launch_forward<T, OutT, 4>(d, keys, rows64, offsets, n_bags, st, out, hdr, stream); break;
    case 8: launch_forward<T, OutT, 8>(d, keys, rows64, offsets, n_bags, st, out, hdr, stream); break;
    case 16: launch_forward<T, OutT, 16>(d, keys, rows64, offsets, n_bags, st, out, hdr, stream); break;
    case 32: launch_forward<T, OutT, 32>(d, keys, rows64, offsets, n_bags, st, out, hdr, stream); break;
    default: launch_forward<T, OutT, 64>(d, keys, rows64, offsets, n_bags, st, out, hdr, stream); break;
  }
}

// Bits of a sorted word's low half that hold the bag number (see BagWord): all 32 unless a mean is
// taken over bags given by offsets and the bag numbers leave at least four bits for the count.
static uint32_t bag_bits_for(bool mean_over_offsets, int64_t n_bags) {
  if (!mean_over_offsets) return 32u;
  const int bits = std::max(1, ceil_log2((uint64_t)n_bags));
  return bits <= 28 ? (uint32_t)bits : 32u;
}

// Launches the three reduction kernels for one view; dmax = widest row of the view.
template <typename T, int LPR, typename View>
static void launch_reduce(const View& view, int dmax, bool once, uint32_t bag_bits, const EmbLayout& L, char* ws,
                          const uint64_t* skv, const int64_t* offsets, float lr, hipStream_t stream) {
  const uint32_t ychunks = (uint32_t)ceil_div(dmax, LPR * 4);
  dim3 grid((uint32_t)ceil_div(L.n_windows, 256 / LPR), ychunks);
  EmbHeader* hdr = reinterpret_cast<EmbHeader*>(ws + L.header);
  float* head = reinterpret_cast<float*>(ws + L.head);
  float* tail = reinterpret_cast<float*>(ws + L.tail);
  uint8_t* tflag = reinterpret_cast<uint8_t*>(ws + L.tail_flag);
  uint32_t* long_list = reinterpret_cast<uint32_t*>(ws + L.long_list);
  const uint32_t* starts_before = reinterpret_cast<const uint32_t*>(ws + L.flags);
  const uint32_t* seg_off = reinterpret_cast<const uint32_t*>(ws + L.seg_off);
  if (once)
    hipLaunchKernelGGL((bwd_reduce_windows<T, LPR, View, true>), grid, dim3(256), 0, stream, view, skv,
                       hdr, offsets, lr, head, tail, tflag, L.window, bag_bits, long_list);
  else
    hipLaunchKernelGGL((bwd_reduce_windows<T, LPR, View, false>), grid, dim3(256), 0, stream, view, skv,
                       hdr, offsets, lr, head, tail, tflag, L.window, bag_bits, long_list);
  const uint32_t short_blocks = (uint32_t)ceil_div(L.n_windows, 1024 / LPR);
  const uint32_t long_blocks = L.n_windows < 256u ? L.n_windows : 256u;
  hipLaunchKernelGGL((bwd_carry<T, LPR, View>), dim3(long_blocks + short_blocks, ychunks), dim3(1024), 0, stream,
                     view, skv, starts_before, seg_off, hdr, lr, (const float*)head, (const float*)tail,
                     (const uint8_t*)tflag, L.window, (const uint32_t*)long_list, bag_bits, long_blocks);
}

template <typename T, typename View>
static void dispatch_reduce_view(const View& view, int dmax, bool once, uint32_t bag_bits, const EmbLayout& L,
                                 char* ws, const uint64_t* skv, const int64_t* offsets, float lr,
                                 hipStream_t stream) {
  int lpr = pow2_ceil((int)ceil_div(dmax, 4));
  lpr = lpr < 4 ? 4 : (lpr > 64 ? 64 : lpr);
  switch (lpr) {
    case 4: launch_reduce<T, 4>(view, dmax, once, bag_bits, L, ws, skv, offsets, lr, stream); break;
    case 8: launch_reduce<T, 8>(view, dmax, once, bag_bits, L, ws, skv, offsets, lr, stream); break;
    case 16: launch_reduce<T, 16>(view, dmax, once, bag_bits, L, ws, skv, offsets, lr, stream); break;
    case 32: launch_reduce<T, 32>(view, dmax, once, bag_bits, L, ws, skv, offsets, lr, stream); break;
    default: launch_reduce<T, 64>(view, dmax, once, bag_bits, L, ws, skv, offsets, lr, stream); break;
  }
}

template <typename T, typename DyT>
static void dispatch_reduce(const hctr_emb_desc* d, int64_t batch, const EmbLayout& L, char* ws,
                            const uint64_t* skv, const int64_t* offsets, const void* dY, float lr,
                            hipStream_t stream) {
  UniformView<T, DyT> view;
  view.table = static_cast<T*>(d->table);
  view.master = d->master;
  view.dY = static_cast<const DyT*>(dY);
  view.D = d->dim;
  view.mean = (d->combiner == HCTR_MEAN && offsets != nullptr) ? 1 : 0;
  const uint32_t bag_bits = bag_bits_for(view.mean != 0, batch * d->num_slots);
  dispatch_reduce_view<T>(view, d->dim, offsets == nullptr, bag_bits, L, ws, skv, offsets, lr, stream);
}

}  // namespace hctr

using namespace hctr;

HCTR_API size_t hctr_emb_workspace_bytes(const hctr_emb_desc* desc, int64_t batch, int64_t nnz_max) {
  (void)batch;
  if (!desc || desc->dim <= 0 || desc->total_rows < 1 || nnz_max < 0 || nnz_max >= (1ll << 31)) return 0;
  return emb_bytes_upto(desc->total_rows, desc->dim, nnz_max, desc->hash != nullptr, 0);
}

HCTR_API hctr_status hctr_emb_forward(const hctr_emb_desc* desc, int64_t batch, const int64_t* keys,
                                      const int64_t* offsets, int64_t nnz, void* out, void* ws,
                                      size_t ws_bytes, void* stream_) {
  EmbLayout L;
  HCTR_TRY(validate_batch(desc, batch, keys, offsets, nnz, out, ws, ws_bytes, &L));
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  char* w = static_cast<char*>(ws);
  EmbHeader* hdr = reinterpret_cast<EmbHeader*>(w + L.header);
  const int64_t n_bags = batch * desc->num_slots;
  if (n_bags == 0) return HCTR_OK;
  const int64_t* rows64 = nullptr;
  if (desc->hash) {
    int64_t* r = reinterpret_cast<int64_t*>(w + L.rows64);
    HCTR_TRY(hash_lookup(desc->hash, keys, nnz, desc->insert_on_miss, r, w + L.hash_ws,
                         L.total - L.hash_ws, stream));
    rows64 = r;
  }
  SlotTable st;
  fill_slots(desc, &st);
  const bool t32 = desc->table_dtype == HCTR_F32, o32 = desc->io_dtype == HCTR_F32;
  if (t32 && o32)
    dispatch_forward<float, float>(lanes_per_row<float>(desc->dim), desc, keys, rows64, offsets, (uint32_t)n_bags,
                                   st, static_cast<float*>(out), hdr, stream);
  else if (t32)
    dispatch_forward<float, __half>(lanes_per_row<float>(desc->dim), desc, keys, rows64, offsets, (uint32_t)n_bags,
                                    st, static_cast<__half*>(out), hdr, stream);
  else if (o32)
    dispatch_forward<__half, float>(lanes_per_row<__half>(desc->dim), desc, keys, rows64, offsets, (uint32_t)n_bags,
                                    st, static_cast<float*>(out), hdr, stream);
  else
    dispatch_forward<__half, __half>(lanes_per_row<__half>(desc->dim), desc, keys, rows64, offsets,
                                     (uint32_t)n_bags, st, static_cast<__half*>(out), hdr, stream);
  return launch_status("hctr_emb_forward");
}

// B1-B3 (reads keys / offsets only and writes the workspace) for keys whose bags cycle through n_slots slots with the row ranges in st (or whose rows
// are given in rows64): packed (row, bag) words, sorted by row, run boundaries.
static hctr_status dedup_core(const int64_t* keys, const int64_t* rows64, const int64_t* offsets, int64_t nnz,
                              uint32_t n_bags, uint32_t n_slots, const SlotTable& st, int64_t total_rows,
                              uint32_t bag_bits, const EmbLayout& L, char* w, hipStream_t stream) {
  EmbHeader* hdr = reinterpret_cast<EmbHeader*>(w + L.header);
  uint32_t* seg_off = reinterpret_cast<uint32_t*>(w + L.seg_off);
  uint32_t* aux = reinterpret_cast<uint32_t*>(w + L.aux);
  const uint32_t zero_count = (uint32_t)(L.sort.aux_count + L.seg_super);
  hipLaunchKernelGGL(emb_init_header, dim3((uint32_t)ceil_div(zero_count, 256)), dim3(256), 0, stream, hdr,
                     seg_off, 0, aux, zero_count);
  if (nnz == 0) return launch_status("emb_init_header");
  const uint32_t n = (uint32_t)nnz;
  uint64_t* kv0 = reinterpret_cast<uint64_t*>(w + L.kv0);
  uint64_t* kv1 = reinterpret_cast<uint64_t*>(w + L.kv1);
  uint32_t* hist = reinterpret_cast<uint32_t*>(w + L.hist);
  uint32_t* segsup = aux + L.sort.aux_count;
  uint32_t* seg_counts = reinterpret_cast<uint32_t*>(w + L.seg_counts);
  uint32_t* flags = reinterpret_cast<uint32_t*>(w + L.flags);
  uint32_t* uniq = reinterpret_cast<uint32_t*>(w + L.uniq);

  // About one tile per compute unit: 1024-thread blocks, so a wave's serial share is 4 rounds, not 16.
  const bool wide = L.sort.n_blocks <= kSortWideMaxTiles;
  const uint32_t bins0 = 1u << L.sort.digit_bits[0];
  uint32_t* sup0 = sort_scans_groups(L.sort) ? nullptr : sort_aux_sup(L.sort, aux, 0);
  const bool pack = offsets != nullptr && bag_bits < 32u;
#define HCTR_BWD_ROWS(NT, PACK)                                                                                 \
  hipLaunchKernelGGL((bwd_rows<NT, PACK>), dim3(L.sort.n_blocks), dim3(NT), 0, stream, keys, rows64, offsets, n, \
                     n_bags, n_slots, st, total_rows, kv0, hdr, bins0, hist, sup0, bag_bits)
  if (wide && pack) HCTR_BWD_ROWS(1024, true);
  else if (wide) HCTR_BWD_ROWS(1024, false);
  else if (pack) HCTR_BWD_ROWS(256, true);
  else HCTR_BWD_ROWS(256, false);
#undef HCTR_BWD_ROWS
  HCTR_TRY(radix_sort_u64(L.sort, nullptr, kv0, kv1, hist, aux, true, stream, true));
  const uint64_t* skv = (L.sort.passes & 1) ? kv1 : kv0;
  if (wide) {
    hipLaunchKernelGGL((seg_count<1024>), dim3(L.seg_tiles), dim3(1024), 0, stream, skv, n, seg_counts, segsup);
    hipLaunchKernelGGL((seg_write<1024>), dim3(L.seg_tiles), dim3(1024), 0, stream, skv, n,
                       (const uint32_t*)seg_counts, (const uint32_t*)segsup, flags, L.window, uniq, seg_off, hdr);
  } else {
    hipLaunchKernelGGL((seg_count<256>), dim3(L.seg_tiles), dim3(256), 0, stream, skv, n, seg_counts, segsup);
    hipLaunchKernelGGL((seg_write<256>), dim3(L.seg_tiles), dim3(256), 0, stream, skv, n,
                       (const uint32_t*)seg_counts, (const uint32_t*)segsup, flags, L.window, uniq, seg_off, hdr);
  }
  return launch_status("dedup");
}

static hctr_status backward_dedup(const hctr_emb_desc* desc, int64_t batch, const int64_t* keys,
                                  const int64_t* offsets, int64_t nnz, const EmbLayout& L, char* w,
                                  hipStream_t stream) {
  const int64_t* rows64 = nullptr;
  if (desc->hash && nnz > 0) {
    int64_t* r = reinterpret_cast<int64_t*>(w + L.rows64);
    if (!desc->reuse_forward_rows)   // else: the forward on this workspace left them there
      HCTR_TRY(hash_lookup(desc->hash, keys, nnz, 0, r, w + L.hash_ws, L.total - L.hash_ws, stream));
    rows64 = r;
  }
  SlotTable st;
  fill_slots(desc, &st);
  const int64_t n_bags = batch * desc->num_slots;
  const uint32_t bag_bits = bag_bits_for(desc->combiner == HCTR_MEAN && offsets != nullptr, n_bags);
  return dedup_core(keys, rows64, offsets, nnz, (uint32_t)n_bags, (uint32_t)desc->num_slots, st, desc->total_rows,
                    bag_bits, L, w, stream);
}

// B4-B5: segmented reduction of dY over the sorted occurrences, fused with the SGD row update.
static hctr_status backward_apply(const hctr_emb_desc* desc, int64_t batch, const int64_t* offsets, int64_t nnz,
                                  const void* dY, float lr, const EmbLayout& L, char* w,
                                  hipStream_t stream) {
  if (nnz == 0) return HCTR_OK;
  const uint64_t* skv = reinterpret_cast<const uint64_t*>(w + ((L.sort.passes & 1) ? L.kv1 : L.kv0));
  const bool t32 = desc->table_dtype == HCTR_F32, g32 = desc->io_dtype == HCTR_F32;
  if (t32 && g32) dispatch_reduce<float, float>(desc, batch, L, w, skv, offsets, dY, lr, stream);
  else if (t32) dispatch_reduce<float, __half>(desc, batch, L, w, skv, offsets, dY, lr, stream);
  else if (g32) dispatch_reduce<__half, float>(desc, batch, L, w, skv, offsets, dY, lr, stream);
  else dispatch_reduce<__half, __half>(desc, batch, L, w, skv, offsets, dY, lr, stream);
  return launch_status("hctr_emb_backward_apply");
}

HCTR_API hctr_status hctr_emb_backward_dedup(const hctr_emb_desc* desc, int64_t batch, const int64_t* keys,
                                             const int64_t* offsets, int64_t nnz, void* ws, size_t ws_bytes,
                                             void* stream) {
  EmbLayout L;
  HCTR_TRY(validate_batch(desc, batch, keys, offsets, nnz, nullptr, ws, ws_bytes, &L, false));
  return backward_dedup(desc, batch, keys, offsets, nnz, L, static_cast<char*>(ws), static_cast<hipStream_t>(stream));
}

HCTR_API hctr_status hctr_emb_backward_apply(const hctr_emb_desc* desc, int64_t batch, const int64_t* offsets,
                                             int64_t nnz, const void* dY, float lr, void* ws,
                                             size_t ws_bytes, void* stream) {
  EmbLayout L;
  HCTR_TRY(validate_batch(desc, batch, nullptr, offsets, nnz, dY, ws, ws_bytes, &L, true, false));
  return backward_apply(desc, batch, offsets, nnz, dY, lr, L, static_cast<char*>(ws), static_cast<hipStream_t>(stream));
}

HCTR_API hctr_status hctr_emb_backward_sgd(const hctr_emb_desc* desc, int64_t batch, const int64_t* keys,
                                           const int64_t* offsets, int64_t nnz, const void* dY, float lr,
                                           void* ws, size_t ws_bytes, void* stream_) {
  EmbLayout L;
  HCTR_TRY(validate_batch(desc, batch, keys, offsets, nnz, dY, ws, ws_bytes, &L));
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  HCTR_TRY(backward_dedup(desc, batch, keys, offsets, nnz, L, static_cast<char*>(ws), stream));
  return backward_apply(desc, batch, offsets, nnz, dY, lr, L, static_cast<char*>(ws), stream);
}

HCTR_API hctr_status hctr_emb_dedup_view(const hctr_emb_desc* desc, int64_t batch, int64_t nnz,
                                         void* ws, size_t ws_bytes, const int64_t** num_unique,
                                         const uint32_t** uniq_rows, const uint32_t** seg_offsets) {
  (void)batch;
  HCTR_TRY(validate_desc(desc));
  if (!ws || !num_unique || !uniq_rows || !seg_offsets) return fail(HCTR_E_NULL_PTR, "NULL argument");
  if (nnz < 0 || nnz >= (1ll << 31)) return fail(HCTR_E_INVALID_ARG, "nnz out of range");
  const EmbLayout L = emb_layout(desc, nnz);
  if (ws_bytes < L.total) return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L.total);
  char* w = static_cast<char*>(ws);
  *num_unique = reinterpret_cast<const int64_t*>(w + L.header + offsetof(EmbHeader, num_unique));
  *uniq_rows = reinterpret_cast<const uint32_t*>(w + L.uniq);
  *seg_offsets = reinterpret_cast<const uint32_t*>(w + L.seg_off);
  return HCTR_OK;
}

HCTR_API hctr_status hctr_emb_workspace_init(void* ws, size_t ws_bytes, void* stream) {
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < kEmbHeadBytes) return fail(HCTR_E_WORKSPACE, "workspace too small");
  hipLaunchKernelGGL(emb_init_header, dim3(kInvalidParts / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<EmbHeader*>(ws), (uint32_t*)nullptr, 1, (uint32_t*)nullptr, 0u);
  return launch_status("emb_init_header");
}

HCTR_API hctr_status hctr_emb_invalid_keys(const void* ws, size_t ws_bytes, void* stream, int64_t* count) {
  if (!ws || !count) return fail(HCTR_E_NULL_PTR, "NULL argument");
  if (ws_bytes < kEmbHeadBytes) return fail(HCTR_E_WORKSPACE, "workspace too small");
  // header and counters in one copy: the mark tells a workspace that never went through
  // hctr_emb_workspace_init (whose counters hold whatever the memory held) from a counted one
  static_assert(sizeof(EmbHeader) % 8 == 0, "counters follow the header as 8-byte words");
  constexpr uint32_t kHeadWords = sizeof(EmbHeader) / 8;
  unsigned long long words[kHeadWords + kInvalidParts];
  HCTR_TRY_HIP(hipMemcpyAsync(words, ws, sizeof(words), hipMemcpyDeviceToHost, static_cast<hipStream_t>(stream)));
  HCTR_TRY_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  if (words[0] != kEmbMark)
    return fail(HCTR_E_WORKSPACE, "workspace was never initialised (hctr_emb_workspace_init): its counters mean nothing");
  const unsigned long long* parts = words + kHeadWords;
  unsigned long long v = 0;
  for (uint32_t i = 0; i < kInvalidParts; ++i) v += parts[i];
  *count = (int64_t)v;
  return HCTR_OK;
}

// ------------------------------------------------------------------------------------------------
// Fused group: host side
// ------------------------------------------------------------------------------------------------
namespace hctr {

struct GroupPlan {
  uint32_t L, width_total, per_sample;
  int dmax;
  int64_t total_rows;
  uint32_t row_base[HCTR_MAX_GROUP_LOOKUPS];   // per table
  GroupLookup lk[HCTR_MAX_GROUP_LOOKUPS];      // per lookup
  uint32_t num_rows[HCTR_MAX_GROUP_LOOKUPS];   // per lookup
  uint32_t hot_of[HCTR_MAX_GROUP_LOOKUPS];     // per lookup: declared hotness (dense input)
  GroupHotness hot;
};

static hctr_status group_plan(const hctr_group_desc* d, GroupPlan* P) {
  if (!d) return fail(HCTR_E_NULL_PTR, "desc is NULL");
  if (d->num_tables < 1 || d->num_tables > HCTR_MAX_GROUP_LOOKUPS || d->num_lookups < 1 ||
      d->num_lookups > HCTR_MAX_GROUP_LOOKUPS)
    return fail(HCTR_E_INVALID_ARG, "num_tables %d / num_lookups %d outside 1..%d", d->num_tables,
                d->num_lookups, HCTR_MAX_GROUP_LOOKUPS);
  if (d->table_dtype != HCTR_F32 && d->table_dtype != HCTR_F16)
    return fail(HCTR_E_INVALID_ARG, "table_dtype %d unknown", d->table_dtype);
  if (!d->tables || !d->lookups) return fail(HCTR_E_NULL_PTR, "tables / lookups is NULL");
  const int mult = d->table_dtype == HCTR_F32 ? 4 : 8;
  int64_t rows = 0;
  for (int t = 0; t < d->num_tables; ++t) {
    const hctr_group_table& tb = d->tables[t];
    if (!tb.data) return fail(HCTR_E_NULL_PTR, "table %d: data is NULL", t);
    if ((uintptr_t)tb.data % 16 != 0) return fail(HCTR_E_INVALID_ARG, "table %d must be 16-byte aligned", t);
    if (tb.dim <= 0 || tb.dim % mult != 0)
      return fail(HCTR_E_INVALID_ARG, "table %d: dim %d must be a positive multiple of %d", t, tb.dim, mult);
    if (tb.num_rows < 1) return fail(HCTR_E_INVALID_ARG, "table %d: num_rows %lld < 1", t, (long long)tb.num_rows);
    P->row_base[t] = (uint32_t)rows;
    rows += tb.num_rows;
    if (rows > 0xFFFFFFFEll) return fail(HCTR_E_UNSUPPORTED, "the group's tables have more than 2^32-2 rows");
  }
  P->total_rows = rows;
  P->L = (uint32_t)d->num_lookups;
  P->dmax = 0;
  uint32_t col = 0, hot = 0;
  for (int l = 0; l < d->num_lookups; ++l) {
    const hctr_group_lookup& lu = d->lookups[l];
    if (lu.table < 0 || lu.table >= d->num_tables)
      return fail(HCTR_E_INVALID_ARG, "lookup %d: table %d outside 0..%d", l, lu.table, d->num_tables - 1);
    if (lu.combiner != HCTR_SUM && lu.combiner != HCTR_MEAN)
      return fail(HCTR_E_INVALID_ARG, "lookup %d: combiner %d unknown", l, lu.combiner);
    const hctr_group_table& tb = d->tables[lu.table];
    P->lk[l].table = tb.data;
    P->lk[l].row_base = P->row_base[lu.table];
    P->lk[l].col = col;
    P->lk[l].dim = (uint32_t)tb.dim;
    P->lk[l].mean = lu.combiner == HCTR_MEAN ? 1u : 0u;
    P->num_rows[l] = (uint32_t)tb.num_rows;
    P->hot.before[l] = hot;
    P->hot_of[l] = lu.hotness > 0 ? (uint32_t)lu.hotness : 0u;
    col += (uint32_t)tb.dim;
    hot += lu.hotness > 0 ? (uint32_t)lu.hotness : 0u;
    if (tb.dim > P->dmax) P->dmax = tb.dim;
  }
  P->width_total = col;
  P->per_sample = hot;
  P->hot.L = P->L;
  P->hot.per_sample = hot;
  return HCTR_OK;
}

static EmbLayout group_layout(const GroupPlan& P, int64_t batch, int64_t nnz_max) {
  return emb_layout_raw(P.total_rows, P.dmax, nnz_max, false, (size_t)(batch * P.L + 1) * 8);
}

// Argument checks shared by forward and backward; *csr gets the offsets to use (the caller's, or
// the ones written into the workspace for dense input).
static hctr_status group_prepare(const hctr_group_desc* d, int64_t batch, const int64_t* keys,
                                 const int64_t* offsets, int64_t nnz, const void* io, void* ws, size_t ws_bytes,
                                 GroupPlan* P, EmbLayout* L, const int64_t** csr, bool need_csr,
                                 hipStream_t stream) {
  HCTR_TRY(group_plan(d, P));
  if (batch < 0 || nnz < 0)
    return fail(HCTR_E_INVALID_ARG, "batch %lld / nnz %lld negative", (long long)batch, (long long)nnz);
  const int64_t n_bags = batch * P->L;
  if (n_bags >= (1ll << 31) || nnz >= (1ll << 31))
    return fail(HCTR_E_UNSUPPORTED, "more than 2^31-1 bags or keys in one call");
  if (!offsets) {
    for (int l = 0; l < d->num_lookups; ++l)
      if (d->lookups[l].hotness < 1)
        return fail(HCTR_E_INVALID_ARG, "dense input (offsets == NULL): lookup %d has hotness %d < 1", l,
                    d->lookups[l].hotness);
    if (nnz != batch * (int64_t)P->per_sample)
      return fail(HCTR_E_INVALID_ARG, "dense input needs nnz == batch * sum of hotness (%lld != %lld)",
                  (long long)nnz, (long long)(batch * (int64_t)P->per_sample));
  }
  if (batch == 0 && nnz != 0) return fail(HCTR_E_INVALID_ARG, "nnz must be 0 when batch is 0");
  if (nnz > 0 && !keys) return fail(HCTR_E_NULL_PTR, "keys is NULL");
  if (n_bags > 0 && !io) return fail(HCTR_E_NULL_PTR, "out / dY is NULL");
  if (io && (uintptr_t)io % 16 != 0) return fail(HCTR_E_INVALID_ARG, "out / dY must be 16-byte aligned");
  *L = group_layout(*P, batch, nnz);
  if (!ws) return fail(HCTR_E_WORKSPACE, "workspace is NULL");
  if ((uintptr_t)ws % 256 != 0) return fail(HCTR_E_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < L->total)
    return fail(HCTR_E_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L->total);
  *csr = offsets;
  // Dense input with one key per lookup is the one-hot case (bag i holds key i): no offsets needed.
  if (!offsets && n_bags > 0 && need_csr && P->per_sample != P->L) {
    int64_t* gen = reinterpret_cast<int64_t*>(static_cast<char*>(ws) + L->extra);
    hipLaunchKernelGGL(group_dense_offsets, dim3((uint32_t)ceil_div(n_bags + 1, 256)), dim3(256), 0, stream, P->hot,
                       (uint64_t)n_bags, gen);
    *csr = gen;
  }
  return HCTR_OK;
}

template <typename T>
static void group_launch_forward(const GroupPlan& P, bool dense, int64_t batch, const int64_t* keys,
                                 const int64_t* csr, float* out, EmbHeader* hdr, hipStream_t stream) {
  GroupFwdArgs a;
  a.L = P.L;
  a.width_total = P.width_total;
  a.per_sample = dense ? P.per_sample : 0;
  for (int l = 0; l < HCTR_MAX_GROUP_LOOKUPS; ++l) {
    const bool used = l < (int)P.L;
    a.lk[l] = used ? P.lk[l] : GroupLookup{nullptr, 0, 0, 0, 0};
    a.num_rows[l] = used ? P.num_rows[l] : 0;
    a.before[l] = used ? P.hot.before[l] : 0;
    a.hot[l] = used ? P.hot_of[l] : 0;
  }
  constexpr int NQ = 2;   // quads per thread: 1, 3, 4 and 6 measured 49, 16, 22 and 31 % slower on 26 tables of mixed widths
  const uint64_t n_quads = (uint64_t)batch * (P.width_total / 4);
  // A grid whose thread count is a multiple of the quads of a sample (W4) lets every thread keep its
  // columns: `unit` blocks are the smallest such grid, and about 4,000 blocks (16 per compute unit)
  // are launched in multiples of it.  A sample too wide for that falls back to one pass over all quads.
  const uint64_t W4 = P.width_total / 4;
  uint64_t g = W4, h = 256;
  while (h) { const uint64_t r = g % h; g = h; h = r; }   // g = gcd(W4, 256)
  const uint64_t unit = W4 / g;
  if (unit <= 4096 && n_quads >= unit * 256) {
    const uint64_t want = 4096;
    uint64_t blocks = unit * (want / unit > 0 ? want / unit : 1);
    const uint64_t enough = ceil_div((int64_t)ceil_div((int64_t)n_quads, 256 * NQ), (int64_t)unit) * unit;
    if (blocks > enough) blocks = enough;   // a small batch: one step per thread
    hipLaunchKernelGGL((fwd_group<T, NQ, true>), dim3((uint32_t)blocks), dim3(256), 0, stream, a, keys, csr, n_quads,
                       out, hdr);
    return;
  }
  uint64_t blocks = ceil_div((int64_t)n_quads, 256 * NQ);
  if (blocks > (1u << 20)) blocks = 1u << 20;   // grid-stride beyond a million blocks
  hipLaunchKernelGGL((fwd_group<T, NQ, false>), dim3((uint32_t)blocks), dim3(256), 0, stream, a, keys, csr, n_quads,
                     out, hdr);
}

template <typename T>
static void group_launch_reduce(const GroupPlan& P, uint32_t bag_bits, const EmbLayout& L, char* w,
                                const uint64_t* skv, const int64_t* csr, const float* dY, float lr,
                                hipStream_t stream) {
  GroupView<T> view;
  view.dY = dY;
  view.L = P.L;
  view.width_total = P.width_total;
  view.dmax_ = P.dmax;
  for (int l = 0; l < HCTR_MAX_GROUP_LOOKUPS; ++l) {
    view.lk[l] = l < (int)P.L ? P.lk[l] : GroupLookup{nullptr, 0, 0, 0, 0};
    if (csr == nullptr) view.lk[l].mean = 0;   // one key per bag: the mean is the sum, and no offsets exist to read
  }
  dispatch_reduce_view<T>(view, P.dmax, false, bag_bits, L, w, skv, csr, lr, stream);
}

}  // namespace hctr

HCTR_API size_t hctr_group_workspace_bytes(const hctr_group_desc* desc, int64_t batch, int64_t nnz_max) {
  GroupPlan P;
  if (batch < 0 || nnz_max < 0 || nnz_max >= (1ll << 31) || group_plan(desc, &P) != HCTR_OK) return 0;
  if (batch * P.L >= (1ll << 31)) return 0;
  return emb_bytes_upto(P.total_rows, P.dmax, nnz_max, false, (size_t)(batch * P.L + 1) * 8);
}

HCTR_API hctr_status hctr_group_forward(const hctr_group_desc* desc, int64_t batch, const int64_t* keys,
                                        const int64_t* offsets, int64_t nnz, float* out, void* ws,
                                        size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  GroupPlan P;
  EmbLayout L;
  const int64_t* csr = nullptr;
  HCTR_TRY(group_prepare(desc, batch, keys, offsets, nnz, out, ws, ws_bytes, &P, &L, &csr, false, stream));
  if (batch == 0) return HCTR_OK;
  EmbHeader* hdr = reinterpret_cast<EmbHeader*>(static_cast<char*>(ws) + L.header);
  const bool dense = offsets == nullptr;   // bag bounds follow from the declared hotness
  if (desc->table_dtype == HCTR_F32) group_launch_forward<float>(P, dense, batch, keys, csr, out, hdr, stream);
  else group_launch_forward<__half>(P, dense, batch, keys, csr, out, hdr, stream);
  return launch_status("hctr_group_forward");
}

HCTR_API hctr_status hctr_group_backward_sgd(const hctr_group_desc* desc, int64_t batch, const int64_t* keys,
                                             const int64_t* offsets, int64_t nnz, const float* dY, float lr,
                                             void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  GroupPlan P;
  EmbLayout L;
  const int64_t* csr = nullptr;
  HCTR_TRY(group_prepare(desc, batch, keys, offsets, nnz, dY, ws, ws_bytes, &P, &L, &csr, true, stream));
  char* w = static_cast<char*>(ws);
  SlotTable st;   // the key -> row kernel sees the lookups as slots whose ranges are their tables' rows
  for (int s = 0; s < HCTR_MAX_SLOTS; ++s) {
    st.base[s] = s < (int)P.L ? (int64_t)P.lk[s].row_base : 0;
    st.num[s] = s < (int)P.L ? (int64_t)P.num_rows[s] : 0;
  }
  bool any_mean = false;
  for (uint32_t l = 0; l < P.L; ++l) any_mean |= P.lk[l].mean != 0;
  const uint32_t bag_bits = bag_bits_for(any_mean && csr != nullptr, batch * P.L);
  HCTR_TRY(dedup_core(keys, nullptr, csr, nnz, (uint32_t)(batch * P.L), P.L, st, P.total_rows, bag_bits, L, w, stream));
  if (nnz == 0) return HCTR_OK;
  const uint64_t* skv = reinterpret_cast<const uint64_t*>(w + ((L.sort.passes & 1) ? L.kv1 : L.kv0));
  if (desc->table_dtype == HCTR_F32) group_launch_reduce<float>(P, bag_bits, L, w, skv, csr, dY, lr, stream);
  else group_launch_reduce<__half>(P, bag_bits, L, w, skv, csr, dY, lr, stream);
  return launch_status("hctr_group_backward_sgd");
}

HCTR_API hctr_status hctr_check_offsets(const int64_t* offsets, int64_t n_bags, int64_t nnz, void* ws,
                                        size_t ws_bytes, void* stream_) {
  if (!offsets) return fail(HCTR_E_NULL_PTR, "offsets is NULL");
  if (n_bags < 0 || nnz < 0) return fail(HCTR_E_INVALID_ARG, "n_bags %lld / nnz %lld negative", (long long)n_bags,
                                         (long long)nnz);
  if (!ws || ws_bytes < 8 || (uintptr_t)ws % 8 != 0) return fail(HCTR_E_WORKSPACE, "ws must hold 8 aligned bytes");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  unsigned long long* bad = static_cast<unsigned long long*>(ws);
  unsigned long long v = 0;
  HCTR_TRY_HIP(hipMemcpyAsync(bad, &v, sizeof(v), hipMemcpyHostToDevice, stream));
  const uint32_t blocks = (uint32_t)std::min<int64_t>(ceil_div(n_bags + 1, 256), 2048);
  hipLaunchKernelGGL(check_offsets, dim3(blocks), dim3(256), 0, stream, offsets, (uint64_t)n_bags, nnz, bad);
  HCTR_TRY(launch_status("check_offsets"));
  HCTR_TRY_HIP(hipMemcpyAsync(&v, bad, sizeof(v), hipMemcpyDeviceToHost, stream));
  HCTR_TRY_HIP(hipStreamSynchronize(stream));
  if (v != 0)
    return fail(HCTR_E_INVALID_ARG, "offsets break the CSR contract at %llu place(s) (first 0, last nnz, non-decreasing)", v);
  return HCTR_OK;
}
