// CPU oracle for the hashed sparse embedding path.  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, plain definition of what the embedding layer computes, used by the tests,
// by the smoke check and by the benchmark's CPU-baseline leg to judge the GPU library.  The
// product path never calls it and shares no code with it.  Everything is a single-threaded loop
// over std::unordered_map / std::vector, floating point accumulates in double and is rounded once
// (the *_mt functions run the same loops on several threads for the benchmark's CPU baseline and
// are checked bit-equal to the single-threaded ones).
//
// What each function follows in the paper (Merlin HugeCTR, RecSys'22 talk abstract):
//   * key -> row lookup in an "embedding hash", one table per slot, and the intra-slot reduction
//     of multi-hot features: section 1, "Localized slot embedding hash".
//   * forward and backward propagation through the embedding: section 1, "Hybrid sparse
//     embedding" (the paper names the passes; the SGD rule and the dedup of repeated keys are the
//     benchmark definition's, the paper gives no optimizer).
//   * FP16 parameter storage: section 1, "Mixed precision training".
//   * the level-1 embedding inference cache with dynamic insertion, and the level-2 store in
//     system memory that serves its misses: section 3, "embedding inference cache" and
//     "Volatile database".
//
// Pins (tests/test_oracle_*.py): dense matrix-product brute force, torch's embedding_bag and
// autograd, numpy.unique, hand-worked traces, textbook LRU / direct-mapped special cases and the
// conservation invariants.  No function here is "parity unpinned".

#include <cstdint>
#include <cstring>
#include <cmath>
#include <thread>
#include <unordered_map>
#include <utility>
#include <vector>
#include <algorithm>

namespace {

enum { DT_F32 = 0, DT_F16 = 1 };
enum { COMB_SUM = 0, COMB_MEAN = 1 };

// IEEE binary16 bit pattern -> double, decoded field by field.
double half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int exp = (h >> 10) & 0x1F;
  int man = h & 0x3FF;
  double v;
  if (exp == 0) v = std::ldexp((double)man, -24);                 // subnormal: man * 2^-24
  else if (exp == 31) v = man ? NAN : INFINITY;
  else v = std::ldexp((double)(man | 0x400), exp - 25);           // (1024+man) * 2^(exp-15-10)
  return sign ? -v : v;
}

// double -> IEEE binary16 bit pattern, round to nearest, ties to even, overflow to infinity.
uint16_t double_to_half(double x) {
  uint16_t sign = std::signbit(x) ? 0x8000 : 0;
  double a = std::fabs(x);
  if (std::isnan(a)) return sign | 0x7E00;
  if (a >= 65520.0) return sign | 0x7C00;                          // rounds to 2^16 => infinity
  if (a == 0.0) return sign;
  int e;
  std::frexp(a, &e);                                               // a = f * 2^e, f in [0.5, 1)
  int exp = e - 1;                                                 // a in [2^exp, 2^(exp+1))
  if (exp < -14) exp = -14;                                        // subnormal range shares 2^-24 spacing
  double q = std::ldexp(a, 10 - exp);                              // in units of the spacing
  double r = std::nearbyint(q);                                    // default mode: ties to even
  // q is in [1024, 2048) for normals, [0, 1024) for subnormals; r may reach 2048 (carry).
  if (exp == -14 && r < 1024.0) return sign | (uint16_t)r;        // subnormal (or zero)
  if (r >= 2048.0) { r = 1024.0; exp += 1; }
  if (exp > 15) return sign | 0x7C00;
  return sign | (uint16_t)(((exp + 15) << 10) | ((int)r - 1024));
}

inline double load_elem(const void* table, int dtype, int64_t idx) {
  if (dtype == DT_F32) return (double)((const float*)table)[idx];
  return half_to_double(((const uint16_t*)table)[idx]);
}

inline void store_elem(void* table, int dtype, int64_t idx, double v) {
  if (dtype == DT_F32) ((float*)table)[idx] = (float)v;            // one rounding, nearest-even
  else ((uint16_t*)table)[idx] = double_to_half(v);
}

inline int64_t bag_begin(const int64_t* offsets, int64_t bag) { return offsets ? offsets[bag] : bag; }
inline int64_t bag_end(const int64_t* offsets, int64_t bag) { return offsets ? offsets[bag + 1] : bag + 1; }

// The backward + SGD loop over the rows r with r mod n_parts == part (all rows for n_parts = 1):
// walks the occurrences in batch order, sums each owned row's gradient in double, applies the update
// and lists the owned rows in ascending order with their occurrence counts.
void backward_rows_of_part(int64_t part, int64_t n_parts, int32_t dim, int32_t dtype, int32_t combiner,
                           void* table, int64_t total_rows, const int64_t* rows, const int64_t* offsets,
                           int64_t n_bags, const float* dY, float lr,
                           std::vector<std::pair<int64_t, int64_t>>* found) {
  std::unordered_map<int64_t, std::vector<double>> grad;
  std::unordered_map<int64_t, int64_t> occ;
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    int64_t b0 = bag_begin(offsets, bag), b1 = bag_end(offsets, bag);
    double w = (combiner == COMB_MEAN && b1 > b0) ? 1.0 / (double)(b1 - b0) : 1.0;
    for (int64_t i = b0; i < b1; ++i) {
      int64_t r = rows[i];
      if (r < 0 || r >= total_rows) continue;
      if (r % n_parts != part) continue;
      std::vector<double>& g = grad[r];
      if (g.empty()) g.assign(dim, 0.0);
      for (int d = 0; d < dim; ++d) g[d] += w * (double)dY[bag * dim + d];
      occ[r] += 1;
    }
  }
  std::vector<int64_t> order;
  order.reserve(grad.size());
  for (auto& kv : grad) order.push_back(kv.first);
  std::sort(order.begin(), order.end());
  for (int64_t r : order) {
    const std::vector<double>& g = grad[r];
    for (int d = 0; d < dim; ++d) {
      double t = load_elem(table, dtype, r * dim + d);
      store_elem(table, dtype, r * dim + d, t - (double)lr * g[d]);
    }
    found->push_back({r, occ[r]});
  }
}

}  // namespace

extern "C" {

// Direct-index key -> global row of the fused table: the keys of bag (b, s) address the table of
// slot s, which occupies rows [slot_base[s], slot_base[s] + slot_rows[s]) (slots may share a
// table).  A key outside [0, slot_rows[s]) has no row (-1).  Returns the number of such keys.
// offsets == NULL means one key per bag.
int64_t oracle_rows_direct(int32_t num_slots, const int64_t* slot_base, const int64_t* slot_rows,
                           int64_t n_bags, const int64_t* keys, const int64_t* offsets,
                           int64_t* rows) {
  int64_t bad = 0;
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    int64_t s = bag % num_slots;
    for (int64_t i = bag_begin(offsets, bag); i < bag_end(offsets, bag); ++i) {
      if (keys[i] >= 0 && keys[i] < slot_rows[s]) rows[i] = slot_base[s] + keys[i];
      else { rows[i] = -1; ++bad; }
    }
  }
  return bad;
}

// Forward: out[bag, :] = w * sum_j T[row_j, :], w = 1 (sum) or 1/hotness (mean), hotness counting
// every key of the bag (also repeated keys and keys without a row); an empty bag gives zeros.
// Keys without a row (row < 0 or >= total_rows) add nothing.
void oracle_emb_forward(int32_t dim, int32_t dtype, int32_t combiner, const void* table,
                        int64_t total_rows, const int64_t* rows, const int64_t* offsets,
                        int64_t n_bags, float* out) {
  std::vector<double> acc(dim);
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    std::fill(acc.begin(), acc.end(), 0.0);
    int64_t b0 = bag_begin(offsets, bag), b1 = bag_end(offsets, bag);
    for (int64_t i = b0; i < b1; ++i) {
      int64_t r = rows[i];
      if (r < 0 || r >= total_rows) continue;
      for (int d = 0; d < dim; ++d) acc[d] += load_elem(table, dtype, r * dim + d);
    }
    double w = (combiner == COMB_MEAN && b1 > b0) ? 1.0 / (double)(b1 - b0) : 1.0;
    for (int d = 0; d < dim; ++d) out[bag * dim + d] = (float)(acc[d] * w);
  }
}

// Backward + SGD: for every distinct row r touched by the batch,
//   g_r = sum over occurrences (bag, j) with row_j = r of w_bag * dY[bag, :],
//   T[r, :] <- T[r, :] - lr * g_r   (evaluated in double, rounded once to the storage type).
// A key repeated inside a bag counts once per occurrence.  Rows never touched keep their bits.
// Also returns the dedup result: the distinct rows in ascending order with their occurrence
// counts (uniq_rows / counts hold up to nnz entries), and their number.
int64_t oracle_emb_backward_sgd(int32_t dim, int32_t dtype, int32_t combiner, void* table,
                                int64_t total_rows, const int64_t* rows, const int64_t* offsets,
                                int64_t n_bags, const float* dY, float lr,
                                int64_t* uniq_rows, int64_t* counts) {
  std::vector<std::pair<int64_t, int64_t>> found;
  backward_rows_of_part(0, 1, dim, dtype, combiner, table, total_rows, rows, offsets, n_bags, dY, lr, &found);
  int64_t u = 0;
  for (auto& rc : found) {
    if (uniq_rows) uniq_rows[u] = rc.first;
    if (counts) counts[u] = rc.second;
    ++u;
  }
  return u;
}

// ---------------------------------------------------------------------------------------------
// All-cores variants of the three functions above, for the benchmark's CPU baseline: the same loops
// on `threads` std::thread workers.  Forward and key -> row: bags are independent, a worker takes a
// contiguous run of whole samples and calls the single-threaded function on it.  Backward: rows are
// independent, worker t owns the rows with r mod threads == t, walks all occurrences in batch order
// and handles only its own, so every row sees the additions of the single-threaded loop in the same
// order: results are bit-identical (tests/test_oracle_mt.py).
// ---------------------------------------------------------------------------------------------
int32_t oracle_hardware_threads(void) {
  unsigned n = std::thread::hardware_concurrency();
  return n ? (int32_t)n : 1;
}

// [first, last) samples of worker t when `batch` samples are split over `threads` workers
static void samples_of(int64_t batch, int threads, int t, int64_t* first, int64_t* last) {
  int64_t per = (batch + threads - 1) / threads;
  *first = std::min(batch, per * t);
  *last = std::min(batch, per * (t + 1));
}

int64_t oracle_rows_direct_mt(int32_t threads, int32_t num_slots, const int64_t* slot_base,
                              const int64_t* slot_rows, int64_t n_bags, const int64_t* keys,
                              const int64_t* offsets, int64_t* rows) {
  if (threads < 1) threads = 1;
  const int64_t batch = n_bags / num_slots;   // whole samples, so that a worker's bags start at slot 0
  std::vector<int64_t> bad(threads, 0);
  std::vector<std::thread> pool;
  for (int t = 0; t < threads; ++t) {
    pool.emplace_back([&, t]() {
      int64_t s0, s1;
      samples_of(batch, threads, t, &s0, &s1);
      const int64_t g0 = s0 * num_slots, g1 = s1 * num_slots;
      if (offsets) bad[t] = oracle_rows_direct(num_slots, slot_base, slot_rows, g1 - g0, keys, offsets + g0, rows);
      else bad[t] = oracle_rows_direct(num_slots, slot_base, slot_rows, g1 - g0, keys + g0, nullptr, rows + g0);
    });
  }
  for (auto& th : pool) th.join();
  int64_t total = 0;
  for (int64_t b : bad) total += b;
  return total;
}

void oracle_emb_forward_mt(int32_t threads, int32_t dim, int32_t dtype, int32_t combiner, const void* table,
                           int64_t total_rows, const int64_t* rows, const int64_t* offsets,
                           int64_t n_bags, float* out) {
  if (threads < 1) threads = 1;
  std::vector<std::thread> pool;
  for (int t = 0; t < threads; ++t) {
    pool.emplace_back([&, t]() {
      int64_t g0, g1;
      samples_of(n_bags, threads, t, &g0, &g1);
      if (offsets) oracle_emb_forward(dim, dtype, combiner, table, total_rows, rows, offsets + g0, g1 - g0, out + g0 * dim);
      else oracle_emb_forward(dim, dtype, combiner, table, total_rows, rows + g0, nullptr, g1 - g0, out + g0 * dim);
    });
  }
  for (auto& th : pool) th.join();
}

int64_t oracle_emb_backward_sgd_mt(int32_t threads, int32_t dim, int32_t dtype, int32_t combiner, void* table,
                                   int64_t total_rows, const int64_t* rows, const int64_t* offsets,
                                   int64_t n_bags, const float* dY, float lr,
                                   int64_t* uniq_rows, int64_t* counts) {
  if (threads < 1) threads = 1;
  std::vector<std::vector<std::pair<int64_t, int64_t>>> found(threads);
  std::vector<std::thread> pool;
  for (int t = 0; t < threads; ++t) {
    pool.emplace_back([&, t]() {
      backward_rows_of_part(t, threads, dim, dtype, combiner, table, total_rows, rows, offsets, n_bags, dY, lr,
                            &found[t]);
    });
  }
  for (auto& th : pool) th.join();
  std::vector<std::pair<int64_t, int64_t>> all;
  for (auto& f : found) all.insert(all.end(), f.begin(), f.end());
  std::sort(all.begin(), all.end());
  int64_t u = 0;
  for (auto& rc : all) {
    if (uniq_rows) uniq_rows[u] = rc.first;
    if (counts) counts[u] = rc.second;
    ++u;
  }
  return u;
}

// ---------------------------------------------------------------------------------------------
// Mixed precision (section 1, "Mixed precision training": parameters kept in FP16, the layers
// downstream computing in reduced precision).  Same definitions as above with
//   * io_dtype = FP16: the pooled output is rounded once, from the double sum, to binary16; the
//     upstream gradient arrives as binary16 and is widened exactly;
//   * master != NULL (FP16 table only): master is an fp32 copy [total_rows, dim] of the
//     parameters.  The update is applied to the master row, m <- m - lr * g rounded once to fp32,
//     and the table row becomes that fp32 value rounded to binary16, so the FP16 table never
//     accumulates its own rounding errors.
// ---------------------------------------------------------------------------------------------
void oracle_emb_forward_mixed(int32_t dim, int32_t dtype, int32_t combiner, const void* table,
                              int64_t total_rows, const int64_t* rows, const int64_t* offsets,
                              int64_t n_bags, int32_t io_dtype, void* out) {
  std::vector<double> acc(dim);
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    std::fill(acc.begin(), acc.end(), 0.0);
    int64_t b0 = bag_begin(offsets, bag), b1 = bag_end(offsets, bag);
    for (int64_t i = b0; i < b1; ++i) {
      int64_t r = rows[i];
      if (r < 0 || r >= total_rows) continue;
      for (int d = 0; d < dim; ++d) acc[d] += load_elem(table, dtype, r * dim + d);
    }
    double w = (combiner == COMB_MEAN && b1 > b0) ? 1.0 / (double)(b1 - b0) : 1.0;
    for (int d = 0; d < dim; ++d) store_elem(out, io_dtype, bag * dim + d, acc[d] * w);
  }
}

int64_t oracle_emb_backward_sgd_mixed(int32_t dim, int32_t dtype, int32_t combiner, void* table,
                                      float* master, int64_t total_rows, const int64_t* rows,
                                      const int64_t* offsets, int64_t n_bags, int32_t io_dtype,
                                      const void* dY, float lr) {
  std::unordered_map<int64_t, std::vector<double>> grad;
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    int64_t b0 = bag_begin(offsets, bag), b1 = bag_end(offsets, bag);
    double w = (combiner == COMB_MEAN && b1 > b0) ? 1.0 / (double)(b1 - b0) : 1.0;
    for (int64_t i = b0; i < b1; ++i) {
      int64_t r = rows[i];
      if (r < 0 || r >= total_rows) continue;
      std::vector<double>& g = grad[r];
      if (g.empty()) g.assign(dim, 0.0);
      for (int d = 0; d < dim; ++d) g[d] += w * load_elem(dY, io_dtype, bag * dim + d);
    }
  }
  for (auto& kv : grad) {
    const int64_t r = kv.first;
    for (int d = 0; d < dim; ++d) {
      if (master) {
        master[r * dim + d] = (float)((double)master[r * dim + d] - (double)lr * kv.second[d]);
        store_elem(table, dtype, r * dim + d, (double)master[r * dim + d]);
      } else {
        double t = load_elem(table, dtype, r * dim + d);
        store_elem(table, dtype, r * dim + d, t - (double)lr * kv.second[d]);
      }
    }
  }
  return (int64_t)grad.size();
}

// ---------------------------------------------------------------------------------------------
// Fused group of lookups (section 4, "Future Work": one embedding fusing tables of different
// vector size and combiner, fed by dense or sparse inputs).  T tables, each [table_rows[t],
// table_dim[t]]; L lookups, lookup l reads table lookup_table[l] with combiner lookup_comb[l];
// bag = sample * L + l; the keys of a bag are direct row indices into the lookup's table (a key
// outside the table adds nothing but counts in a mean's denominator).  The output row of a sample
// is the concatenation of its L pooled vectors, lookup l at column col_l = sum of the widths of
// the lookups before it.  Dense input is the CSR special case with constant bag lengths; the
// caller passes offsets either way.
// ---------------------------------------------------------------------------------------------
void oracle_group_forward(int32_t num_tables, const void* const* tables, const int64_t* table_rows,
                          const int32_t* table_dim, int32_t dtype, int32_t num_lookups,
                          const int32_t* lookup_table, const int32_t* lookup_comb, int64_t batch,
                          const int64_t* keys, const int64_t* offsets, float* out) {
  (void)num_tables;
  int64_t width = 0;
  for (int l = 0; l < num_lookups; ++l) width += table_dim[lookup_table[l]];
  for (int64_t b = 0; b < batch; ++b) {
    int64_t col = 0;
    for (int l = 0; l < num_lookups; ++l) {
      const int t = lookup_table[l];
      const int dim = table_dim[t];
      const int64_t bag = b * num_lookups + l;
      const int64_t b0 = offsets[bag], b1 = offsets[bag + 1];
      std::vector<double> acc(dim, 0.0);
      for (int64_t i = b0; i < b1; ++i) {
        const int64_t k = keys[i];
        if (k < 0 || k >= table_rows[t]) continue;
        for (int d = 0; d < dim; ++d) acc[d] += load_elem(tables[t], dtype, k * dim + d);
      }
      const double w = (lookup_comb[l] == COMB_MEAN && b1 > b0) ? 1.0 / (double)(b1 - b0) : 1.0;
      for (int d = 0; d < dim; ++d) out[b * width + col + d] = (float)(acc[d] * w);
      col += dim;
    }
  }
}

// Backward + SGD over the group: every distinct (table, row) touched through any lookup gets
//   T_t[r, :] <- T_t[r, :] - lr * sum over its occurrences of w_bag * dY[b, col_l : col_l + dim].
// Returns the number of distinct (table, row) pairs.
int64_t oracle_group_backward_sgd(int32_t num_tables, void* const* tables, const int64_t* table_rows,
                                  const int32_t* table_dim, int32_t dtype, int32_t num_lookups,
                                  const int32_t* lookup_table, const int32_t* lookup_comb, int64_t batch,
                                  const int64_t* keys, const int64_t* offsets, const float* dY, float lr) {
  int64_t width = 0;
  for (int l = 0; l < num_lookups; ++l) width += table_dim[lookup_table[l]];
  std::vector<std::unordered_map<int64_t, std::vector<double>>> grad(num_tables);
  for (int64_t b = 0; b < batch; ++b) {
    int64_t col = 0;
    for (int l = 0; l < num_lookups; ++l) {
      const int t = lookup_table[l];
      const int dim = table_dim[t];
      const int64_t bag = b * num_lookups + l;
      const int64_t b0 = offsets[bag], b1 = offsets[bag + 1];
      const double w = (lookup_comb[l] == COMB_MEAN && b1 > b0) ? 1.0 / (double)(b1 - b0) : 1.0;
      for (int64_t i = b0; i < b1; ++i) {
        const int64_t k = keys[i];
        if (k < 0 || k >= table_rows[t]) continue;
        std::vector<double>& g = grad[t][k];
        if (g.empty()) g.assign(dim, 0.0);
        for (int d = 0; d < dim; ++d) g[d] += w * (double)dY[b * width + col + d];
      }
      col += dim;
    }
  }
  int64_t touched = 0;
  for (int t = 0; t < num_tables; ++t) {
    const int dim = table_dim[t];
    for (auto& kv : grad[t]) {
      for (int d = 0; d < dim; ++d) {
        const double x = load_elem(tables[t], dtype, kv.first * dim + d);
        store_elem(tables[t], dtype, kv.first * dim + d, x - (double)lr * kv.second[d]);
      }
      ++touched;
    }
  }
  return touched;
}

// ---------------------------------------------------------------------------------------------
// Hash: key -> dense row id, rows handed out in order of first appearance.
// ---------------------------------------------------------------------------------------------
struct oracle_hash {
  std::unordered_map<uint64_t, int64_t> map;
  int64_t max_rows;
};

oracle_hash* oracle_hash_create(int64_t max_rows) {
  oracle_hash* h = new oracle_hash();
  h->max_rows = max_rows;
  return h;
}
void oracle_hash_destroy(oracle_hash* h) { delete h; }
int64_t oracle_hash_size(const oracle_hash* h) { return (int64_t)h->map.size(); }

// Scan keys in array order.  Present -> its row.  Absent: if inserting and the table still has
// room, the key gets row = current size; otherwise -1.  Negative keys are never stored (-1).
void oracle_hash_insert_or_find(oracle_hash* h, const int64_t* keys, int64_t n, int32_t insert,
                                int64_t* rows) {
  for (int64_t i = 0; i < n; ++i) {
    if (keys[i] < 0) { rows[i] = -1; continue; }
    auto it = h->map.find((uint64_t)keys[i]);
    if (it != h->map.end()) { rows[i] = it->second; continue; }
    if (insert && (int64_t)h->map.size() < h->max_rows) {
      int64_t r = (int64_t)h->map.size();
      h->map.emplace((uint64_t)keys[i], r);
      rows[i] = r;
    } else {
      rows[i] = -1;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Set-associative embedding cache over a host-resident table, LRU at the granularity of a call.
// ---------------------------------------------------------------------------------------------
struct oracle_cache {
  int64_t num_sets;
  int32_t ways, dim;
  const float* host_table;
  int64_t host_rows;
  std::vector<uint64_t> tag;      // [num_sets * ways], EMPTY = all ones
  std::vector<uint32_t> stamp;    // [num_sets * ways], epoch of last hit / insert
  std::vector<float> data;        // [num_sets * ways * dim], copies of host rows
  uint32_t epoch;
  uint32_t epoch_limit;           // see oracle_cache_set_epoch_limit
  int64_t stats[6];               // queries, hits, misses, inserts, evictions, skipped inserts
};

static const uint64_t kEmptyTag = ~0ull;

// Set index of a key: x = key * 0x9E3779B97F4A7C15 (mod 2^64); x ^= x >> 32; set = x mod num_sets.
static int64_t cache_set_of(uint64_t key, int64_t num_sets) {
  uint64_t x = key * 0x9E3779B97F4A7C15ull;
  x ^= x >> 32;
  return (int64_t)(x % (uint64_t)num_sets);
}

oracle_cache* oracle_cache_create(int64_t num_sets, int32_t ways, int32_t dim,
                                  const float* host_table, int64_t host_rows) {
  oracle_cache* c = new oracle_cache();
  c->num_sets = num_sets; c->ways = ways; c->dim = dim;
  c->host_table = host_table; c->host_rows = host_rows;
  c->tag.assign((size_t)num_sets * ways, kEmptyTag);
  c->stamp.assign((size_t)num_sets * ways, 0u);
  c->data.assign((size_t)num_sets * ways * dim, 0.0f);
  c->epoch = 0;
  c->epoch_limit = 0xFFFFFF00u;
  std::memset(c->stats, 0, sizeof(c->stats));
  return c;
}
// Stamps are 32-bit call counts, so the count must not run out.  A call that finds the count at or
// above the limit first lowers every stamp and the count by half the limit; stamps at or below
// that half become 0, i.e. "never used" (among those the lowest way goes first, as after a clear).
// The order of all stamps above the half, and so the victim among ways used in the last limit/2
// calls, is unchanged.  (The paper gives no replacement policy; this keeps the least-recently-used
// choice meaningful for a server that never restarts.)  limit: 2 .. 2^32 - 256.
void oracle_cache_set_epoch_limit(oracle_cache* c, uint32_t limit) { c->epoch_limit = limit; }
uint32_t oracle_cache_epoch(const oracle_cache* c) { return c->epoch; }
void oracle_cache_destroy(oracle_cache* c) { delete c; }
void oracle_cache_stats(const oracle_cache* c, int64_t* out) { std::memcpy(out, c->stats, sizeof(c->stats)); }
void oracle_cache_state(const oracle_cache* c, uint64_t* tags, uint32_t* stamps, float* data) {
  if (tags) std::memcpy(tags, c->tag.data(), c->tag.size() * sizeof(uint64_t));
  if (stamps) std::memcpy(stamps, c->stamp.data(), c->stamp.size() * sizeof(uint32_t));
  if (data) std::memcpy(data, c->data.data(), c->data.size() * sizeof(float));
}

// Step 4 of a query: the distinct missing keys (where[i] < 0, key inside the host table), in
// first-appearance order, each into the lowest-index empty way of its set, else over the way with
// the smallest stamp among those not touched in this call (ties: lowest way), else skipped.
static void cache_insert_missing(oracle_cache* c, const int64_t* keys, int64_t nnz,
                                 const std::vector<int64_t>& where) {
  const int W = c->ways, D = c->dim;
  std::unordered_map<uint64_t, char> placed;      // missing keys already handled in this call
  for (int64_t i = 0; i < nnz; ++i) {
    if (where[i] >= 0 || keys[i] < 0 || keys[i] >= c->host_rows) continue;
    uint64_t k = (uint64_t)keys[i];
    if (!placed.emplace(k, 1).second) continue;
    int64_t set = cache_set_of(k, c->num_sets);
    int victim = -1;
    for (int w = 0; w < W && victim < 0; ++w)
      if (c->tag[set * W + w] == kEmptyTag) victim = w;
    bool evict = false;
    if (victim < 0) {
      uint32_t best = 0;
      for (int w = 0; w < W; ++w) {
        uint32_t st = c->stamp[set * W + w];
        if (st < c->epoch && (victim < 0 || st < best)) { victim = w; best = st; }
      }
      evict = victim >= 0;
    }
    if (victim < 0) { c->stats[5] += 1; continue; }
    int64_t line = set * W + victim;
    c->tag[line] = k;
    c->stamp[line] = c->epoch;
    std::memcpy(&c->data[line * D], &c->host_table[(int64_t)k * D], sizeof(float) * D);
    c->stats[3] += 1;
    if (evict) c->stats[4] += 1;
  }
}

// One query call.  Every key is classified against the cache as it was when the call began (all
// occurrences of a key get the same answer).  A hit reads the cached copy and refreshes its stamp;
// a miss reads the host table (key = host row; out-of-range keys read as a zero row and are never
// cached).  out[bag, :] is the plain sum of the bag's vectors.  With insert_missing, the distinct
// missing keys are then placed in first-appearance order: lowest-index empty way, else the way
// with the smallest stamp among those not touched in this call (ties: lowest way), else skipped.
void oracle_cache_query(oracle_cache* c, int64_t n_bags, const int64_t* keys,
                        const int64_t* offsets, int64_t hotness, int64_t nnz,
                        int32_t insert_missing, float* out, uint8_t* hit_mask) {
  if (c->epoch >= c->epoch_limit) {
    const uint32_t by = c->epoch_limit / 2;
    for (uint32_t& st : c->stamp) st = st > by ? st - by : 0u;
    c->epoch -= by;
  }
  c->epoch += 1;
  const int W = c->ways, D = c->dim;
  std::vector<int64_t> where(nnz, -1);            // cache line (set*ways+way) for hits
  for (int64_t i = 0; i < nnz; ++i) {             // classify against the entry state: tags only
    if (keys[i] < 0) continue;
    int64_t set = cache_set_of((uint64_t)keys[i], c->num_sets);
    for (int w = 0; w < W; ++w)
      if (c->tag[set * W + w] == (uint64_t)keys[i]) { where[i] = set * W + w; break; }
  }
  std::vector<double> acc(D);
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    std::fill(acc.begin(), acc.end(), 0.0);
    int64_t b0 = offsets ? offsets[bag] : bag * hotness;
    int64_t b1 = offsets ? offsets[bag + 1] : (bag + 1) * hotness;
    for (int64_t i = b0; i < b1; ++i) {
      c->stats[0] += 1;
      if (where[i] >= 0) {
        c->stats[1] += 1;
        c->stamp[where[i]] = c->epoch;
        if (hit_mask) hit_mask[i] = 1;
        for (int d = 0; d < D; ++d) acc[d] += (double)c->data[where[i] * D + d];
      } else {
        c->stats[2] += 1;
        if (hit_mask) hit_mask[i] = 0;
        if (keys[i] >= 0 && keys[i] < c->host_rows)
          for (int d = 0; d < D; ++d) acc[d] += (double)c->host_table[keys[i] * D + d];
      }
    }
    for (int d = 0; d < D; ++d) out[bag * D + d] = (float)acc[d];
  }
  if (insert_missing) cache_insert_missing(c, keys, nnz, where);
}

// Query in two phases, for a consumer that starts on the hits while the missing rows are still on
// their way across the host link (section 3: parameter migration overlapped with the dense network;
// "embedding inference cache": dynamic insertion, asynchronous mechanisms).
//
// Phase 1, "hits": one call (epoch) that classifies every key against the cache as it stands, stamps
// and counts the hits exactly as oracle_cache_query does, and pools ONLY the hits: a missing key adds
// nothing yet.  miss_pos receives the positions whose key is missing and lies inside the host table,
// in ascending order; the return value is their number.
int64_t oracle_cache_query_hits(oracle_cache* c, int64_t n_bags, const int64_t* keys,
                                const int64_t* offsets, int64_t hotness, int64_t nnz, float* out,
                                uint8_t* hit_mask, int64_t* miss_pos) {
  (void)nnz;
  if (c->epoch >= c->epoch_limit) {
    const uint32_t by = c->epoch_limit / 2;
    for (uint32_t& st : c->stamp) st = st > by ? st - by : 0u;
    c->epoch -= by;
  }
  c->epoch += 1;
  const int W = c->ways, D = c->dim;
  int64_t n_missing = 0;
  std::vector<double> acc(D);
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    std::fill(acc.begin(), acc.end(), 0.0);
    int64_t b0 = offsets ? offsets[bag] : bag * hotness;
    int64_t b1 = offsets ? offsets[bag + 1] : (bag + 1) * hotness;
    for (int64_t i = b0; i < b1; ++i) {
      int64_t line = -1;
      if (keys[i] >= 0) {
        int64_t set = cache_set_of((uint64_t)keys[i], c->num_sets);
        for (int w = 0; w < W && line < 0; ++w)
          if (c->tag[set * W + w] == (uint64_t)keys[i]) line = set * W + w;
      }
      c->stats[0] += 1;
      if (line >= 0) {
        c->stats[1] += 1;
        c->stamp[line] = c->epoch;                // tags do not change in this phase: order is free
        hit_mask[i] = 1;
        for (int d = 0; d < D; ++d) acc[d] += (double)c->data[line * D + d];
      } else {
        c->stats[2] += 1;
        hit_mask[i] = 0;
        if (keys[i] >= 0 && keys[i] < c->host_rows) miss_pos[n_missing++] = i;
      }
    }
    for (int d = 0; d < D; ++d) out[bag * D + d] = (float)acc[d];
  }
  return n_missing;
}

// Phase 2, "complete": follows the hits call on the same keys with nothing in between.  Every bag
// that holds missing keys gets their host rows, summed in double, added to what phase 1 left in
// out[bag, :] (one rounding to fp32); bags without missing keys keep their bits.  With
// insert_missing the distinct missing keys are then inserted under the epoch of phase 1, exactly
// as by oracle_cache_query.  hit_mask is phase 1's.
void oracle_cache_query_complete(oracle_cache* c, int64_t n_bags, const int64_t* keys,
                                 const int64_t* offsets, int64_t hotness, int64_t nnz,
                                 const uint8_t* hit_mask, int32_t insert_missing, float* out) {
  const int D = c->dim;
  std::vector<double> acc(D);
  for (int64_t bag = 0; bag < n_bags; ++bag) {
    std::fill(acc.begin(), acc.end(), 0.0);
    int64_t b0 = offsets ? offsets[bag] : bag * hotness;
    int64_t b1 = offsets ? offsets[bag + 1] : (bag + 1) * hotness;
    bool any = false;
    for (int64_t i = b0; i < b1; ++i) {
      if (hit_mask[i] || keys[i] < 0 || keys[i] >= c->host_rows) continue;
      any = true;
      for (int d = 0; d < D; ++d) acc[d] += (double)c->host_table[keys[i] * D + d];
    }
    if (any)
      for (int d = 0; d < D; ++d) out[bag * D + d] = (float)((double)out[bag * D + d] + acc[d]);
  }
  if (!insert_missing) return;
  std::vector<int64_t> where(nnz);
  for (int64_t i = 0; i < nnz; ++i) where[i] = hit_mask[i] ? 0 : -1;   // only the sign is read
  cache_insert_missing(c, keys, nnz, where);
}

// Manipulation operators of the cache (section 3, "embedding inference cache": query and
// manipulation operators, refresh; "Online model updating": cached embeddings are replaced when
// updates arrive).
//
// Insert: one call (epoch) that classifies and inserts like a query but pools nothing.
void oracle_cache_insert(oracle_cache* c, const int64_t* keys, int64_t n) {
  std::vector<float> sink((size_t)(n > 0 ? n : 1) * c->dim);
  oracle_cache_query(c, n, keys, nullptr, 1, n, 1, sink.data(), nullptr);
}

// Update: for i = 0..n-1 in order, if keys[i] is resident its cached row becomes rows[i, :] (so the
// last of several rows for one key wins).  Keys that are not resident are ignored; tags, stamps,
// the epoch and the statistics do not change.  Returns the number of resident keys met (with
// repetitions).
int64_t oracle_cache_update(oracle_cache* c, const int64_t* keys, const float* rows, int64_t n) {
  const int W = c->ways, D = c->dim;
  int64_t met = 0;
  for (int64_t i = 0; i < n; ++i) {
    if (keys[i] < 0) continue;
    int64_t set = cache_set_of((uint64_t)keys[i], c->num_sets);
    for (int w = 0; w < W; ++w) {
      if (c->tag[set * W + w] == (uint64_t)keys[i]) {
        std::memcpy(&c->data[(set * W + w) * D], &rows[i * D], sizeof(float) * D);
        ++met;
        break;
      }
    }
  }
  return met;
}

// Refresh: every resident line re-reads its row from the host table as it is now.
void oracle_cache_refresh(oracle_cache* c) {
  const int D = c->dim;
  for (size_t line = 0; line < c->tag.size(); ++line) {
    if (c->tag[line] == kEmptyTag) continue;
    std::memcpy(&c->data[line * D], &c->host_table[(int64_t)c->tag[line] * D], sizeof(float) * D);
  }
}

// ---------------------------------------------------------------------------------------------
// Embedding training cache, staged in host memory (section 1, "Online training": subsets of the
// embedding tables are loaded on demand into the GPU, the whole table lives in host memory).
// State: the host table [host_rows, dim] (the model), a working table [max_rows, dim] (what the
// GPU holds), a key -> row map with rows handed out in first-appearance order as by the hash above,
// and the key of every row.
//   load(keys): keys in array order; a key already resident keeps its row; a new key with
//     0 <= key < host_rows gets row = number of resident keys (if below max_rows, else it is
//     rejected, row -1) and the working row becomes a copy of host row `key`; a key outside the
//     host table is never loaded (row -1).
//   dump(evict): every resident row is written back to its host row; with evict the cache then
//     forgets all keys.
// Training between load and dump addresses the working table through the rows load returned.
// ---------------------------------------------------------------------------------------------
struct oracle_etc {
  int64_t max_rows, host_rows;
  int32_t dim;
  float* host;
  float* work;
  std::unordered_map<int64_t, int64_t> row_of;
  std::vector<int64_t> key_of;
  int64_t stats[3];   // loaded rows, rejected key occurrences, occurrences outside the host table (totals)
};

oracle_etc* oracle_etc_create(int64_t max_rows, int32_t dim, float* host, int64_t host_rows, float* work) {
  oracle_etc* e = new oracle_etc();
  e->max_rows = max_rows; e->host_rows = host_rows; e->dim = dim; e->host = host; e->work = work;
  e->stats[0] = e->stats[1] = e->stats[2] = 0;
  return e;
}
void oracle_etc_destroy(oracle_etc* e) { delete e; }

void oracle_etc_load(oracle_etc* e, const int64_t* keys, int64_t n, int64_t* rows) {
  for (int64_t i = 0; i < n; ++i) {
    const int64_t k = keys[i];
    if (k < 0 || k >= e->host_rows) { rows[i] = -1; e->stats[2] += 1; continue; }
    auto it = e->row_of.find(k);
    if (it != e->row_of.end()) { rows[i] = it->second; continue; }
    if ((int64_t)e->key_of.size() >= e->max_rows) { rows[i] = -1; e->stats[1] += 1; continue; }
    const int64_t r = (int64_t)e->key_of.size();
    e->row_of[k] = r;
    e->key_of.push_back(k);
    std::memcpy(e->work + r * e->dim, e->host + k * e->dim, sizeof(float) * e->dim);
    e->stats[0] += 1;
    rows[i] = r;
  }
}

void oracle_etc_dump(oracle_etc* e, int32_t evict) {
  for (size_t r = 0; r < e->key_of.size(); ++r)
    std::memcpy(e->host + e->key_of[r] * e->dim, e->work + (int64_t)r * e->dim, sizeof(float) * e->dim);
  if (evict) { e->row_of.clear(); e->key_of.clear(); }
}

// out[0] = resident keys, out[1..3] = the three running totals above
void oracle_etc_stats(const oracle_etc* e, int64_t* out) {
  out[0] = (int64_t)e->key_of.size();
  out[1] = e->stats[0]; out[2] = e->stats[1]; out[3] = e->stats[2];
}

}  // extern "C"
