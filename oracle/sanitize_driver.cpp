// Runs every function of the oracle once or more on small seeded inputs.  Built together with
// oracle.cpp under -fsanitize=address,undefined by oracle.sanitize_check(): a bad index, a read of
// freed or uninitialised-size memory, a signed overflow or a misaligned access in the oracle aborts
// the program.  TEST INFRASTRUCTURE ONLY, like the oracle itself.  Exit status 0 = clean.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

extern "C" {
int32_t oracle_hardware_threads(void);
int64_t oracle_rows_direct(int32_t, const int64_t*, const int64_t*, int64_t, const int64_t*, const int64_t*, int64_t*);
int64_t oracle_rows_direct_mt(int32_t, int32_t, const int64_t*, const int64_t*, int64_t, const int64_t*, const int64_t*, int64_t*);
void oracle_emb_forward(int32_t, int32_t, int32_t, const void*, int64_t, const int64_t*, const int64_t*, int64_t, float*);
void oracle_emb_forward_mt(int32_t, int32_t, int32_t, int32_t, const void*, int64_t, const int64_t*, const int64_t*, int64_t, float*);
int64_t oracle_emb_backward_sgd(int32_t, int32_t, int32_t, void*, int64_t, const int64_t*, const int64_t*, int64_t, const float*, float, int64_t*, int64_t*);
int64_t oracle_emb_backward_sgd_mt(int32_t, int32_t, int32_t, int32_t, void*, int64_t, const int64_t*, const int64_t*, int64_t, const float*, float, int64_t*, int64_t*);
void oracle_emb_forward_mixed(int32_t, int32_t, int32_t, const void*, int64_t, const int64_t*, const int64_t*, int64_t, int32_t, void*);
int64_t oracle_emb_backward_sgd_mixed(int32_t, int32_t, int32_t, void*, float*, int64_t, const int64_t*, const int64_t*, int64_t, int32_t, const void*, float);
void oracle_group_forward(int32_t, const void* const*, const int64_t*, const int32_t*, int32_t, int32_t, const int32_t*, const int32_t*, int64_t, const int64_t*, const int64_t*, float*);
int64_t oracle_group_backward_sgd(int32_t, void* const*, const int64_t*, const int32_t*, int32_t, int32_t, const int32_t*, const int32_t*, int64_t, const int64_t*, const int64_t*, const float*, float);
struct oracle_hash; struct oracle_cache; struct oracle_etc;
oracle_hash* oracle_hash_create(int64_t);
void oracle_hash_destroy(oracle_hash*);
int64_t oracle_hash_size(const oracle_hash*);
void oracle_hash_insert_or_find(oracle_hash*, const int64_t*, int64_t, int32_t, int64_t*);
oracle_cache* oracle_cache_create(int64_t, int32_t, int32_t, const float*, int64_t);
void oracle_cache_destroy(oracle_cache*);
void oracle_cache_set_epoch_limit(oracle_cache*, uint32_t);
void oracle_cache_stats(const oracle_cache*, int64_t*);
void oracle_cache_state(const oracle_cache*, uint64_t*, uint32_t*, float*);
void oracle_cache_query(oracle_cache*, int64_t, const int64_t*, const int64_t*, int64_t, int64_t, int32_t, float*, uint8_t*);
int64_t oracle_cache_query_hits(oracle_cache*, int64_t, const int64_t*, const int64_t*, int64_t, int64_t, float*, uint8_t*, int64_t*);
void oracle_cache_query_complete(oracle_cache*, int64_t, const int64_t*, const int64_t*, int64_t, int64_t, const uint8_t*, int32_t, float*);
void oracle_cache_insert(oracle_cache*, const int64_t*, int64_t);
int64_t oracle_cache_update(oracle_cache*, const int64_t*, const float*, int64_t);
void oracle_cache_refresh(oracle_cache*);
oracle_etc* oracle_etc_create(int64_t, int32_t, float*, int64_t, float*);
void oracle_etc_destroy(oracle_etc*);
void oracle_etc_load(oracle_etc*, const int64_t*, int64_t, int64_t*);
void oracle_etc_dump(oracle_etc*, int32_t);
void oracle_etc_stats(const oracle_etc*, int64_t*);
}

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {   // splitmix64
  uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
static float rndf() { return (float)((int64_t)(rnd() % 4001) - 2000) / 1024.0f; }
static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::printf("check failed: %s (line %d)\n", #c, __LINE__); ++fails; } } while (0)

int main() {
  const int S = 3, D = 8, rows_per = 40, batch = 50;
  const int64_t total = S * rows_per, n_bags = (int64_t)batch * S;
  std::vector<int64_t> base(S), num(S);
  for (int s = 0; s < S; ++s) { base[s] = s * rows_per; num[s] = rows_per; }
  for (int dtype = 0; dtype < 2; ++dtype) {
    for (int csr = 0; csr < 2; ++csr) {
      std::vector<int64_t> offsets(n_bags + 1, 0);
      if (csr) for (int64_t b = 0; b < n_bags; ++b) offsets[b + 1] = offsets[b] + (int64_t)(rnd() % 5);
      const int64_t nnz = csr ? offsets[n_bags] : n_bags;
      std::vector<int64_t> keys(nnz > 0 ? nnz : 1), rows(keys.size()), rows2(keys.size());
      for (int64_t i = 0; i < nnz; ++i) keys[i] = (int64_t)(rnd() % (rows_per + 4)) - 2;   // some outside
      const int64_t* off = csr ? offsets.data() : nullptr;
      const int64_t bad = oracle_rows_direct(S, base.data(), num.data(), n_bags, keys.data(), off, rows.data());
      CHECK(bad == oracle_rows_direct_mt(3, S, base.data(), num.data(), n_bags, keys.data(), off, rows2.data()));
      CHECK(rows == rows2);
      std::vector<float> t32(total * D);
      std::vector<uint16_t> t16(total * D);
      for (auto& x : t32) x = rndf();
      for (auto& x : t16) x = (uint16_t)(0x3000 + rnd() % 0x800);   // finite halves around 0.1 .. 0.5
      void* table = dtype ? (void*)t16.data() : (void*)t32.data();
      std::vector<float> out(n_bags * D), out2(n_bags * D), dY(n_bags * D);
      for (auto& x : dY) x = rndf();
      for (int comb = 0; comb < 2; ++comb) {
        oracle_emb_forward(D, dtype, comb, table, total, rows.data(), off, n_bags, out.data());
        oracle_emb_forward_mt(4, D, dtype, comb, table, total, rows.data(), off, n_bags, out2.data());
        CHECK(std::memcmp(out.data(), out2.data(), out.size() * 4) == 0);
        std::vector<uint16_t> o16(n_bags * D);
        oracle_emb_forward_mixed(D, dtype, comb, table, total, rows.data(), off, n_bags, 1, o16.data());
        std::vector<int64_t> uq(keys.size()), ct(keys.size());
        std::vector<float> a32 = t32, b32 = t32;
        std::vector<uint16_t> a16 = t16, b16 = t16;
        void* ta = dtype ? (void*)a16.data() : (void*)a32.data();
        void* tb = dtype ? (void*)b16.data() : (void*)b32.data();
        const int64_t u1 = oracle_emb_backward_sgd(D, dtype, comb, ta, total, rows.data(), off, n_bags, dY.data(), 0.05f, uq.data(), ct.data());
        const int64_t u2 = oracle_emb_backward_sgd_mt(5, D, dtype, comb, tb, total, rows.data(), off, n_bags, dY.data(), 0.05f, uq.data(), ct.data());
        CHECK(u1 == u2 && a32 == b32 && a16 == b16);
        if (dtype == 1) {
          std::vector<float> master(total * D, 0.25f);
          oracle_emb_backward_sgd_mixed(D, 1, comb, a16.data(), master.data(), total, rows.data(), off, n_bags, 1, o16.data(), 0.05f);
        }
      }
    }
  }
  {  // fused group: two tables of different widths, three lookups
    std::vector<float> ta(30 * 4), tb(20 * 8);
    for (auto& x : ta) x = rndf();
    for (auto& x : tb) x = rndf();
    void* tables[2] = {ta.data(), tb.data()};
    const int64_t trows[2] = {30, 20};
    const int32_t tdim[2] = {4, 8}, lt[3] = {0, 1, 0}, lc[3] = {0, 1, 1};
    const int64_t B = 17;
    std::vector<int64_t> offsets(B * 3 + 1, 0);
    for (int64_t b = 0; b < B * 3; ++b) offsets[b + 1] = offsets[b] + (int64_t)(rnd() % 4);
    std::vector<int64_t> keys(offsets.back() + 1);
    for (auto& k : keys) k = (int64_t)(rnd() % 33) - 1;
    std::vector<float> out(B * 16), dY(B * 16);
    for (auto& x : dY) x = rndf();
    oracle_group_forward(2, tables, trows, tdim, 0, 3, lt, lc, B, keys.data(), offsets.data(), out.data());
    oracle_group_backward_sgd(2, tables, trows, tdim, 0, 3, lt, lc, B, keys.data(), offsets.data(), dY.data(), 0.1f);
  }
  {  // hash: fill past the limit, find-only, negative keys
    oracle_hash* h = oracle_hash_create(100);
    std::vector<int64_t> keys(400), rows(400);
    for (auto& k : keys) k = (int64_t)(rnd() % 300) - 5;
    oracle_hash_insert_or_find(h, keys.data(), 400, 1, rows.data());
    oracle_hash_insert_or_find(h, keys.data(), 400, 0, rows.data());
    CHECK(oracle_hash_size(h) == 100);
    oracle_hash_insert_or_find(h, keys.data(), 0, 1, rows.data());
    oracle_hash_destroy(h);
  }
  {  // cache: every operator, ragged bags, the lowering of the call count
    const int64_t host_rows = 200, num_sets = 5, n_bags = 12;
    const int ways = 4, dim = 8;
    std::vector<float> host(host_rows * dim);
    for (auto& x : host) x = rndf();
    oracle_cache* c = oracle_cache_create(num_sets, ways, dim, host.data(), host_rows);
    oracle_cache_set_epoch_limit(c, 6);
    for (int it = 0; it < 25; ++it) {
      std::vector<int64_t> offsets(n_bags + 1, 0);
      for (int64_t b = 0; b < n_bags; ++b) offsets[b + 1] = offsets[b] + (int64_t)(rnd() % 6);
      const int64_t nnz = offsets[n_bags];
      std::vector<int64_t> keys(nnz + 1), miss(nnz + 1);
      for (auto& k : keys) k = (int64_t)(rnd() % (host_rows + 6)) - 3;
      std::vector<float> out(n_bags * dim);
      std::vector<uint8_t> hit(nnz + 1);
      if (it % 3 == 0) {
        oracle_cache_query(c, n_bags, keys.data(), offsets.data(), 0, nnz, it % 2, out.data(), hit.data());
      } else if (it % 3 == 1) {
        const int64_t m = oracle_cache_query_hits(c, n_bags, keys.data(), offsets.data(), 0, nnz, out.data(), hit.data(), miss.data());
        CHECK(m <= nnz);
        oracle_cache_query_complete(c, n_bags, keys.data(), offsets.data(), 0, nnz, hit.data(), it % 2, out.data());
      } else {
        oracle_cache_insert(c, keys.data(), nnz);
        std::vector<float> rows((nnz + 1) * dim, 1.5f);
        oracle_cache_update(c, keys.data(), rows.data(), nnz);
        oracle_cache_refresh(c);
      }
    }
    int64_t stats[6];
    oracle_cache_stats(c, stats);
    std::vector<uint64_t> tags(num_sets * ways);
    std::vector<uint32_t> stamps(num_sets * ways);
    std::vector<float> data(num_sets * ways * dim);
    oracle_cache_state(c, tags.data(), stamps.data(), data.data());
    CHECK(stats[0] == stats[1] + stats[2]);
    oracle_cache_destroy(c);
  }
  {  // training cache: load past the capacity, dump with and without eviction
    const int64_t host_rows = 60, max_rows = 25;
    const int dim = 4;
    std::vector<float> host(host_rows * dim, 0.5f), work(max_rows * dim, 0.f);
    oracle_etc* e = oracle_etc_create(max_rows, dim, host.data(), host_rows, work.data());
    for (int pass = 0; pass < 3; ++pass) {
      std::vector<int64_t> keys(90), rows(90);
      for (auto& k : keys) k = (int64_t)(rnd() % (host_rows + 8)) - 4;
      oracle_etc_load(e, keys.data(), 90, rows.data());
      for (auto& x : work) x += 0.125f;
      oracle_etc_dump(e, pass % 2);
    }
    int64_t st[4];
    oracle_etc_stats(e, st);
    oracle_etc_destroy(e);
  }
  CHECK(oracle_hardware_threads() >= 1);
  std::printf(fails ? "sanitize driver: %d check(s) failed\n" : "sanitize driver: clean\n", fails);
  return fails ? 1 : 0;
}
