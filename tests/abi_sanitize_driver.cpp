// Host-side checks of libhctr under AddressSanitizer / UndefinedBehaviorSanitizer: every entry point is
// called with arguments that the host must reject (or only measure) before anything is launched, so
// the run needs no GPU.  Linked against a build of the library whose HOST code is instrumented
// (paper_2210_08803_amd/build.py, build_host_sanitized).  Exit status 0 = every call answered as
// expected and the sanitizers stayed silent.
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "hctr.h"

static int fails = 0;
#define EXPECT(call, want) do { long got_ = (long)(call); if (got_ != (long)(want)) { \
  std::printf("line %d: %s = %ld, expected %ld (%s)\n", __LINE__, #call, got_, (long)(want), hctr_last_error()); ++fails; } } while (0)

int main() {
  void* dev = reinterpret_cast<void*>(4096);   // never dereferenced on the host
  int64_t base[2] = {0, 10}, num[2] = {10, 5};
  hctr_emb_desc d;
  std::memset(&d, 0, sizeof(d));
  d.num_slots = 2; d.dim = 8; d.table_dtype = HCTR_F32; d.combiner = HCTR_SUM; d.table = dev; d.total_rows = 15;
  d.slot_row_base = base; d.slot_num_rows = num;
  const int64_t* keys = reinterpret_cast<const int64_t*>(dev);
  EXPECT(hctr_emb_forward(nullptr, 1, keys, nullptr, 2, dev, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  hctr_emb_desc b = d; b.num_slots = 0;
  EXPECT(hctr_emb_forward(&b, 1, keys, nullptr, 2, dev, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  b = d; b.num_slots = HCTR_MAX_SLOTS + 1;
  EXPECT(hctr_emb_forward(&b, 1, keys, nullptr, 2, dev, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  b = d; b.dim = 6;
  EXPECT(hctr_emb_forward(&b, 1, keys, nullptr, 2, dev, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  b = d; b.total_rows = 14;
  EXPECT(hctr_emb_forward(&b, 1, keys, nullptr, 2, dev, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  b = d; b.total_rows = 0;
  EXPECT(hctr_emb_forward(&b, 1, keys, nullptr, 2, dev, dev, 1 << 20, nullptr), HCTR_E_UNSUPPORTED);
  EXPECT(hctr_emb_forward(&d, 1, keys, nullptr, 3, dev, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  EXPECT(hctr_emb_forward(&d, 1, keys, nullptr, 2, dev, nullptr, 1 << 20, nullptr), HCTR_E_WORKSPACE);
  EXPECT(hctr_emb_forward(&d, 1, keys, nullptr, 2, dev, dev, 16, nullptr), HCTR_E_WORKSPACE);
  EXPECT(hctr_emb_backward_sgd(&d, 1, keys, nullptr, 2, nullptr, 0.1f, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_emb_backward_dedup(&d, -1, keys, nullptr, 2, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  EXPECT(hctr_emb_backward_apply(&d, 1, nullptr, 2, nullptr, 0.1f, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_emb_workspace_init(nullptr, 1 << 20, nullptr), HCTR_E_WORKSPACE);
  EXPECT(hctr_emb_invalid_keys(nullptr, 0, nullptr, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_check_offsets(nullptr, 1, 1, dev, 8, nullptr), HCTR_E_NULL_PTR);
  // sizes: never shrinking in nnz_max, multiples of 256, across the layout switches
  size_t prev = 0;
  const int64_t points[] = {0, 1, 4095, 4096, 4097, 3145727, 3145728, 3145729, 4194304, 4194305, 8388607, 8388608,
                            8388609, 10000000, 12400000, 90000000, 2147483647};
  hctr_emb_desc big = d; big.num_slots = 1; big.dim = 128; big.total_rows = 1ll << 28; num[0] = 1ll << 28; base[0] = 0;
  for (int64_t n : points) {
    const size_t sz = hctr_emb_workspace_bytes(&big, 1, n);
    if (sz == 0 || sz % 256 != 0 || sz < prev) { std::printf("workspace_bytes(%lld) = %zu after %zu\n", (long long)n, sz, prev); ++fails; }
    prev = sz;
    const int64_t* nu; const uint32_t* ur; const uint32_t* so;
    EXPECT(hctr_emb_dedup_view(&big, 1, n, dev, sz, &nu, &ur, &so), HCTR_OK);
    EXPECT(hctr_emb_dedup_view(&big, 1, n, dev, 4096, &nu, &ur, &so), HCTR_E_WORKSPACE);
  }
  EXPECT(hctr_emb_workspace_bytes(&big, 1, -1), 0);
  EXPECT(hctr_emb_workspace_bytes(&big, 1, 1ll << 31), 0);
  num[0] = 10;
  // fused group
  hctr_group_table gt[2] = {{dev, 10, 8, 0}, {dev, 5, 16, 0}};
  hctr_group_lookup gl[3] = {{0, 0, 1, 0}, {1, 1, 2, 0}, {0, 1, 1, 0}};
  hctr_group_desc g = {2, 3, HCTR_F32, 0, gt, gl};
  EXPECT(hctr_group_forward(nullptr, 1, keys, nullptr, 4, (float*)dev, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_group_forward(&g, 2, keys, nullptr, 7, (float*)dev, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  EXPECT(hctr_group_forward(&g, 2, keys, nullptr, 8, (float*)dev, dev, 64, nullptr), HCTR_E_WORKSPACE);
  hctr_group_lookup bad_l[1] = {{2, 0, 1, 0}};
  hctr_group_desc gb = {2, 1, HCTR_F32, 0, gt, bad_l};
  EXPECT(hctr_group_forward(&gb, 2, keys, nullptr, 2, (float*)dev, dev, 1 << 20, nullptr), HCTR_E_INVALID_ARG);
  EXPECT(hctr_group_backward_sgd(&g, 2, keys, nullptr, 8, nullptr, 0.1f, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  if (hctr_group_workspace_bytes(&g, 1000, 8) <= hctr_group_workspace_bytes(&g, 2, 8)) { std::printf("group sizes\n"); ++fails; }
  EXPECT(hctr_group_workspace_bytes(nullptr, 2, 8), 0);
  // hash, training cache, inference cache
  hctr_hash* h = nullptr;
  EXPECT(hctr_hash_storage_bytes(10), 0);
  EXPECT(hctr_hash_storage_bytes(1024), 256 + 128 * 128);
  EXPECT(hctr_hash_create(nullptr, 1 << 20, 1024, 100, nullptr, &h), HCTR_E_NULL_PTR);
  EXPECT(hctr_hash_create(dev, 1 << 20, 1024, 900, nullptr, &h), HCTR_E_INVALID_ARG);
  EXPECT(hctr_hash_create(dev, 100, 1024, 100, nullptr, &h), HCTR_E_INVALID_ARG);
  EXPECT(hctr_hash_insert_or_find(nullptr, keys, 1, 1, (int64_t*)dev, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_hash_clear(nullptr, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_hash_workspace_bytes(1000) % 256, 0);
  hctr_etc* e = nullptr;
  EXPECT(hctr_etc_storage_bytes(0), 0);
  EXPECT(hctr_etc_workspace_bytes(-1), 0);
  EXPECT(hctr_etc_create(nullptr, dev, 8, (float*)dev, 10, dev, 1 << 20, nullptr, &e), HCTR_E_NULL_PTR);
  EXPECT(hctr_etc_load(nullptr, keys, 4, nullptr, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_etc_dump(nullptr, 1, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_etc_stats(nullptr, nullptr, nullptr), HCTR_E_NULL_PTR);
  hctr_cache* c = nullptr;
  EXPECT(hctr_cache_storage_bytes(8, 3, 16), 0);
  EXPECT(hctr_cache_storage_bytes(0, 4, 8), 0);
  EXPECT(hctr_cache_create(dev, 1 << 20, 8, 3, 16, (const float*)dev, 10, nullptr, &c), HCTR_E_INVALID_ARG);
  EXPECT(hctr_cache_create(dev, 16, 8, 4, 16, (const float*)dev, 10, nullptr, &c), HCTR_E_INVALID_ARG);
  EXPECT(hctr_cache_create(dev, 1 << 20, 8, 4, 16, nullptr, 10, nullptr, &c), HCTR_E_NULL_PTR);
  EXPECT(hctr_cache_query(nullptr, 1, 1, keys, nullptr, 1, 1, (float*)dev, nullptr, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_cache_query_hits(nullptr, 1, 1, keys, nullptr, 1, (float*)dev, nullptr, nullptr, nullptr, dev, 1 << 20, nullptr, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_cache_query_complete(nullptr, 1, 1, keys, nullptr, 1, 1, (float*)dev, dev, 1 << 20, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_cache_query_static(nullptr, 1, 1, keys, nullptr, 1, 1, (float*)dev, nullptr, nullptr), HCTR_E_NULL_PTR);
  EXPECT(hctr_cache_set_epoch_limit(nullptr, 100), HCTR_E_NULL_PTR);
  EXPECT(hctr_cache_set_small_call_limit(nullptr, 100), HCTR_E_NULL_PTR);
  EXPECT(hctr_cache_workspace_bytes(nullptr, 100), 0);
  if (hctr_last_error() == nullptr || hctr_last_error()[0] == 0) { std::printf("no error text\n"); ++fails; }
  std::printf(fails ? "abi sanitize driver: %d failure(s)\n" : "abi sanitize driver: clean\n", fails);
  return fails ? 1 : 0;
}
