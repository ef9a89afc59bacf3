// Host-side view of the embedding hash shared by hash.hip (owner) and emb.hip (hashed lookups).
#pragma once

#include "common.h"

struct hctr_hash {
  unsigned long long* slots;  // device, [n_buckets * 8] pairs {key, row}, 16 bytes each
  uint32_t n_buckets;         // 128-byte buckets of 8 slots
  int64_t capacity;           // slots asked for at creation
  int64_t max_rows;
  unsigned long long* size;   // device counter: keys held
};

namespace hctr {

// First 256 bytes of an insert-or-find (or cache insertion) workspace; n_miss and n_new are adjacent.
struct HashWsHeader {
  uint32_t n_miss;   // positions whose key was not found
  uint32_t n_new;    // distinct keys among them
  uint32_t n_scan;   // insert-or-find: how many positions can hold a missing key (0 once the table is full)
  uint32_t pad[61];
};

// Work arrays of the first-appearance dedup, each [n] unless noted.
struct DedupBuffers {
  uint32_t* flag;       // in: 1 where the key of position i is missing
  uint32_t* idx;        // scratch: exclusive scan of flag
  uint32_t* miss_pos;   // out: missing positions in ascending order, [n_miss]
  uint32_t* scr_slot;   // out: per missing position, the scratch slot of its key
  uint32_t* first;      // out: 1 where the missing position is its key's first appearance
  uint32_t* rank;       // out: exclusive scan of first
  uint32_t* scan_tmp;   // [scan_tmp_count(n)]
  uint32_t* scratch;    // [scratch_cap_max] per key met: the smallest missing position holding it
  uint32_t scratch_cap_max;     // dedup_scratch_capacity(n)
  uint32_t* n_miss;     // device: &HashWsHeader::n_miss
  uint32_t* n_new;      // device: &HashWsHeader::n_new
  const uint32_t* n_scan;  // device, or nullptr: only flag[0 .. *n_scan) can be set (nullptr: all n)
};
uint32_t dedup_scratch_capacity(uint32_t n_max);
hctr_status dedup_first_appearance(const int64_t* keys, uint32_t n, const DedupBuffers& B,
                                   hipStream_t stream);

size_t hash_ws_bytes(int64_t n_max);
// rows[i] = row of keys[i] or -1; insert != 0 inserts absent keys in first-appearance order first.
hctr_status hash_lookup(hctr_hash* h, const int64_t* keys, int64_t n, int insert, int64_t* rows,
                        void* ws, size_t ws_bytes, hipStream_t stream);
}  // namespace hctr
