/*
 * hctr.h - C ABI of the MI355X (gfx950) hashed sparse embedding library.
 *
 * The operations are the hot path of the embedding layer and of the inference cache described in
 * "Merlin HugeCTR: GPU-accelerated Recommender System Training and Inference" (RecSys'22):
 *   - key -> row lookup per slot, row gather and intra-slot reduction (section 1, "Localized slot
 *     embedding hash"), run forward and backward (section 1, "Hybrid sparse embedding"), with
 *     FP16 parameter storage as an option (section 1, "Mixed precision training");
 *   - the "embedding hash" itself: an open-addressing key -> row table with insert on miss
 *     (section 1, "Localized / Distributed slot embedding hash");
 *   - the level-1 GPU embedding cache with dynamic insertion, whose misses are served from system
 *     memory across the host link (section 3, "embedding inference cache", "Volatile database").
 *
 * General conventions
 *   Pointers   Every array argument says "device" or "host".  Device arrays are ordinary HIP device
 *              allocations; "pinned host" means hipHostMalloc'ed, device-mapped host memory.
 *   Ownership  The caller owns every buffer, including table, hash storage, cache storage and
 *              workspaces.  The library never allocates or frees device memory; the opaque handles
 *              are small host-side structs freed by the matching *_destroy.
 *   Streams    `stream` is a hipStream_t passed as void* (NULL = the default stream).  Compute
 *              calls enqueue work and return without waiting; only hctr_hash_size, hctr_cache_stats,
 *              hctr_etc_stats and hctr_emb_invalid_keys wait for the stream.  A workspace must stay untouched by
 *              the caller until the stream has passed the call that uses it.
 *   Errors     Every call returns an hctr_status.  Argument errors are found on the host before
 *              anything is launched.  A failing HIP call gives HCTR_E_DEVICE.  hctr_last_error()
 *              returns a thread-local message for the last failing call on this thread.
 *   Layout     Bags are numbered bag = sample * num_slots + slot.  Keys are int64, bag-major.
 *              CSR offsets are int64 [n_bags + 1], offsets[0] = 0, offsets[n_bags] = nnz,
 *              non-decreasing (not checked by the compute calls, see hctr_check_offsets).  offsets == NULL means exactly one key per bag.
 *              Pooled outputs and upstream gradients are [batch, num_slots, dim] row-major, fp32
 *              (or fp16 when the layer's io_dtype says so).
 *              Tables are [total_rows, dim] row-major in fp32 or fp16, 16-byte aligned.
 */
#ifndef HCTR_H_
#define HCTR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HCTR_OK = 0,
  HCTR_E_INVALID_ARG = -1,
  HCTR_E_NULL_PTR = -2,
  HCTR_E_WORKSPACE = -3,   /* workspace missing, misaligned (256 B), too small or never initialised */
  HCTR_E_UNSUPPORTED = -4,
  HCTR_E_DEVICE = -5
} hctr_status;

typedef enum { HCTR_F32 = 0, HCTR_F16 = 1 } hctr_dtype;
typedef enum { HCTR_SUM = 0, HCTR_MEAN = 1 } hctr_combiner;

#define HCTR_MAX_SLOTS 128
#define HCTR_MAX_GROUP_LOOKUPS 64   /* lookups (and tables) of one fused group, see hctr_group_desc */

typedef struct hctr_hash hctr_hash;   /* opaque */
typedef struct hctr_cache hctr_cache; /* opaque */
typedef struct hctr_etc hctr_etc;     /* opaque */

/*
 * Description of one fused embedding layer (section 1, "Localized slot embedding hash": every
 * slot's table lives on this GPU).
 *
 * Direct mode (hash == NULL): slot s owns rows [slot_row_base[s], slot_row_base[s] + slot_num_rows[s])
 * of `table`; key k of a bag of slot s addresses row slot_row_base[s] + k.  Slots may share a range.
 * A key outside [0, slot_num_rows[s]) has no row.
 * Hashed mode (hash != NULL): all slots share the key space of `hash`; the row of a key is the
 * value the hash holds for it (with insert_on_miss, absent keys are inserted first, as by
 * hctr_hash_insert_or_find); `table` must have at least the hash's max_rows rows and
 * total_rows = max_rows.  slot_row_base / slot_num_rows are ignored.
 * A key without a row contributes a zero vector in forward and nothing in backward (it still
 * counts in a mean's denominator) and is counted (hctr_emb_invalid_keys).
 */
typedef struct {
  int32_t num_slots;            /* S, 1..HCTR_MAX_SLOTS */
  int32_t dim;                  /* D > 0, multiple of 4 (fp32 table) or 8 (fp16 table) */
  int32_t table_dtype;          /* hctr_dtype of the table */
  int32_t combiner;             /* hctr_combiner */
  void* table;                  /* device [total_rows, dim] */
  int64_t total_rows;           /* 1 .. 2^32 - 2 */
  const int64_t* slot_row_base; /* host [S] (direct mode) */
  const int64_t* slot_num_rows; /* host [S] (direct mode) */
  hctr_hash* hash;              /* NULL = direct mode */
  int32_t insert_on_miss;       /* hashed mode, forward only: 1 = insert absent keys */
  int32_t io_dtype;             /* hctr_dtype of out and dY: HCTR_F32 (0), or HCTR_F16 for layers
                                   downstream that compute in half precision (section 1, "Mixed
                                   precision training"); sums are always formed in fp32 */
  int32_t reuse_forward_rows;   /* hashed mode: 1 = backward takes the rows that the last
                                   hctr_emb_forward on the same workspace found, instead of looking
                                   the keys up again.  The caller vouches that it was given the same
                                   keys (same nnz) and that no call has used the workspace since */
  float* master;                /* device [total_rows, dim] fp32 copy of an fp16 table, or NULL.
                                   With it backward updates the master row in fp32 and stores its
                                   rounding (nearest even) as the table row; forward reads only
                                   the fp16 table.  The caller keeps the two consistent at start. */
} hctr_emb_desc;

/* Bytes of workspace that forward and backward need for up to nnz_max keys (multiple of 256). */
size_t hctr_emb_workspace_bytes(const hctr_emb_desc* desc, int64_t batch, int64_t nnz_max);

/* Must run once on a fresh workspace before its first use (it zeroes the counter of keys without
 * a row, which forward and backward only ever add to, and marks the workspace as counted); calling
 * it again resets that counter and forgets the last dedup result.  Forward and backward themselves
 * compute the same results on a workspace that skipped this call (they never read the counter), but
 * hctr_emb_invalid_keys then returns HCTR_E_WORKSPACE instead of a number. */
hctr_status hctr_emb_workspace_init(void* ws, size_t ws_bytes, void* stream);

/*
 * Forward: out[b, s, :] = w * sum_j T[row(key_j), :] over the keys of bag (b, s); w = 1 for
 * HCTR_SUM, 1/hotness for HCTR_MEAN (hotness = number of keys of the bag); an empty bag gives
 * zeros.  fp16 tables are converted exactly to fp32; accumulation is fp32 in a fixed order, so two
 * runs give the same bits.  (Section 1, "Localized slot embedding hash": lookup + intra-slot
 * reduction.)
 *   keys    device [nnz]           offsets device [batch*S + 1] or NULL (then nnz == batch*S)
 *   out     device [batch, S, dim] in desc->io_dtype (fp16: the fp32 sum rounded to nearest even),
 *           16-byte aligned, fully overwritten
 *   ws      device, >= hctr_emb_workspace_bytes(desc, batch, nnz), 256-byte aligned
 * batch == 0 is accepted and does nothing.
 */
hctr_status hctr_emb_forward(const hctr_emb_desc* desc, int64_t batch, const int64_t* keys,
                             const int64_t* offsets, int64_t nnz, void* out, void* ws,
                             size_t ws_bytes, void* stream);

/*
 * Backward with fused SGD: for every distinct table row r addressed by the batch,
 *   g_r = sum over the occurrences (bag, j) of r of w_bag * dY[bag, :]   (w as in forward),
 *   T[r, :] <- T[r, :] - lr * g_r,
 * computed in fp32 in a fixed order (deterministic); fp16 tables are widened, updated in fp32 and
 * stored with round-to-nearest-even.  Rows not addressed keep their bits.  Internally: key -> row,
 * stable radix sort of (row, bag) pairs, run boundaries (= dedup), segmented reduction of dY fused
 * with the row update.  In hashed mode keys are looked up only (never inserted); unknown keys are
 * skipped.  (Section 1, "Hybrid sparse embedding" names the backward pass; the paper gives no
 * optimizer, plain SGD is the benchmark's.)
 *   dY      device [batch, S, dim] in desc->io_dtype (fp16 is widened exactly), 16-byte aligned
 * With desc->master the update goes to the fp32 master row and the fp16 table row becomes its
 * rounding (see hctr_emb_desc).
 * The dedup result of the call stays in the workspace, see hctr_emb_dedup_view.
 */
hctr_status hctr_emb_backward_sgd(const hctr_emb_desc* desc, int64_t batch, const int64_t* keys,
                                  const int64_t* offsets, int64_t nnz, const void* dY, float lr,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * The two halves of hctr_emb_backward_sgd as separate calls, for callers that overlap them with
 * other work.  hctr_emb_backward_dedup does the key-only part (key -> row, sort, run boundaries): it
 * reads keys / offsets and writes `ws`, so in direct mode it may run on another stream at the same
 * time as hctr_emb_forward of the same batch, even on the same workspace (in hashed mode it looks
 * keys up in the hash and must be ordered after the forward that inserts them).
 * hctr_emb_backward_apply then reduces dY over the sorted occurrences and updates the table; it
 * must be ordered after the dedup call on the same `ws`, with the same batch, offsets, nnz and
 * combiner.  One dedup call serves any number of apply calls (different dY or lr), one after the
 * other on the stream; two apply calls on one `ws` must not overlap.
 */
hctr_status hctr_emb_backward_dedup(const hctr_emb_desc* desc, int64_t batch, const int64_t* keys,
                                    const int64_t* offsets, int64_t nnz, void* ws, size_t ws_bytes,
                                    void* stream);
hctr_status hctr_emb_backward_apply(const hctr_emb_desc* desc, int64_t batch, const int64_t* offsets,
                                    int64_t nnz, const void* dY, float lr, void* ws, size_t ws_bytes,
                                    void* stream);

/*
 * Where the last backward call on `ws` left its dedup result (device pointers into ws, valid until
 * ws is reused; `nnz` must be the nnz of that call, the workspace is laid out by it): *num_unique -> one int64 U; *uniq_rows -> uint32 [U] distinct global rows in
 * ascending order; *seg_offsets -> uint32 [U + 1], seg_offsets[u+1] - seg_offsets[u] = number of
 * occurrences of uniq_rows[u].  Pure pointer arithmetic, no device work.
 */
hctr_status hctr_emb_dedup_view(const hctr_emb_desc* desc, int64_t batch, int64_t nnz, void* ws,
                                size_t ws_bytes, const int64_t** num_unique,
                                const uint32_t** uniq_rows, const uint32_t** seg_offsets);

/*
 * The compute calls do not check CSR offsets (a kernel that trusts broken offsets reads outside its
 * buffers).  This call does, for callers that cannot vouch for their input: offsets device
 * [n_bags + 1] must start at 0, end at nnz and never decrease; otherwise HCTR_E_INVALID_ARG.  ws:
 * device, 8 bytes, 8-byte aligned.  Waits for the stream.
 */
hctr_status hctr_check_offsets(const int64_t* offsets, int64_t n_bags, int64_t nnz, void* ws, size_t ws_bytes,
                               void* stream);

/* Number of keys without a row seen by all forward and backward calls on `ws` since
 * hctr_emb_workspace_init (host int64; waits for the stream).  HCTR_E_WORKSPACE if `ws` does not
 * carry the mark that hctr_emb_workspace_init leaves (the memory was never initialised, or was
 * overwritten since). */
hctr_status hctr_emb_invalid_keys(const void* ws, size_t ws_bytes, void* stream, int64_t* count);

/*
 * Fused group of lookups (section 4, "Future Work": one embedding that fuses tables of different
 * vector size and combiner and takes both dense and sparse inputs).  A group has T tables, each
 * with its own allocation, row count and width, and L lookups; lookup l reads table
 * lookups[l].table with its own combiner, and several lookups may read the same table (their
 * gradients then meet in one update).  Keys are direct row indices into the lookup's table.
 *   Bags      bag = sample * L + l; keys bag-major.
 *   Input     sparse: CSR offsets [batch * L + 1] as for a layer.  Dense: offsets == NULL, every
 *             sample brings exactly lookups[l].hotness keys for lookup l, so nnz = batch * sum of
 *             hotness (for backward the library writes the CSR offsets of that shape into the workspace,
 *             unless every lookup has hotness 1).
 *   Output    out / dY are fp32 [batch, width] row-major, width = sum of the lookups' table widths;
 *             lookup l occupies columns [col_l, col_l + dim_l), col_l = sum of the widths before it.
 *   Rows      for the dedup the tables' rows are numbered over their concatenation in tables[]
 *             order; the total must stay below 2^32 - 1.
 * A key outside [0, num_rows) contributes nothing and is counted, as for a layer.  The workspace
 * starts with the same header as a layer's: hctr_emb_workspace_init and hctr_emb_invalid_keys apply.
 * The host arrays are read during the call only.
 */
typedef struct {
  void* data;        /* device [num_rows, dim], 16-byte aligned */
  int64_t num_rows;  /* >= 1 */
  int32_t dim;       /* > 0, multiple of 4 (fp32 tables) or 8 (fp16 tables) */
  int32_t reserved;  /* 0 */
} hctr_group_table;

typedef struct {
  int32_t table;     /* index into tables[] */
  int32_t combiner;  /* hctr_combiner */
  int32_t hotness;   /* dense input: keys per sample, >= 1; ignored for sparse input */
  int32_t reserved;  /* 0 */
} hctr_group_lookup;

typedef struct {
  int32_t num_tables;                /* T, 1..HCTR_MAX_GROUP_LOOKUPS */
  int32_t num_lookups;               /* L, 1..HCTR_MAX_GROUP_LOOKUPS */
  int32_t table_dtype;               /* hctr_dtype shared by all tables; out and dY are fp32 */
  int32_t reserved;                  /* 0 */
  const hctr_group_table* tables;    /* host [T] */
  const hctr_group_lookup* lookups;  /* host [L] */
} hctr_group_desc;

/* Workspace bytes for calls with at most nnz_max keys and `batch` samples (0 on invalid arguments). */
size_t hctr_group_workspace_bytes(const hctr_group_desc* desc, int64_t batch, int64_t nnz_max);

/* out[b, col_l : col_l + dim_l] = w * sum of the rows named by bag (b, l); w = 1 (sum) or
 * 1 / number of keys in the bag (mean); empty bag = zeros.  keys device [nnz]; offsets device or
 * NULL (dense); out device [batch, width]; ws device, 256-byte aligned. */
hctr_status hctr_group_forward(const hctr_group_desc* desc, int64_t batch, const int64_t* keys,
                               const int64_t* offsets, int64_t nnz, float* out, void* ws, size_t ws_bytes,
                               void* stream);

/* Backward with plain SGD for every table of the group: row r of table t gets
 * r -= lr * sum over the occurrences of (t, r) in the call, whatever lookup they came through,
 * of w * dY[b, col_l : col_l + dim_l].  Same dedup / segmented reduction as hctr_emb_backward_sgd;
 * additions in an order fixed by the sorted (row, bag) list. */
hctr_status hctr_group_backward_sgd(const hctr_group_desc* desc, int64_t batch, const int64_t* keys,
                                    const int64_t* offsets, int64_t nnz, const float* dY, float lr,
                                    void* ws, size_t ws_bytes, void* stream);

/*
 * Embedding hash (section 1, the "embedding hash" layers): open addressing, 16-byte slots
 * {key, row} in 128-byte buckets, probed by groups of 8 lanes.  Valid keys are 0 <= key < 2^63.
 * Rows are dense: the table holds keys with rows 0 .. size-1, a row never changes, and a call
 * assigns new rows in the order in which new keys first appear in its key array.
 *   capacity  number of slots (>= 64); max_rows = most keys it will ever hold, 1 <= max_rows <=
 *             0.8 * capacity.  Once size == max_rows further new keys are rejected (row -1).
 *   storage   device, >= hctr_hash_storage_bytes(capacity), 256-byte aligned; hctr_hash_create
 *             enqueues its initialisation on `stream`.
 */
size_t hctr_hash_storage_bytes(int64_t capacity);
hctr_status hctr_hash_create(void* storage, size_t storage_bytes, int64_t capacity, int64_t max_rows,
                             void* stream, hctr_hash** out);
size_t hctr_hash_workspace_bytes(int64_t n_max);
/*
 *   keys  device [n]; rows device [n] int64, row of each key or -1 (absent / rejected / negative key)
 *   insert 0 = look up only, 1 = insert absent keys first
 *   ws    device, >= hctr_hash_workspace_bytes(n), 256-byte aligned (may be NULL when n == 0)
 */
hctr_status hctr_hash_insert_or_find(hctr_hash* hash, const int64_t* keys, int64_t n, int32_t insert,
                                     int64_t* rows, void* ws, size_t ws_bytes, void* stream);
/* Number of keys held (host int64; waits for the stream). */
hctr_status hctr_hash_size(hctr_hash* hash, void* stream, int64_t* size);
/* Forgets every key (size 0, all slots empty); enqueued on `stream`. */
hctr_status hctr_hash_clear(hctr_hash* hash, void* stream);
void hctr_hash_destroy(hctr_hash* hash);

/*
 * Embedding training cache staged in host memory (section 1, "Online training": the Embedding
 * Training Cache loads subsets of the embedding tables on demand into the GPU; its "Staged-PS"
 * keeps the whole table in host memory).  The model is host_table, pinned host [host_rows, dim]
 * fp32, a key being its row index.  The GPU holds a working table, device [max_rows, dim] fp32,
 * addressed through `hash` (max_rows = the hash's): train on it with a hashed-mode layer
 * (hctr_emb_desc.hash = hash, insert_on_miss = 0, table = the working table).  One pass:
 *   hctr_etc_load   keys device [n], the keys the coming batches will use (repeats allowed).  Keys
 *                   already resident keep their rows.  New keys with 0 <= key < host_rows get rows
 *                   in first-appearance order, as by hctr_hash_insert_or_find, and their host rows
 *                   are copied into the working table (one read of the row across the host link).
 *                   New keys that find no room (size == max_rows) and keys outside the host table
 *                   are not loaded (row -1, counted); a layer treats them as keys without a row.
 *                   rows: device [n] or NULL, receives the row of every key.
 *   (training calls on the working table)
 *   hctr_etc_dump   writes every resident row back to its host row (one write of the row across the
 *                   host link); with evict != 0 the hash is then cleared, so the next load starts
 *                   from an empty working table.  The host must not read host_table before the
 *                   stream has passed the call.
 *   storage   device, >= hctr_etc_storage_bytes(max_rows), 256-byte aligned (counters and the key of
 *             every row); ws device, >= hctr_etc_workspace_bytes(n), 256-byte aligned.
 *   hctr_etc_stats  host int64 [4] = resident keys, rows loaded, rejected key occurrences,
 *                   occurrences outside the host table (the last three running totals); waits for
 *                   the stream.
 * The handle does not own hash, tables or storage.
 */
size_t hctr_etc_storage_bytes(int64_t max_rows);
size_t hctr_etc_workspace_bytes(int64_t n_max);
hctr_status hctr_etc_create(hctr_hash* hash, void* table, int32_t dim, float* host_table, int64_t host_rows,
                            void* storage, size_t storage_bytes, void* stream, hctr_etc** out);
hctr_status hctr_etc_load(hctr_etc* etc, const int64_t* keys, int64_t n, int64_t* rows, void* ws,
                          size_t ws_bytes, void* stream);
hctr_status hctr_etc_dump(hctr_etc* etc, int32_t evict, void* stream);
hctr_status hctr_etc_stats(hctr_etc* etc, void* stream, int64_t* stats);
void hctr_etc_destroy(hctr_etc* etc);

/*
 * Inference embedding cache (section 3, "embedding inference cache"): set-associative, num_sets
 * sets of `ways` lines (ways a power of two, 1..64), each line one fp32 row of `dim` values
 * (multiple of 4).  The backing store is a table in pinned host memory read by the GPU across the
 * host link (section 3, "Volatile database"); key = row index in that table.
 * Set of a key: x = key * 0x9E3779B97F4A7C15 mod 2^64; x ^= x >> 32; set = x mod num_sets.
 * Replacement is LRU at the granularity of a query call, see hctr_cache_query.
 *   storage     device, >= hctr_cache_storage_bytes(...), 256-byte aligned; initialised on `stream`
 *   host_table  pinned host [host_rows, dim] fp32, must stay valid while the cache lives
 */
size_t hctr_cache_storage_bytes(int64_t num_sets, int32_t ways, int32_t dim);
hctr_status hctr_cache_create(void* storage, size_t storage_bytes, int64_t num_sets, int32_t ways,
                              int32_t dim, const float* host_table, int64_t host_rows, void* stream,
                              hctr_cache** out);
size_t hctr_cache_workspace_bytes(const hctr_cache* cache, int64_t nnz_max);
/* Calls with at most max_keys keys (0..8192, default 8192; rows of at most 256 values) run as two
 * fused kernels instead of the general pipeline, because at that size launches cost more than
 * bytes.  Both paths give identical results; 0 switches the fused path off. */
hctr_status hctr_cache_set_small_call_limit(hctr_cache* cache, int64_t max_keys);
/* The recency stamps are 32-bit counts of the query / insert calls made so far; the count lives in
 * device memory and is read and advanced by the kernels, so a call captured in a HIP graph may be
 * replayed (each replay is one more call).  The host keeps a copy to see the limit coming, which
 * replays do not advance: hctr_cache_stats brings it up to date, so a server that replays captured
 * calls should read the statistics at least once every 2^31 replays.  A call that finds
 * the count at or above `limit` (2 .. 2^32 - 256, the default) first lowers every stamp and the
 * count by limit / 2, stamps at or below that becoming 0 = never used (among those the lowest way
 * is replaced first).  The order of the ways used within the last limit / 2 calls is unchanged, so
 * a cache serves any number of calls.  Lower limits exist for tests; set one before the count
 * has passed it (a count far above the limit comes down by only limit / 2 per call).  (The paper gives no
 * replacement policy; section 3, "embedding inference cache", only names dynamic insertion.) */
hctr_status hctr_cache_set_epoch_limit(hctr_cache* cache, int64_t limit);
/*
 * One query: out[bag, :] = sum of the vectors of the bag's keys (fp32, fixed order).  Every key is
 * classified against the cache contents at call entry: a hit reads the cached line and marks it
 * used in this call; a miss reads host_table[key] (a key outside [0, host_rows) reads as zeros and
 * is never cached).  With insert_missing != 0 the distinct missing keys are then inserted in order
 * of first appearance: into the lowest-index empty way of their set, else over the least recently
 * used way among those not used in this call (ties: lowest way), else the insert is skipped.
 *   n_bags   batch * num_slots bags;  keys device [nnz]
 *   offsets  device [n_bags + 1] or NULL = fixed hotness nnz / n_bags (nnz must divide evenly);
 *            bags may be empty, also all of them (nnz = 0: zeros in out, nothing inserted); every
 *            call counts as one call for the replacement order, also one without keys or without
 *            bags (batch = 0, which reads and writes nothing else and needs no workspace)
 *   out      device [n_bags, dim] fp32;  hit_mask device [nnz] uint8 (1 = hit) or NULL
 *   ws       device, >= hctr_cache_workspace_bytes(cache, nnz), 256-byte aligned
 */
hctr_status hctr_cache_query(hctr_cache* cache, int64_t batch, int32_t num_slots, const int64_t* keys,
                             const int64_t* offsets, int64_t nnz, int32_t insert_missing, float* out,
                             uint8_t* hit_mask, void* ws, size_t ws_bytes, void* stream);
/*
 * Manipulation operators (section 3, "embedding inference cache": query and manipulation operators,
 * dynamic insertion, asynchronous refresh; "Online model updating": cached embeddings are replaced
 * when updates arrive and the cache periodically re-reads its contents).
 *
 * hctr_cache_query_async  as hctr_cache_query, and records `results_ready_event` (a hipEvent_t
 *     created by the caller) on `stream` as soon as `out` and `hit_mask` are complete, i.e. before
 *     the insertion work of the call is enqueued: a consumer on another stream can wait for the
 *     event and overlap its own work with the insertion.
 * hctr_cache_insert   one call (epoch) that classifies `keys` [n] and inserts the missing ones
 *     exactly as hctr_cache_query(insert_missing = 1) does, but pools nothing.
 * hctr_cache_update   for every key of `keys` [n] that is resident, the cached row is replaced by
 *     its row of `rows` (device [n, dim] fp32, 16-byte aligned); of several rows given for one key
 *     the last one wins.  Keys that are not resident are ignored; tags, stamps, statistics and the
 *     call counter do not change.  ws >= hctr_cache_workspace_bytes(cache, n).
 * hctr_cache_refresh  every resident line re-reads its row from the host table as it is now.
 */
hctr_status hctr_cache_query_async(hctr_cache* cache, int64_t batch, int32_t num_slots, const int64_t* keys,
                                   const int64_t* offsets, int64_t nnz, int32_t insert_missing, float* out,
                                   uint8_t* hit_mask, void* ws, size_t ws_bytes, void* stream,
                                   void* results_ready_event);
/*
 * The query in two phases, for a consumer that starts on the hits while the missing rows are still
 * crossing the host link (section 3: parameter migration overlapped with the dense network;
 * "embedding inference cache": dynamic insertion, asynchronous mechanisms).
 *
 * hctr_cache_query_hits  one call (it advances the call count like hctr_cache_query): classifies
 *     every key, marks the hits used, writes hit_mask, and pools ONLY the hits: out[bag, :] = sum of
 *     the cached vectors of the bag's resident keys, a missing key adding nothing yet.  Nothing is
 *     read across the host link.  With miss_positions != NULL it also lists the positions of the keys
 *     that are missing and lie inside the host table, in ascending order (device uint32 [nnz]; their
 *     number goes to *n_missing, device uint32; both NULL or both given; costs up to four small
 *     launches).  hits_ready_event (a hipEvent_t of the caller's, or NULL) is recorded on `stream`
 *     behind this work.
 * hctr_cache_query_complete  the rest of the same query, on any stream ordered after the hits call
 *     (typically a side stream that waits for the event): every bag that holds missing keys gets
 *     their host rows added to what the first phase left in out (bags without keys keep their bits),
 *     each distinct missing row crossing the host link once; with insert_missing != 0 the missing
 *     keys are then inserted exactly as by hctr_cache_query.  It must be given the keys, offsets,
 *     nnz, out and ws of the hits call, with ws untouched in between, and no other call on this cache
 *     may run between the two.  The consumer may read the hit-only `out` after the event, but must be
 *     done with it before the stream reaches this call; the final `out` is ready when the stream has
 *     passed it.
 * After the pair, the cache (tags, stamps, rows, statistics) is what hctr_cache_query with the same
 * insert_missing would have left; `out` equals its output up to the order of the fp32 additions
 * (hits first, then the missing rows).
 *
 * Ordering: calls on one cache (query, the two phases, insert, update, refresh) must not overlap in
 * time; order them on one stream or with events.  A refresh or update that ran beside a query could
 * hand it a row that is half old and half new.
 */
hctr_status hctr_cache_query_hits(hctr_cache* cache, int64_t batch, int32_t num_slots, const int64_t* keys,
                                  const int64_t* offsets, int64_t nnz, float* out, uint8_t* hit_mask,
                                  uint32_t* miss_positions, uint32_t* n_missing, void* ws, size_t ws_bytes,
                                  void* stream, void* hits_ready_event);
hctr_status hctr_cache_query_complete(hctr_cache* cache, int64_t batch, int32_t num_slots, const int64_t* keys,
                                      const int64_t* offsets, int64_t nnz, int32_t insert_missing, float* out,
                                      void* ws, size_t ws_bytes, void* stream);
hctr_status hctr_cache_insert(hctr_cache* cache, const int64_t* keys, int64_t n, void* ws, size_t ws_bytes,
                              void* stream);
hctr_status hctr_cache_update(hctr_cache* cache, const int64_t* keys, const float* rows, int64_t n, void* ws,
                              size_t ws_bytes, void* stream);
hctr_status hctr_cache_refresh(hctr_cache* cache, void* stream);

/*
 * hctr_cache_query for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, same results and same effect
 * on the cache as hctr_cache_query, without `ws` / `ws_bytes`.  The work arrays of the call live in
 * a device array of HCTR_STATIC_SCRATCH_BYTES bytes inside the library, of which every GPU the
 * library runs on holds one copy until the process ends.  The call allocates and frees nothing.
 *   Limit   nnz <= HCTR_STATIC_MAX_KEYS; beyond it, or when the call's work arrays would not fit
 *           (only possible for rows wider than 256 values, or with the small-call limit lowered and
 *           rows wider than 128 values), HCTR_E_UNSUPPORTED and nothing is launched.
 *   Sharing all calls on one GPU use that GPU's array: two calls of this function that overlap in
 *           time on one GPU (different streams, different caches) race and give wrong results; calls
 *           that follow each other on one stream are safe, the array needs no clearing in between.
 *   Set-up  the first call on a device looks up the array's address (once per device, with that
 *           device current); make that call outside graph capture.
 */
#define HCTR_STATIC_MAX_KEYS 8192
#define HCTR_STATIC_SCRATCH_BYTES (8u << 20)
hctr_status hctr_cache_query_static(hctr_cache* cache, int64_t batch, int32_t num_slots, const int64_t* keys,
                                    const int64_t* offsets, int64_t nnz, int32_t insert_missing, float* out,
                                    uint8_t* hit_mask, void* stream);

/* stats[6] (host) = cumulative {keys queried, hits, misses, inserts, evictions, skipped inserts};
 * waits for the stream. */
hctr_status hctr_cache_stats(hctr_cache* cache, void* stream, int64_t stats[6]);
/* Device pointers to the cache state inside its storage (for inspection): tags uint64
 * [num_sets, ways] (all ones = empty), stamps uint32 [num_sets, ways], data fp32 [num_sets*ways, dim]. */
hctr_status hctr_cache_state_view(hctr_cache* cache, const uint64_t** tags, const uint32_t** stamps,
                                  const float** data);
void hctr_cache_destroy(hctr_cache* cache);

/* Thread-local text of the last error on this thread; never NULL. */
const char* hctr_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HCTR_H_ */
