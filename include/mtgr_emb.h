/*
 * mtgr_emb.h - C ABI of the MI355X sparse-embedding library.
 *
 * One GPU's share of the embedding path of a generative recommendation model:
 *   tagged IDs of merged tables (Sec. 3.2, Eq. 8)  ->  ID deduplication (Sec. 3.3)
 *   ->  dynamic hash table find-or-insert and row gather (Sec. 3.1)  ->  expand
 *   (forward);  per-ID gradient aggregation  ->  row-wise Adagrad on the activated
 *   rows (Sec. 2 "Backward Update", App. C "Gradient Accumulation");  eviction and
 *   key-structure expansion (Sec. 3.1 "Capacity Expansion").
 *
 * Conventions (every entry point):
 *   - Pointers marked [dev] are device (HBM) addresses, [host] are host addresses.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     are asynchronous on it unless stated; the library never synchronises behind
 *     the caller's back except in ht_stats.
 *   - The caller owns every buffer.  The library allocates and frees no device
 *     memory; it keeps raw pointers handed to it until they are replaced
 *     (ht_rehash) or the table is destroyed.  A buffer may be released once the
 *     stream has passed the last call that used it.
 *   - `n_dev` [dev, may be NULL]: address of the true element count (int64), e.g.
 *     the n_unique written by emb_dedup.  Kernels are launched over `n_max` and
 *     read the count on the device, so no host read-back sits on the path.  NULL
 *     means "exactly n_max elements".
 *   - Return value: EMB_OK (0) or a negative emb_status (ht_find_or_insert may also
 *     return the positive EMB_CHECK_STATUS).  Conditions that only the device can
 *     see (load-factor limit reached, out of row storage, probe sequence exhausted)
 *     set sticky bits in the table's device status word, reported by ht_stats; the
 *     affected elements get row index -1 and nothing is left half-inserted.
 *   - Calls on the same table must be ordered (one stream, or events).  Two calls
 *     that overlap on one table race.
 *   - Valid keys have bit 63 clear (Eq. 8 keeps the top bit zero).  2^64-1 and
 *     2^64-2 are reserved for "empty" and "deleted" slots.
 */
#ifndef MTGR_EMB_H
#define MTGR_EMB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct emb_table emb_table_t; /* opaque host object; owns no device memory */

typedef enum { EMB_F32 = 0, EMB_BF16 = 1 } emb_dtype_t;

typedef enum {
    EMB_OK = 0,
    EMB_ERR_INVALID_ARG = -1,
    EMB_ERR_KEY_RANGE = -2,
    EMB_ERR_WORKSPACE = -3,   /* workspace too small or misaligned */
    EMB_ERR_NO_STORAGE = -4,  /* no key storage / not enough row chunks registered for n_max inserts */
    EMB_ERR_HIP = -5,         /* a HIP runtime call failed */
    EMB_ERR_TOO_LARGE = -7,   /* emb_dedup_noalloc: n beyond EMB_DEDUP_NOALLOC_MAX_KEYS */
    EMB_ERR_NEED_REHASH = -6, /* ht_rehash: the live keys do not fit under the limit of the new structure */
    /* Positive, ht_find_or_insert only: the kernels were launched, but the host-side upper bounds could not prove
     * that n_max new keys fit.  The device admits new keys only while live + deleted slots stay within
     * floor(max_load_factor * capacity) and rows remain; compare ht_stats().refused before and after to learn
     * whether any were turned away. */
    EMB_CHECK_STATUS = 1
} emb_status_t;

/* bits of ht_stats_t.status (sticky, device-side; cleared by ht_clear_status) */
#define EMB_DEV_PROBE_EXHAUSTED 1u /* every line of a key's probe sequence was visited without finding room */
#define EMB_DEV_OUT_OF_ROWS 2u     /* new keys were turned away because the registered chunks are full */
#define EMB_DEV_BAD_KEY 4u         /* a key with bit 63 set was passed; it got row index -1 */
#define EMB_DEV_NEED_REHASH 8u     /* new keys were turned away at the load-factor limit (Sec. 3.1 "Capacity Expansion") */

typedef struct {
    int32_t dim;             /* elements per embedding row; row bytes must be a multiple of 16 */
    int32_t dtype;           /* emb_dtype_t of the stored rows */
    float init_scale;        /* new rows are uniform on [-init_scale, init_scale) */
    float max_load_factor;   /* expansion trigger, (live+deleted)/capacity; 0 -> 0.75 (Sec. 3.1).  At most 1.0;
                                values above 0.95 let probe sequences grow very long and serve tests only */
    int32_t chunk_rows_log2; /* every value chunk holds 2^this rows */
    int32_t count_probes;    /* nonzero: maintain the probe/CAS/allocation counters of ht_stats_t */
} emb_table_desc_t;

typedef struct {
    uint64_t live;          /* keys present */
    uint64_t tombstones;    /* deleted slots not yet reclaimed by a rehash */
    uint64_t capacity;      /* slots in the key structure (power of two) */
    uint64_t rows_used;     /* high-water mark of the row allocator */
    uint64_t rows_free;     /* rows on the free list (from evictions) */
    uint64_t rows_capacity; /* rows in all registered chunks */
    uint64_t n_rehash;
    uint64_t n_chunks;
    uint64_t status;        /* EMB_DEV_* bits */
    /* counters, only maintained when count_probes != 0 */
    uint64_t lookups;       /* keys probed by find / find-or-insert */
    uint64_t probes;        /* 128-byte slot lines inspected for them */
    uint64_t cas_attempts;
    uint64_t cas_failures;
    uint64_t alloc_atomics; /* atomics issued by admission and the row allocator (per block of 512 keys that brings new keys) */
    /* hot store (ht_set_hot_storage); all zero without one */
    uint64_t hot_rows_used;     /* high-water mark of the hot store's allocator */
    uint64_t hot_rows_free;     /* hot rows returned by evictions */
    uint64_t hot_rows_capacity;
    uint64_t probe_hist[8]; /* count_probes != 0: keys that inspected 1, 2, .. 7, and 8 or more slot lines */
    uint64_t refused;       /* new keys turned away so far by find-or-insert (limit reached or out of rows); each got -1 */
    uint64_t occupied;      /* the device's own count of live + deleted slots, the figure its load-factor limit bounds
                               (equal to live + tombstones whenever no call is in flight) */
} ht_stats_t;

/* ------------------------------------------------------------------ host-only planning */

/* Identifier bits for m merged-in tables: k = ceil(log2(m+1))  (Sec. 3.2). */
int emb_tag_bits(int m);

/* Automated table merging (Sec. 3.2): logical tables with equal (dim, dtype) share one hash
 * table.  dims/dtypes [host, m entries] -> merged_of [host, m entries] = index of the merged
 * table, numbered by first appearance.  Returns the number of merged tables or a negative status. */
int emb_plan_merge(const int32_t* dims, const int32_t* dtypes, int m, int32_t* merged_of);

/* The table's probe sequence on the host, for checking Theorem 1: returns the index of the t-th
 * 8-slot line visited for `key` in a key structure of 2^capacity_log2 slots (capacity_log2 >= 3).
 * For t = 0 .. lines-1 the values are a permutation of the lines (odd stride, power-of-two size). */
uint64_t ht_probe_line(uint64_t key, int capacity_log2, uint64_t t);

const char* emb_status_string(int status);

/* ------------------------------------------------------------------ table life cycle (Sec. 3.1) */

/* Bytes of device memory the table needs for its counters and chunk directory. */
size_t emb_table_state_bytes(void);

/* Create a table.  state [dev]: emb_table_state_bytes() bytes, 256-byte aligned, zeroed here
 * (asynchronously on `stream`).  The table starts without key storage and without chunks. */
int emb_table_create(emb_table_t** out, const emb_table_desc_t* desc, void* state, size_t state_bytes,
                     void* stream);
int emb_table_destroy(emb_table_t* t);

/* Give an EMPTY table its key structure: slots [dev, 128-byte aligned, 2^capacity_log2 x 16 bytes],
 * 6 <= capacity_log2 <= 30.  A slot holds the 64-bit key and the 32-bit index of its embedding
 * row (plus 4 unused bytes).  All slots are marked empty here. */
int ht_set_key_storage(emb_table_t* t, void* slots, int capacity_log2, void* stream);

/* Register one more value chunk of 2^chunk_rows_log2 rows (Sec. 3.1: chunked embedding
 * structure; keep a spare chunk registered so inserts never wait for an allocation).
 * values [dev, 16-byte aligned]: rows x dim elements of the table dtype;
 * meta [dev, 16-byte aligned]: rows x 16 bytes of per-row auxiliary data (Adagrad accumulator f32,
 *   last-seen step u32, touch count u32, 4 reserved bytes);
 * free_list [dev]: rows x u32 scratch for the row free list.  values and free_list need no
 * initialisation; meta is zeroed by this call. */
int ht_add_chunk(emb_table_t* t, void* values, void* meta, uint32_t* free_list, void* stream);

/* Optional optimizer state for ht_apply_adam: fp32 first / second moment rows [2^chunk_rows_log2, dim]
 * for the oldest chunk that has none yet (chunks get their state in the order they were added).
 * Register it right after ht_add_chunk, before any key can be placed in the chunk; rows are zeroed
 * when a key is inserted.  Inserts zero the moments only while every chunk has its state. */
int ht_add_chunk_adam_state(emb_table_t* t, float* m, float* v, void* stream);

/* Host-side capacity planning (Sec. 3.1 "Capacity Expansion": expand when the load factor passes the limit,
 * doubling; keys only) from upper bounds of the device counters: the newest copy of the
 * counters that has reached the host (every find-or-insert / evict / rehash queues one, without
 * blocking; ht_stats fetches one synchronously) plus the n_max of every find-or-insert issued since.
 * n_incoming = keys still to be added (after a refusal: the number turned away).
 * *new_capacity_log2 = 0 if live + deleted + n_incoming slots stay within floor(max_load_factor * capacity),
 * else the size to rehash to: the same size when purging deleted slots is enough, otherwise doubled until
 * (live+n_incoming)/capacity is at most half the load-factor limit.  *chunks_needed = chunks to add so that
 * n_incoming rows fit. */
int ht_plan(emb_table_t* t, int64_t n_incoming, int* new_capacity_log2, int* chunks_needed);

/* Capacity expansion (Sec. 3.1): move every live (key,row) pair into new key storage of
 * 2^new_capacity_log2 slots (same layout and alignment as above), dropping deleted slots.
 * Embedding rows do not move.  The old array is no longer referenced once this call's work on
 * `stream` has finished.  Fails with EMB_ERR_NEED_REHASH if the live keys would exceed the
 * load-factor limit of the new structure. */
int ht_rehash(emb_table_t* t, void* new_slots, int new_capacity_log2, void* stream);

/* Copy the counters to *out [host].  Synchronises `stream`. */
int ht_stats(emb_table_t* t, ht_stats_t* out, void* stream);

/* ------------------------------------------------------------------ forward */

/* Eq. 8: key[e] = (field_tag[f] << (63 - tag_bits)) | x[e] for field_off[f] <= e < field_off[f+1].
 * x, key_out [dev, n];  field_off [dev, n_fields+1, int64, field_off[n_fields] == n];
 * field_tag [dev, n_fields] = 0-based logical table index.  0 <= tag_bits <= 16, n_fields <= 4096.
 * A raw ID that needs more than 63-tag_bits bits is counted in *err_count [dev, int64, zeroed by
 * this call] and wrapped into range. */
int emb_tag_keys(const uint64_t* x, const int64_t* field_off, const uint8_t* field_tag, int n_fields,
                 int64_t n, int tag_bits, uint64_t* key_out, int64_t* err_count, void* stream);

/* Stage-1 deduplication (Sec. 3.3).  key [dev, n] ->
 *   uniq [dev, n]: distinct keys ascending, first *n_unique entries valid;
 *   inverse [dev, n, int32, optional]: uniq[inverse[i]] == key[i].  The same mapping is delivered in
 *     sorted order by (perm, seg_of), which is what emb_expand_sorted, ht_gather_expand_sorted and
 *     grad_segment_reduce consume; the position-ordered array is a scatter of n random 4-byte writes
 *     (about a sixth of the call's time on long-sequence batches), so pass NULL when nothing reads it;
 *   counts [dev, n, int32, optional]: occurrences of uniq[u];
 *   perm [dev, n, int32, optional]: positions ordered by (key, position); the positions of
 *     uniq[u] are perm[seg_off[u] .. seg_off[u+1]);
 *   seg_off [dev, n+1, int32, optional];
 *   seg_of [dev, n, int32, optional]: seg_of[j] = inverse[perm[j]], the distinct-key index of the
 *     j-th position in sorted order (non-decreasing);
 *   n_unique [dev, int64].
 * workspace [dev, 256-byte aligned] of at least emb_dedup_workspace_bytes(n).  n < 2^31. */
size_t emb_dedup_workspace_bytes(int64_t n);
int emb_dedup(const uint64_t* key, int64_t n, uint64_t* uniq, int32_t* inverse, int32_t* counts,
              int32_t* perm, int32_t* seg_off, int32_t* seg_of, int64_t* n_unique, void* workspace,
              size_t workspace_bytes, void* stream);

/* Eq. 8 and Sec. 3.3 in one call: the results of emb_tag_keys followed by emb_dedup on the tagged keys, without
 * writing the tagged keys (unless key_out is given) and with fewer, narrower sort passes.
 * id_bits: declared width of the raw IDs, 1 <= id_bits <= 63 - tag_bits (e.g. 40 for IDs drawn from a 2^40
 *   space).  A raw ID that needs more bits is counted in *err_count and its excess bits are dropped - the
 *   same treatment emb_tag_keys gives IDs beyond Eq. 8's 63 - tag_bits bits.
 * key_out [dev, n, optional]: the tagged keys, as emb_tag_keys writes them.  All other outputs as emb_dedup.
 * The table identifier is a function of the position (IDs arrive field by field), so the sort carries 8-byte
 * records (ID, position) whenever id_bits + ceil(log2 n) <= 64 and n_fields <= 1024, and ceil((id_bits +
 * tag_bits) / 9) radix passes are planned on the host; otherwise the call runs emb_tag_keys and emb_dedup
 * internally.  workspace [dev, 256-byte aligned] of at least emb_tag_dedup_workspace_bytes(...) bytes. */
size_t emb_tag_dedup_workspace_bytes(int64_t n, int n_fields, int tag_bits, int id_bits);
int emb_tag_dedup(const uint64_t* x, const int64_t* field_off, const uint8_t* field_tag, int n_fields, int64_t n,
                  int tag_bits, int id_bits, uint64_t* key_out, uint64_t* uniq, int32_t* inverse, int32_t* counts,
                  int32_t* perm, int32_t* seg_off, int32_t* seg_of, int64_t* n_unique, int64_t* err_count,
                  void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or hand in a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  emb_dedup with the same arguments and results, minus the
 * workspace: its scratch is a fixed array in the library's device image (about 24.3 bytes per key of
 * EMB_DEDUP_NOALLOC_MAX_KEYS, i.e. 25 MB, held on every GPU the library runs on until the process ends).
 * Calls no hipMalloc / hipFree or any allocating routine.  n > EMB_DEDUP_NOALLOC_MAX_KEYS -> EMB_ERR_TOO_LARGE
 * (nothing launched).  The first call on a device resolves the array's address (hipGetSymbolAddress) with
 * that device current: make it outside stream capture.  Every call on a GPU shares that GPU's array: calls that
 * overlap on one GPU (different streams without ordering) race; calls ordered on one stream do not.  Nothing
 * in the scratch needs clearing between calls (every word that is read is written earlier in the same call). */
#define EMB_DEDUP_NOALLOC_MAX_KEYS (1 << 20)
int emb_dedup_noalloc(const uint64_t* key, int64_t n, uint64_t* uniq, int32_t* inverse, int32_t* counts,
                      int32_t* perm, int32_t* seg_off, int32_t* seg_of, int64_t* n_unique, void* stream);

/* Measuring aid, not a step of the paper's path: one launch of a bare access pattern over rows of 256 bytes
 * (16 lanes x 16 bytes per row, as in the row kernels), so that the rates reported for those kernels can be read
 * against what the memory system gives a kernel that only reads, only writes, or mixes the two.
 * src, dst [dev, 256-byte rows, 16-byte aligned]; idx [dev, int32, rows entries, each in [0, rows)] or null = the
 * rows in order; rows > 0, a multiple of 64.  Nothing is allocated; errors: EMB_ERR_INVALID_ARG, EMB_ERR_HIP.
 *   EMB_PROBE_READ              rows src[idx[r]] are read once and summed; dst (any 4 device bytes) is not written
 *   EMB_PROBE_WRITE             dst row idx[r] <- (float)r in all 64 elements          (dst: rows rows)
 *   EMB_PROBE_READ_STORE_4TH    as READ, and dst row q <- src[idx[4q]] + ... + src[idx[4q+3]], added in that order
 *                               elementwise in fp32, stored non-temporally             (dst: rows/4 rows)
 *   EMB_PROBE_READ_STORE_64TH   the same with 64 rows per sum                          (dst: rows/64 rows) */
enum { EMB_PROBE_READ = 0, EMB_PROBE_WRITE = 1, EMB_PROBE_READ_STORE_4TH = 2, EMB_PROBE_READ_STORE_64TH = 3 };
int emb_probe_memory(int pattern, const void* src, void* dst, const int32_t* idx, int64_t rows, void* stream);

/* Sec. 3.1 (real-time insertion; open addressing with cooperative probing; "Capacity Expansion"):
 * find each key; insert the absent ones (claim a never-used slot by compare-and-swap, allocate a row,
 * initialise the row from the key, acc = 0).  Every element counts one touch: freq += 1, last_seen = step.
 * key [dev], row_idx [dev, int32] <- row of each key (-1: see below),
 * inserted [dev, u8, optional] <- 1 for the element that created its entry.  Duplicate keys in
 * one call are allowed and share one row.
 * Capacity: new keys are admitted on the device while live + deleted slots stay within
 * floor(max_load_factor * capacity) and registered rows remain.  A key that is turned away gets -1, is counted
 * in ht_stats_t.refused and sets EMB_DEV_NEED_REHASH / EMB_DEV_OUT_OF_ROWS; nothing of it remains in the table
 * (a key that got a slot but no row leaves a deleted marker in that slot).  Returns EMB_OK when the host-side bounds (see ht_plan) prove that n_max
 * new keys fit, EMB_CHECK_STATUS when they do not (the caller then reads ht_stats, makes room with ht_rehash /
 * ht_add_chunk and calls ht_find_or_insert_retry), EMB_ERR_NO_STORAGE without key storage or chunks. */
int ht_find_or_insert(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, uint32_t step,
                      int32_t* row_idx, uint8_t* inserted, void* stream);

/* Second attempt after room was made: the same call restricted to the elements whose row_idx[i] is negative
 * on entry (the ones turned away); all others, their touch counts and their `inserted` flags are left as the
 * first call wrote them.  touch != 0: as ht_find_or_insert, touch == 0: as ht_find_or_insert_notouch. */
int ht_find_or_insert_retry(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, uint32_t step,
                            int32_t* row_idx, uint8_t* inserted, int touch, void* stream);

/* Clear the given EMB_DEV_* bits of the device status word (asynchronously on `stream`). */
int ht_clear_status(emb_table_t* t, uint32_t bits, void* stream);

/* Sec. 3.1 (hash lookup by cooperative probing, Theorem 1 for the probe sequence), read-only:
 * row_idx[i] = row of key[i], or -1 if absent (static tables fall back to a default embedding there; here the
 * caller decides: ht_gather turns -1 into a zero row). */
int ht_find(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, int32_t* row_idx,
            void* stream);

/* Sec. 3.1 "Table Lookup" (Eq. 7: the key structure yields the position of the row in the chunked embedding
 * structure): out[u,:] = values[row_idx[u],:] in the table dtype, row-major [n, dim]; row -1 reads as zeros. */
int ht_gather(emb_table_t* t, const int32_t* row_idx, const int64_t* n_dev, int64_t n_max, void* out,
              void* stream);

/* Sec. 3.3 (after the embeddings of the distinct IDs have come back, every position gets the row of its ID;
 * Fig. 6): out[i,:] = uniq_rows[inverse[i],:].  dtype: element type of both. */
int emb_expand(const void* uniq_rows, const int32_t* inverse, int64_t n, int dim, int dtype, void* out,
               void* stream);

/* The same result as emb_expand, computed in sorted order from emb_dedup's by-products:
 * out[perm[j],:] = uniq_rows[seg_of[j],:] for j in [0,n).  Every distinct row is read once (runs of
 * equal seg_of are adjacent) at the price of scattered, row-sized writes; on the long-sequence
 * workload this moves 12 % fewer bytes than indexing by `inverse`. */
int emb_expand_sorted(const void* uniq_rows, const int32_t* seg_of, const int32_t* perm, int64_t n, int dim,
                      int dtype, void* out, void* stream);

/* ------------------------------------------------------------------ backward */

/* Sec. 2 "Backward Update" and App. C "Gradient Accumulation" (gradients of one ID are aggregated before the
 * owner updates the row): reduced[u,:] = sum over positions i with inverse[i] == u of grad[i,:], fp32 accumulation,
 * fp32 output [*n_unique, dim].  grad [dev, n x dim] of grad_dtype, dim <= 256.  perm and seg_of as
 * written by emb_dedup for the same keys (the sum for u runs over grad[perm[j]] for the j with
 * seg_of[j] == u).  The order of additions is fixed, so results are reproducible run to run. */
size_t grad_segment_reduce_workspace_bytes(int64_t n, int dim);
int grad_segment_reduce(const void* grad, int grad_dtype, const int32_t* seg_of, const int32_t* perm, int64_t n,
                        int dim, float* reduced, void* workspace, size_t workspace_bytes, void* stream);

/* Sec. 2 "Backward Update", App. C (only the activated rows are updated; the benchmark fixes the sparse optimizer:
 * row-wise Adagrad with one fp32 accumulator per row).  On the listed rows only:
 *   acc += mean_j(g_j^2);  w_j -= lr * g_j / (sqrt(acc) + eps).
 * row_idx [dev]: distinct rows (as returned for deduplicated keys); -1 entries are skipped.
 * reduced [dev, n x dim, f32]. */
int ht_apply_adagrad(emb_table_t* t, const int32_t* row_idx, const float* reduced, const int64_t* n_dev,
                     int64_t n_max, float lr, float eps, void* stream);

/* Sparse (lazy) Adam on the listed rows only - the optimizer the paper trains with (Sec. 4.1):
 *   m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   w -= lr * sqrt(1-beta2^step) / (1-beta1^step) * m / (sqrt(v) + eps),   step >= 1 = optimizer step count.
 * Needs moment rows for every chunk (ht_add_chunk_adam_state), else EMB_ERR_NO_STORAGE.  row_idx as for
 * ht_apply_adagrad. */
int ht_apply_adam(emb_table_t* t, const int32_t* row_idx, const float* reduced, const int64_t* n_dev, int64_t n_max,
                  float lr, float beta1, float beta2, float eps, int64_t step, void* stream);

/* ------------------------------------------------------------------ fused form (no communication between lookup and expand) */

/* ht_gather followed by emb_expand_sorted without materialising the distinct rows:
 * out[perm[j],:] = values[row_idx[seg_of[j]],:] (zeros where the row index is -1).  Same result,
 * 2 x rowbytes x n_unique fewer bytes moved.  The unfused calls remain the form to use when the
 * distinct rows travel between devices (Sec. 3.3). */
int ht_gather_expand_sorted(emb_table_t* t, const int32_t* row_idx, const int32_t* seg_of, const int32_t* perm,
                            int64_t n, void* out, void* stream);

/* ------------------------------------------------------------------ pooling (Sec. 3.2: "performs pooling computations as needed") */

/* A bag is a run of consecutive positions (the ID list of one sample in one field); bag b covers
 * positions bag_off[b] .. bag_off[b+1]-1, bag_off [dev, int64, n_bags+1], bag_off[n_bags] == n.
 *
 * emb_pool_bags: pooled[b,:] = sum (mean != 0: mean) over the positions i of bag b of
 * uniq_rows[inverse[i],:], fp32 accumulation in a fixed order, fp32 output [n_bags, dim]; an empty bag
 * gives zeros.  It replaces emb_expand when the model consumes one vector per bag.
 *
 * grad_segment_reduce_pooled: the matching backward pass.  d_pooled [dev, n_bags x dim, f32] is the
 * gradient of the pooled output; position i receives d_pooled[bag(i),:] (divided by the bag length for
 * the mean) and these are summed per distinct key exactly like grad_segment_reduce does, into
 * reduced [*n_unique, dim].  seg_of / perm as written by emb_dedup.
 *
 * workspace [dev, 256-byte aligned] of at least emb_pool_workspace_bytes(n, n_bags, dim) for both. */
size_t emb_pool_workspace_bytes(int64_t n, int n_bags, int dim);
int emb_pool_bags(const void* uniq_rows, int dtype, const int32_t* inverse, const int64_t* bag_off, int n_bags,
                  int64_t n, int dim, int mean, float* pooled, void* workspace, size_t workspace_bytes, void* stream);
int grad_segment_reduce_pooled(const float* d_pooled, const int64_t* bag_off, int n_bags, const int32_t* seg_of,
                               const int32_t* perm, int64_t n, int dim, int mean, float* reduced, void* workspace,
                               size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ maintenance */

/* Sec. 3.1 (real-time deletion of entries; the embedding structure keeps timestamps as auxiliary data).
 * Delete every key that was not touched for `ttl` steps (rule active when ttl > 0) or that was
 * touched fewer than `min_freq` times and not within the last `grace` steps (active when
 * min_freq > 0).  Slots become deleted markers, rows return to the free list.
 * evicted_keys [dev, evicted_cap, optional]: the deleted keys in no particular order (at most
 * evicted_cap are stored);  n_evicted [dev, int64]: how many were deleted. */
int ht_evict(emb_table_t* t, uint32_t now, uint32_t ttl, uint32_t min_freq, uint32_t grace,
             uint64_t* evicted_keys, int64_t evicted_cap, int64_t* n_evicted, void* stream);

/* Dump the table in no particular order (for checks): up to `cap` entries of keys [dev],
 * values [dev, cap x dim, table dtype], acc, last_seen, freq [dev]; any of the last four may be
 * NULL.  *n [dev, int64] <- number of live entries. */
int ht_export(emb_table_t* t, uint64_t* keys, void* values, float* acc, uint32_t* last_seen, uint32_t* freq,
              int64_t cap, int64_t* n, void* stream);

/* Overwrite the contents of existing rows: values[row_idx[u],:] = values_in[u,:] (table dtype) and the
 * row's accumulator / last-seen step / touch count; any of the four sources may be NULL (left as is),
 * row index -1 is skipped.  Together with ht_find_or_insert this restores an ht_export dump
 * (App. C "Checkpoint Resuming": every device saves its own shard; a device of a resized job reads
 * the dump of rank r mod old_world and keeps the keys it owns). */
int ht_put(emb_table_t* t, const int32_t* row_idx, const void* values_in, const float* acc, const uint32_t* last_seen,
           const uint32_t* freq, int64_t n, void* stream);

/* ---- one record update per training step.
 * A row's 16-byte record (accumulator, last-seen step, touch count) is a random small access; memory
 * serves it as a read-modify-write, about as dear as reading the whole row.  A training step that
 * looks a key up and later updates it can pay this once instead of twice:
 *   ht_find_or_insert_notouch  = ht_find_or_insert, except that existing keys are not touched and a
 *     created row starts with last_seen = step and touch count 0;
 *   ht_apply_adagrad_touch     = ht_apply_adagrad, and every updated row also gets last_seen = step and
 *     touch count + 1, written together with the accumulator (row_idx must hold distinct rows).
 * After both calls on the distinct keys of a step the table is in the state that ht_find_or_insert +
 * ht_apply_adagrad leave.  Keys that are looked up but get no update keep their old record. */
int ht_find_or_insert_notouch(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, uint32_t step,
                              int32_t* row_idx, uint8_t* inserted, void* stream);
int ht_apply_adagrad_touch(emb_table_t* t, const int32_t* row_idx, const float* reduced, const int64_t* n_dev,
                           int64_t n_max, float lr, float eps, uint32_t step, void* stream);

/* Backward pass in one call for the case without communication between aggregation and update
 * (Sec. 2 "Backward Update"): grad_segment_reduce followed by ht_apply_adagrad (touch == 0) or
 * ht_apply_adagrad_touch (touch != 0), without materialising the reduced matrix.  grad [n, dim] is in
 * the table's dtype; seg_of / perm as for grad_segment_reduce; row_idx [n_unique] gives the row of
 * every segment (-1 = skip).  The segment sums and the update arithmetic are those of the two calls, so
 * the table ends up bit-identical.  workspace: grad_segment_reduce_workspace_bytes(n, dim) bytes.
 * What it saves is the reduced matrix (n_max x dim x 4 bytes of caller memory), not time: every completed
 * sum needs its row from memory before the next one can be parked, and with a few positions per distinct ID
 * that wait is exposed (about 1.5x the time of the two calls on long-sequence batches).
 * Not available for tables with a hot store (EMB_ERR_INVALID_ARG). */
int grad_reduce_apply_adagrad(emb_table_t* t, const void* grad, const int32_t* seg_of, const int32_t* perm, int64_t n,
                              const int32_t* row_idx, float lr, float eps, int touch, uint32_t step, void* workspace,
                              size_t workspace_bytes, void* stream);

/* ---- hot / cold rows (App. C "Mixed Precision Training"): a 16-bit table whose frequently used keys
 * keep an fp32 master row, so that many small updates of a hot row are not lost to 16-bit rounding,
 * while the bulk of the table stays at 2 bytes per element.
 *
 * ht_set_hot_storage attaches the hot store, once, to a table of dtype EMB_BF16: hot_values
 * [hot_rows, dim] fp32 (16-byte aligned) and hot_free [hot_rows] u32 scratch, both owned by the caller
 * for the table's lifetime.  With a hot store attached:
 *   ht_gather / ht_gather_expand_sorted deliver every row in the table dtype, a hot row as its master
 *     rounded to nearest even;
 *   ht_apply_adagrad updates a hot row's master in fp32 and a cold row in place as before (the 16-bit
 *     copy of a hot row is stale from then on and never read);
 *   ht_evict returns the hot rows of evicted keys to the hot store; ht_export dumps a hot row as its
 *     rounded master; ht_put refreshes the master of a hot row it overwrites;
 *   ht_apply_adam, like ht_apply_adagrad, updates a hot row's master in fp32. */
int ht_set_hot_storage(emb_table_t* t, float* hot_values, uint32_t* hot_free, int64_t hot_rows, void* stream);

/* Promote by access frequency: every row of row_idx [device; distinct rows, -1 skipped; count as for
 * ht_gather] that has been touched at least min_freq times and has no master yet gets one (a copy of
 * its current 16-bit values, which is exact), as long as the hot store has room; the rest stay cold.
 * *n_promoted [device, optional] receives the number promoted by this call.  Which rows win when the
 * store runs out is not specified.  EMB_ERR_NO_STORAGE without a hot store. */
int ht_promote(emb_table_t* t, const int32_t* row_idx, const int64_t* n_dev, int64_t n_max, uint32_t min_freq,
               int64_t* n_promoted, void* stream);

/* Demote by idle time (App. C: the hot set is partitioned dynamically, so it follows the access pattern both ways;
 * the criterion is this library's): every hot row whose key no find-or-insert has touched for `idle` steps
 * (now - last_seen >= idle, as in ht_evict) gives its master back to the hot store; its 16-bit row becomes the
 * master rounded to nearest even - the values lookups delivered for it anyway - and later updates round like any
 * cold row's.  *n_demoted [device, optional] receives the number demoted by this call.  Scans the key structure
 * (one pass over all slots).  EMB_ERR_NO_STORAGE without a hot store. */
int ht_demote(emb_table_t* t, uint32_t now, uint32_t idle, int64_t* n_demoted, void* stream);

/* Restore masters from a dump (App. C "Checkpoint Resuming" for a table with hot rows): for every u < n
 * whose row row_idx[u] [device; -1 skipped] has a master, the master becomes masters[u,:] [device, fp32,
 * row-major, 16-byte aligned], e.g. what ht_export_hot wrote; rows without a master are skipped (promote them
 * first: ht_promote with min_freq 0 gives every listed row a master).  The 16-bit row is left as it is (it is
 * stale while a master exists).  *n_written [device, optional] receives the number of masters written.
 * EMB_ERR_NO_STORAGE without a hot store. */
int ht_put_hot(emb_table_t* t, const int32_t* row_idx, const float* masters, int64_t n, int64_t* n_written, void* stream);

/* Unordered dump of the masters: keys[cap], values[cap, dim] fp32 (optional); *n [device] = number of
 * hot rows (may exceed cap; only the first cap are written). */
int ht_export_hot(emb_table_t* t, uint64_t* keys, float* values, int64_t cap, int64_t* n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MTGR_EMB_H */
