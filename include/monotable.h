/* monotable.h — C ABI of the MI355X-native collisionless embedding table.
 *
 * The operations are those of the `HashTable` of arxiv 2209.07663 (Monolith), section 2.1: a
 * key-value table for sparse parameters built on a cuckoo hashmap with two sub-tables T0/T1 and two
 * hash functions h0/h1 (an element lives in exactly one of T0[h0(x)], T1[h1(x)]; an insertion that
 * finds its cell occupied evicts the occupant, which is re-inserted in the other sub-table), with
 * the two memory-saving heuristics of the same section: IDs are filtered by their number of
 * occurrences before they are admitted, and IDs that stay inactive for a configured time expire.
 * Lookups and updates are separate operations (end of section 2.1).  Pooling, duplicate-ID
 * gradient reduction and row-wise Adagrad are the build's own problem statement around that table.
 *
 * Conventions
 *  - Every pointer named d_* is DEVICE memory owned by the caller; h_* is HOST memory owned by
 *    the caller.  The library never frees caller memory and keeps no pointer to it after a call
 *    returns (work already queued on the stream still reads/writes it: keep it alive until the
 *    stream has passed the call).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All hot calls only
 *    queue work on that stream and never synchronise.  Calls on one table must be issued in
 *    stream order on one stream; two calls on the same table that overlap race.
 *  - Return value: MONO_OK or a negative error; argument and launch errors only.  Data-dependent
 *    events (a failed eviction chain, a full table) are counted on the device and read with
 *    mono_table_stats.
 *  - Key -1 (all ones) is reserved as padding: it resolves to row -1 and is never counted or
 *    stored.  Every other int64 bit pattern is a legal key.
 *  - `step` / `now` are the caller's training-step counter: non-decreasing from call to call and
 *    below 2^24.
 *  - The step and a per-call tag of the table travel to the kernels as launch arguments, and the
 *    export / import / migrate / stats calls copy to the host and wait: a call recorded into a HIP
 *    graph would replay stale values.  Do not capture these calls; issue them on a live stream.
 *  - A table belongs to the device that was current when it was created; make that device current
 *    for every later call on it.
 */
#ifndef MONOTABLE_H_
#define MONOTABLE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mono_table mono_table; /* opaque; one table = one embedding dimension */

enum { MONO_OK = 0, MONO_EINVAL = -1, MONO_ENOMEM = -2, MONO_EHIP = -3, MONO_ELIMIT = -4 };
enum { MONO_ROWS_FP32 = 0, MONO_ROWS_BF16 = 1 }; /* `flags`: storage type of the embedding rows */

typedef struct mono_stats {
  uint64_t capacity;        /* slots = rows */
  uint64_t size;            /* keys currently stored (stash included) */
  uint64_t n_admitted;      /* keys admitted since creation */
  uint64_t n_expired;       /* keys removed by expire_sweep since creation */
  uint64_t n_insert_failed; /* eviction chains that hit the kick bound (element went to the stash) */
  uint64_t n_lost;          /* elements dropped because the stash was full too, or updates skipped because the
                               library's own bound on the rows in use was wrong (must stay 0) */
  uint64_t n_full;          /* admissible keys refused because their call would have passed the fill limit (see capacity) */
  uint64_t stash_size;      /* elements currently in the stash */
  uint64_t max_chain;       /* longest eviction chain seen */
} mono_stats;

/* Bytes of device memory a table needs (table proper + per-call workspace for batches of at most
 * max_ids IDs in at most max_bags bags).  0 on invalid arguments. */
size_t mono_table_bytes(uint64_t capacity, uint32_t dim, uint32_t flags, uint64_t max_ids, uint64_t max_bags);

/* Creates a table (section 2.1: cuckoo hashmap + occurrence filter + expiry).
 *   capacity        total slots = embedding rows; power of two in [16, 2^30]; each sub-table has half.
 *                   At most capacity - capacity/32 keys are stored at a time: beyond that load the
 *                   eviction chains of section 2.1 become long enough to fail.  A lookup_or_insert (or
 *                   import) call whose new keys would take the table past that limit places NONE of its
 *                   new keys (row -1, each counted in n_full; which keys are refused thus never depends
 *                   on an order); they are admitted by a later call once keys have expired or the table
 *                   has grown (their counters stay at or above the threshold)
 *   dim             embedding dimension; a multiple of 4 up to 256, or 512, 768 or 1024 (section 3.2.2
 *                   sizes its synchronisation example with 1024 fp32 elements = 4 KB per row)
 *   seed            fixes h0, h1, the counter hash and the initial value of every row
 *   freq_threshold  a key is admitted once its occurrence counter reaches it; 0 and 1 admit on
 *                   first sight; at most 255
 *   expire_steps    a key unseen for this many steps is removed by mono_expire_sweep; 0 = never
 *   flags           MONO_ROWS_FP32 or MONO_ROWS_BF16
 *   max_ids/max_bags largest batch any later call will pass (1 <= max_ids <= 2^28, 1 <= max_bags <= max_ids + 1)
 *   d_arena         NULL: the library allocates (and frees in destroy) its own device memory;
 *                   else caller-owned device memory of arena_bytes >= mono_table_bytes(...),
 *                   256-byte aligned, which must outlive the table
 * Initialisation is queued on `stream`.  Errors: MONO_EINVAL (bad argument, arena too small),
 * MONO_ENOMEM (allocation failed), MONO_EHIP (a HIP call failed). */
int mono_table_create(mono_table** out, uint64_t capacity, uint32_t dim, uint64_t seed, uint32_t freq_threshold,
                      uint32_t expire_steps, uint32_t flags, uint64_t max_ids, uint64_t max_bags, void* d_arena,
                      size_t arena_bytes, void* stream);

/* The same with the occurrence filter spelled out (section 2.1 names two filters: a threshold on
 * occurrences and a probabilistic one that saves memory; here both are one array of counters):
 *   filter_hashes  counters per key, 1..4.  Every missed occurrence of a key bumps all of them and the
 *                  key's count is their minimum (a counting filter with several hashes: it can
 *                  over-count when keys share counters, never under-count).  1 = mono_table_create.
 *   filter_log2    log2 of the number of counters (4..34), or 0 for 4 * capacity (mono_table_create).
 * mono_table_bytes_ex is the matching size query; mono_filter_export / _import cover 2^filter_log2 words. */
size_t mono_table_bytes_ex(uint64_t capacity, uint32_t dim, uint32_t flags, uint64_t max_ids, uint64_t max_bags,
                           uint32_t filter_log2);
int mono_table_create_ex(mono_table** out, uint64_t capacity, uint32_t dim, uint64_t seed, uint32_t freq_threshold,
                         uint32_t expire_steps, uint32_t flags, uint64_t max_ids, uint64_t max_bags,
                         uint32_t filter_hashes, uint32_t filter_log2, void* d_arena, size_t arena_bytes, void* stream);

/* Frees the table after waiting for the stream of the latest call that queued work for it (the calls of a
 * table go to one stream in order).  The caller's arena, if any, is not freed. */
int mono_table_destroy(mono_table* t);

/* Batched lookup-or-insert (section 2.1: lookup in T0[h0(x)] / T1[h1(x)]; insertion with eviction
 * chain; admission gated by the occurrence filter; keys are time-stamped for expiry).
 * Batch semantics: hits and misses are judged against the table before the call; every miss
 * occurrence is counted; then every distinct missing key whose counter reached freq_threshold is
 * admitted with its initial row, accumulator 0 and last_seen = step; hit keys get last_seen = step.
 *   d_keys[n]      int64 keys (device)
 *   d_rows_out[n]  receives the embedding row index of each occurrence, or -1 if its key is not
 *                  in the table (not admitted, padding, or no room).  Row indices stay valid
 *                  until the key expires.
 * Errors: MONO_EINVAL if n > max_ids, step >= 2^24 or step went backwards. */
int mono_lookup_or_insert(mono_table* t, const int64_t* d_keys, uint64_t n, uint32_t step, int32_t* d_rows_out,
                          void* stream);

/* Embedding gather with per-bag sum pooling: d_out[b, :] = sum of the rows d_rows[i] >= 0 for
 * i in [d_offsets[b], d_offsets[b+1]).  d_offsets[n_bags + 1] is int64, non-decreasing, starts at
 * 0 and ends at n.  d_out[n_bags * dim] is fp32 whatever the storage type; empty bags give zeros.
 * Errors: MONO_EINVAL if n > max_ids or n_bags > max_bags. */
int mono_gather_pool(mono_table* t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets, uint64_t n_bags,
                     float* d_out, void* stream);

/* The embedding of the quotient-remainder decomposition (section 3.1: the hashing baseline the paper
 * compares the collisionless table with; an ID of a space of 2^(2m) values is split into ID_r = ID mod 2^m
 * and ID_q = ID div 2^m, and its embedding is E_r[ID_r] + E_q[ID_q] from two dense tables of 2^m rows each,
 * 2^(m+1) rows instead of 2^(2m); the paper uses m = 24), gathered and sum-pooled per bag exactly like
 * mono_gather_pool: d_out[b, :] = sum over i in [d_offsets[b], d_offsets[b+1]) of E_r[..] + E_q[..].
 * No table object, no hashing, no lookup: the no-hash yardstick of the pooling kernel.
 *   d_table_r, d_table_q  [2^log2_rows * dim] each, fp32 or bf16 (flags), row-major, device, caller-owned
 *   log2_rows             m, 1..30;  dim as in mono_table_create
 *   d_ids[n]              int64; an ID outside [0, 2^(2m)) (e.g. the padding key -1) contributes zero
 * d_out[n_bags * dim] is fp32.  Errors: MONO_EINVAL on a bad argument. */
int mono_qr_gather_pool(const void* d_table_r, const void* d_table_q, uint32_t log2_rows, uint32_t dim, uint32_t flags,
                        const int64_t* d_ids, uint64_t n, const int64_t* d_offsets, uint64_t n_bags, float* d_out,
                        void* stream);

/* Sparse update (section 2: the parameter side applies the gradients the workers computed):
 * the pooled gradient d_grad[n_bags * dim] (fp32) of bag b is the gradient of each of its
 * occurrences; gradients of occurrences of the same row are summed, then row-wise Adagrad is
 * applied once per distinct row: acc += mean_j g_j^2; w_j -= lr * g_j / (sqrt(acc) + eps).
 * Occurrences with row -1 are dropped.  d_rows / d_offsets as in mono_gather_pool. */
int mono_apply_grad_adagrad(mono_table* t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets,
                            uint64_t n_bags, const float* d_grad, float lr, float eps, void* stream);

/* mono_apply_grad_adagrad for callers that must not allocate device memory and cannot bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * same result as mono_apply_grad_adagrad, but the per-call workspace (bag indices, the two buffers of
 * sorted (row, bag) pairs, radix histograms, partial sums) is a fixed array inside the library instead of
 * the table's arena: about 13 MB of device memory per GPU the library runs on, held until the process
 * ends.  The call allocates nothing (no hipMalloc / hipFree, no event creation) and never synchronises.
 *   limit   n <= mono_noalloc_max_ids() (262144) IDs per call, any dim the table can have; a larger batch
 *           is refused with MONO_ELIMIT and nothing is done (split the batch by whole bags, or use
 *           mono_apply_grad_adagrad)
 *   sharing every call on one GPU uses the same array, whatever the table: two such calls that overlap on
 *           one GPU (different streams, different threads) race; issue them in order on one stream.
 *           Nothing in the array needs clearing between calls.
 * The table's device must be the current device. */
int mono_apply_grad_adagrad_noalloc(mono_table* t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets,
                                    uint64_t n_bags, const float* d_grad, float lr, float eps, void* stream);
uint64_t mono_noalloc_max_ids(void);

/* Expiry (section 2.1, second heuristic): removes every key with now - last_seen >= expire_steps
 * (nothing if expire_steps == 0) and frees its row.
 *   d_n_expired     nullable; receives the number of keys removed by this call
 *   d_expired_keys  nullable; receives up to max_expired of the removed keys, in no particular order */
int mono_expire_sweep(mono_table* t, uint32_t now, uint64_t* d_n_expired, int64_t* d_expired_keys,
                      uint64_t max_expired, void* stream);

/* ---- maintenance: incremental synchronisation (not part of the timed step; synchronises `stream`) ---- */

/* Incremental parameter synchronisation (section 2.2.3: the training side keeps the set of touched
 * keys, the IDs whose embeddings were trained since the last synchronisation, and pushes only
 * those).  A key is touched once mono_apply_grad_adagrad has updated its row; a key that expires
 * before the next synchronisation is not reported.  Writes the touched keys in no particular order:
 *   d_keys[max_n], d_row[max_n] (row index), d_values[max_n * dim] (rows widened to fp32),
 *   d_acc[max_n]; any of them may be NULL (d_values / d_acc need d_row).
 * *h_n receives the number of touched keys.  If it is at most max_n the set is now empty (a new
 * window starts); otherwise nothing was taken and the call can be repeated with larger buffers.
 * Marking a row costs the update no extra memory access, and starting a window clears nothing. */
int mono_export_touched(mono_table* t, int64_t* d_keys, int32_t* d_row, float* d_values, float* d_acc, uint64_t max_n,
                        uint64_t* h_n, void* stream);

/* ---- maintenance: snapshot / restore, rehash / grow (not part of the timed step) ---- */

/* Restore (section 2.3: a parameter server recovers from its latest snapshot).  A snapshot is what
 * mono_table_export and mono_filter_export return; this call places n records (key, row values,
 * accumulator, last-seen step) into the table: each gets a free row, is inserted by the eviction-chain
 * insertion of section 2.1 without consulting the occurrence filter, and is not marked touched.
 * On a table that never expires keys (expire_steps == 0) the occurrence counters of a placed key are
 * raised to freq_threshold if they are below it (there a stored key has been seen at least that often
 * at all times), so records may be restored without their counters; counters that age are left alone.
 *   d_keys[n], d_values[n * dim] (fp32; rounded to nearest-even for bf16 rows), d_acc[n], d_last_seen[n]
 *   n <= max_ids per call (call repeatedly for more)
 *   h_refused  nullable; receives the number of records not placed: key already stored, key -1,
 *              second record of a key within the call, or every record of a call that would take the
 *              table past its fill limit.  Non-NULL synchronises `stream`.
 * Later lookups need step >= the largest restored last-seen step for expiry to be meaningful. */
int mono_table_import(mono_table* t, const int64_t* d_keys, const float* d_values, const float* d_acc,
                      const uint32_t* d_last_seen, uint64_t n, uint64_t* h_refused, void* stream);

/* Writes occurrence counters [first, first + count) from canonical words (see mono_filter_export), as
 * when the counters of a snapshot are restored (section 2.3).  On a table that never expires keys a
 * stored key stays counted: each of its counters among the written ones that would end up below
 * freq_threshold is raised to it, as mono_table_import does for a record that comes without its
 * counters; so the two calls can be made in either order, and no words, not even all zeros, can hide a
 * stored key from a later lookup (that costs one scan of the table, 16 bytes per slot, after the words
 * are written).  On a table with expiry the words are stored as given. */
int mono_filter_import(mono_table* t, const uint32_t* d_words, uint64_t first, uint64_t count, void* stream);

/* Rehash / grow (section 2.1: a rehash answers an insertion that runs into a cycle; the table is
 * meant to be adjusted elastically).  `dst` is a table just created with the same dim, flags, seed,
 * freq_threshold, expire_steps and filter_hashes as `src`, a capacity >= src's with the number of
 * counters grown by the same factor, and not yet used.  Every key of
 * src (its overflow stash included) is inserted into dst under the hash functions h0 / h1 of rehash
 * `generation` (0 = the functions a new table starts with; any other value gives fresh ones); rows
 * keep their indices, values, accumulators, last-seen steps and touched marks; the free-row stack
 * and the life-time counters carry over; an occurrence counter of a grown table starts with the
 * value of the counter its keys shared before, so no count is lost.  src is left unchanged and can
 * be destroyed afterwards.  Synchronises `stream` once (to read src's counters).
 * A caller rehashes when mono_table_stats reports stash_size > 0 or a load factor it finds too high.
 * Errors: MONO_EINVAL if dst does not match src or has been used (nothing was done); after
 * MONO_EHIP the contents of dst are undefined and it can only be destroyed. */
int mono_table_migrate(mono_table* dst, mono_table* src, uint32_t generation, void* stream);

/* ---- observability / test surface (not part of the timed path; these synchronise `stream`) ---- */

int mono_table_stats(mono_table* t, mono_stats* h_out, void* stream);

/* Dumps up to max_n stored keys in no particular order.  Any of the d_* outputs may be NULL.
 *   d_keys[max_n], d_row[max_n] (row index), d_last_seen[max_n],
 *   d_slot[max_n]: global slot = sub-table * capacity/2 + bucket * 8 + lane, or -2 for the stash,
 *   d_values[max_n * dim]: the rows widened to fp32, d_acc[max_n]: Adagrad accumulators.
 * *h_n receives the number of keys stored (which may exceed max_n; only max_n are written). */
int mono_table_export(mono_table* t, int64_t* d_keys, int32_t* d_row, uint32_t* d_last_seen, int64_t* d_slot,
                      float* d_values, float* d_acc, uint64_t max_n, uint64_t* h_n, void* stream);

/* Occurrence counters [first, first + count) in canonical form (step & 0xFFFFFF) << 8 | min(count, 255).
 * There are 4 * capacity counters unless mono_table_create_ex said otherwise. */
int mono_filter_export(mono_table* t, uint32_t* d_words, uint64_t first, uint64_t count, void* stream);

/* Benchmark instrumentation.  While enabled, every kernel launched for this table is bracketed by
 * two HIP events on its stream (this costs a little, so throughput is measured with it off).
 * mono_profile_read synchronises the device, then reports, for each kernel launched since the last
 * read, its name (static string), the sum of its durations in milliseconds and its launch count;
 * at most max_kernels entries are written, *h_n receives how many. */
int mono_profile_enable(mono_table* t, int on);
int mono_profile_read(mono_table* t, const char** h_names, double* h_ms, uint64_t* h_launches, uint32_t max_kernels,
                      uint32_t* h_n);

/* Static description of an error code. */
const char* mono_strerror(int err);

#ifdef __cplusplus
}
#endif
#endif /* MONOTABLE_H_ */
