// Host-side launchers of the table's kernels (internal to the library).
#pragma once

#include "common.h"
#include "profile.h"

namespace mono {

// Per-call scratch for the update path, carved out of the table's arena.
struct UpdateWorkspace {
  uint32_t* unit_bag;   // [max_ids]: first [sort_units] words: the bag that holds each sort unit's first occurrence
                        // (a restore call borrows the whole array for its per-record results)
  uint2* pair_a;        // [max_ids] (row, bag) pairs, ping
  uint2* pair_b;        // [max_ids] pong
  uint32_t* hist;       // [sort_hist_words(max_ids)]: per-unit digit histograms (bin-major), then the bin totals
  float* part;          // [2 * tiles * dim] partial gradient sums of runs that cross tile borders
  uint32_t* part_row;   // [2 * tiles] row (+ head flag) of each partial, kNoRow if unused
};

// The sort comes in two shapes, chosen per call by the host from its bound on the rows in use:
//   narrow  digits of at most 8 bits, blocks of 256 threads that own 2048 elements: three passes up to 2^24 rows
//   wide    digits of at most 9 bits, blocks of 512 threads that own 4096 elements (so that a block's share of a
//           bin still leaves as pieces of eight elements): three passes up to 2^27 rows, where narrow needs four.
//           A wide pass takes a quarter longer than a narrow one (measured: 56 us against 45 us on 6.8 M pairs),
//           so wide is taken only where it saves a pass: 1.33 -> 1.30 ms per step on the streaming workload
//           (25 M rows in use), 5.78 -> 5.70 ms on the 26 M-ID workload.
struct SortShape {
  uint32_t max_bits, block, items;
};
constexpr SortShape kSortNarrow = {8, 256, 2048};
constexpr SortShape kSortWide = {9, 512, 4096};
constexpr uint32_t kSortNarrowMaxRows = 1u << 24;  // beyond this many rows in use the wide shape saves a pass
inline SortShape sort_shape_for(uint32_t hwm_bound) { return hwm_bound > kSortNarrowMaxRows ? kSortWide : kSortNarrow; }
constexpr int kPairsPerLane = 16;                  // sorted pairs per lane of a lane group in seg_reduce
constexpr uint32_t kReduceTile = 256 * kPairsPerLane;  // sorted pairs reduced by one block

#ifndef MONO_NOALLOC_MAX_IDS
#define MONO_NOALLOC_MAX_IDS (1ull << 18)
#endif

inline uint64_t sort_units(uint64_t n, uint32_t items) { return (n + items - 1) / items; }
// words of the histogram workspace for batches of at most n elements: one histogram per unit, then the bin
// totals, for whichever shape needs more
inline uint64_t sort_hist_words(uint64_t n) {
  const uint64_t narrow = (1ull << kSortNarrow.max_bits) * (sort_units(n, kSortNarrow.items) + 1);
  const uint64_t wide = (1ull << kSortWide.max_bits) * (sort_units(n, kSortWide.items) + 1);
  return narrow > wide ? narrow : wide;
}
inline uint64_t reduce_tiles(uint64_t n) { return (n + 255) / 256; }  // most tiles a batch can need (one pair per lane)

// How many bits of the row index are sorted, in how many passes (computed alike on host and device).
struct SortPlan {
  uint32_t hwm, bits, passes, per;
  __host__ __device__ uint32_t shift(uint32_t p) const { return p * per; }
  __host__ __device__ uint32_t width(uint32_t p) const { return bits - p * per < per ? bits - p * per : per; }
};
__host__ __device__ inline SortPlan make_sort_plan(uint32_t hwm, uint32_t max_bits) {
  SortPlan s;
  s.hwm = hwm;
  s.bits = 1;
  const uint32_t top = hwm > 0 ? hwm - 1 : 0;  // sorted keys are row indices below hwm (hwm itself marks "dropped")
  while (s.bits < 32 && (top >> s.bits) != 0) ++s.bits;
  s.passes = (s.bits + max_bits - 1) / max_bits;
  s.per = (s.bits + s.passes - 1) / s.passes;
  return s;
}

// What a restore call supplies per record instead of the initial state of a fresh key
// (values == nullptr: an ordinary lookup_or_insert).
struct RestoreSource {
  const float* values;   // [n * dim] fp32, rounded to the storage type on the way in
  const float* acc;      // [n] accumulators
  const uint32_t* seen;  // [n] last-seen steps
};

hipError_t launch_lookup_or_insert(const TableView& t, const int64_t* d_keys, uint64_t n, uint32_t step, uint32_t epoch,
                                   int32_t* d_rows_out, const RestoreSource& src, hipStream_t stream, Profiler* prof);

// Re-inserts every element of src into dst (dst empty, same dim and storage type, capacity >= src's),
// carries the free-row stack over and spreads the occurrence counters; rows are copied by the caller.
hipError_t launch_migrate(const TableView& dst, const TableView& src, int32_t src_free_n, hipStream_t stream);

hipError_t launch_gather_pool(const TableView& t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets,
                              uint64_t n_bags, float* d_out, hipStream_t stream, Profiler* prof);

// Pooled embeddings of the quotient-remainder decomposition: two dense tables of 2^log2_rows rows each.
hipError_t launch_qr_gather_pool(const void* d_rem, const void* d_quot, uint32_t log2_rows, uint32_t dim, bool bf16,
                                 const int64_t* d_ids, uint64_t n, const int64_t* d_offsets, uint64_t n_bags,
                                 float* d_out, hipStream_t stream);

// hwm_bound: a number the table's high-water mark of rows cannot exceed when the call runs (the capacity, or
// less if the host knows better): it decides how many sort passes are launched.
hipError_t launch_apply_grad_adagrad(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                                     const int64_t* d_offsets, uint64_t n_bags, const float* d_grad, float lr, float eps,
                                     uint32_t hwm_bound, hipStream_t stream, Profiler* prof);

// Stable LSD radix sort of the (row, bag) pairs of a batch; the result is in pair_b if the plan for
// the device's high-water mark (digits of at most *max_bits bits) has an odd number of passes, else in pair_a.
// Returns how many passes were queued (those the plan for hwm_bound needs) and the widest digit of the shape used.
hipError_t launch_sort_pairs(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                             const int64_t* d_offsets, uint64_t n_bags, uint32_t hwm_bound, uint32_t* launched,
                             uint32_t* max_bits, hipStream_t stream, Profiler* prof);

hipError_t launch_expire_sweep(const TableView& t, uint32_t now, uint64_t* d_n_expired, int64_t* d_expired_keys,
                               uint64_t max_expired, hipStream_t stream, Profiler* prof);

hipError_t launch_export(const TableView& t, int64_t* d_keys, int32_t* d_row, uint32_t* d_last_seen, int64_t* d_slot,
                         uint64_t max_n, bool touched_only, hipStream_t stream);
hipError_t launch_export_values(const TableView& t, const int32_t* d_row, uint64_t n, float* d_values, float* d_acc,
                                hipStream_t stream);
hipError_t launch_filter_export(const TableView& t, uint32_t* d_words, uint64_t first, uint64_t count,
                                hipStream_t stream);
hipError_t launch_filter_import(const TableView& t, const uint32_t* d_words, uint64_t first, uint64_t count,
                                hipStream_t stream);
hipError_t launch_table_init(const TableView& t, uint64_t dset_size, hipStream_t stream);

}  // namespace mono
