// Host-side launchers of the table's kernels (internal to the library).
#pragma once

#include "common.h"
#include "profile.h"

namespace mono {

// Per-call scratch for the update path, carved out of the table's arena.
struct UpdateWorkspace {
  uint32_t* key_a;      // [max_ids] sort keys (row index, or `capacity` for dropped occurrences)
  uint32_t* key_b;      // [max_ids]
  uint32_t* val_a;      // [max_ids] bag of each occurrence
  uint32_t* val_b;      // [max_ids]
  uint32_t* hist;       // [kSortMaxBins * sort_units(max_ids)]
  float* part;          // [2 * n_chunks(max_ids) * dim] partial gradient sums of runs that cross chunks
  uint32_t* part_row;   // [2 * n_chunks(max_ids)] row of each partial, kNoRow if unused
};

constexpr uint32_t kSortMaxBits = 10;              // widest radix digit
constexpr uint32_t kSortMaxBins = 1u << kSortMaxBits;
constexpr uint32_t kSortItemsPerWave = 2048;       // consecutive elements ranked by one wave
constexpr uint32_t kChunk = 128;                   // sorted occurrences reduced by one lane group

inline uint64_t sort_units(uint64_t n) { return (n + kSortItemsPerWave - 1) / kSortItemsPerWave; }
inline uint64_t reduce_chunks(uint64_t n) { return (n + kChunk - 1) / kChunk; }

hipError_t launch_lookup_or_insert(const TableView& t, const int64_t* d_keys, uint64_t n, uint32_t step, uint32_t epoch,
                                   int32_t* d_rows_out, hipStream_t stream, Profiler* prof);

hipError_t launch_gather_pool(const TableView& t, const int32_t* d_rows, const int64_t* d_offsets, uint64_t n_bags,
                              float* d_out, hipStream_t stream, Profiler* prof);

hipError_t launch_apply_grad_adagrad(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                                     const int64_t* d_offsets, uint64_t n_bags, const float* d_grad, float lr, float eps,
                                     hipStream_t stream, Profiler* prof);

// Stable LSD radix sort of (key, value) pairs on the low `bits` bits of the key.  Input in
// (key_a, val_a) unless `keys_in` is given (first pass then reads keys from there, transformed by
// min(key, clamp) on unsigned values); returns which buffer pair holds the result (0 = a, 1 = b).
hipError_t launch_sort_pairs(const UpdateWorkspace& ws, const uint32_t* keys_in, uint32_t clamp, uint64_t n,
                             uint32_t bits, int* result_in_b, hipStream_t stream, Profiler* prof);

hipError_t launch_expire_sweep(const TableView& t, uint32_t now, uint64_t* d_n_expired, int64_t* d_expired_keys,
                               uint64_t max_expired, hipStream_t stream, Profiler* prof);

hipError_t launch_export(const TableView& t, int64_t* d_keys, int32_t* d_row, uint32_t* d_last_seen, int64_t* d_slot,
                         uint64_t max_n, hipStream_t stream);
hipError_t launch_export_values(const TableView& t, const int32_t* d_row, uint64_t n, float* d_values, float* d_acc,
                                hipStream_t stream);
hipError_t launch_filter_export(const TableView& t, uint32_t* d_words, uint64_t first, uint64_t count,
                                hipStream_t stream);
hipError_t launch_table_init(const TableView& t, uint64_t dset_size, hipStream_t stream);

}  // namespace mono
