// Device-side layout and helpers shared by the kernels of the collisionless table (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mono {

constexpr uint64_t kEmptyKey = ~0ull;       // reserved key: padding / free slot
constexpr uint32_t kNoRow = 0xFFFFFFFFu;    // slot has no published row: free, or being written
constexpr int kBucket = 8;                  // slots per bucket
constexpr int kMaxKicks = 512;              // bound of an eviction chain
constexpr int kReserveShift = 5;            // capacity >> 5 rows are never handed out: see rows_on_offer()
constexpr uint32_t kStashCap = 4096;        // homeless elements kept aside after a failed chain
constexpr int32_t kRowAbsent = -1;          // rows_out: key not in the table
constexpr int32_t kRowMiss = -2;            // rows_out, between the kernels of one call: missed, undecided
// rows_out values <= -3 between the kernels of one call: duplicate of an admitted key, encodes the
// position of that key in the per-call dedup set

// One bucket = one 128-byte line (the unit the memory system fetches): eight keys, then eight
// `meta` words = last-seen step << 32 | row index.  A probe costs one line per bucket; the row and
// the stamp of a hit sit in the line already fetched.  meta == kNoMeta: slot free or being written.
struct __attribute__((aligned(128))) Bucket {
  uint64_t key[kBucket];
  unsigned long long meta[kBucket];
};
static_assert(sizeof(Bucket) == 128, "bucket must be one 128-byte line");
constexpr unsigned long long kNoMeta = ~0ull;
__host__ __device__ inline uint32_t meta_row(unsigned long long m) { return (uint32_t)m; }
__host__ __device__ inline uint32_t meta_seen(unsigned long long m) { return (uint32_t)(m >> 32); }
__host__ __device__ inline unsigned long long make_meta(uint32_t row, uint32_t seen) {
  return ((unsigned long long)seen << 32) | row;
}
constexpr int kWinLists = 64;               // sub-lists of elected occurrences (spreads the append counter)
constexpr int kWinStride = 32;              // u32 words between two sub-list counters (one 128-byte line each)

constexpr int kSweepRemoved = 0;            // Control::scratch slot: keys removed so far by the running sweep
constexpr int kExportCount = 1;             // Control::scratch slot: elements found by the running export
constexpr int kValidPairs = 2;              // Control::scratch slot: (row, bag) pairs kept by the sort
constexpr int kRefusedRecords = 3;          // Control::scratch slot: records refused by the running restore call

struct StashEntry {
  uint64_t key;
  uint32_t row;
  uint32_t seen;
};

// Per-row optimizer state.  `touch` is the number of the synchronisation window in which the row
// was last trained (paper section 2.2.3: touched keys); it shares the accumulator's 8-byte word so
// that marking a row costs no memory access of its own.
struct alignas(8) RowState {
  float acc;
  uint32_t touch;
};

// An elected occurrence: its key travels with it, so that the insertion reads the list and nothing else.
struct alignas(16) Winner {
  uint64_t key;
  uint32_t occ;   // occurrence index in the batch
  uint32_t pos;   // position of the key in the per-call dedup set
};

// Counters that live on the device for the whole life of the table.
struct Control {
  int32_t free_n;            // rows on the free stack
  uint32_t stash_n;          // elements pushed to the stash (may exceed kStashCap: then some were lost)
  uint32_t hwm;              // every row index ever handed out is below this high-water mark
  uint32_t pad_;
  unsigned long long n_admitted, n_expired, n_insert_failed, n_lost, n_full, max_chain;
  unsigned long long scratch[8];  // per-call scalars, indexed by the constants above
};

// Everything a kernel needs to know about a table; passed by value.
struct TableView {
  Bucket* buckets;           // [2 * n_buckets]: T0 then T1
  unsigned long long* filter;  // [n_filter] occurrence counters: step << 32 | count
  void* rows;                // [capacity * dim] fp32 or bf16
  RowState* state;           // [capacity] Adagrad accumulator + touched mark
  uint32_t* free_rows;       // [capacity] stack of free row indices
  Control* ctl;
  StashEntry* stash;         // [kStashCap]
  unsigned long long* dset;  // [dset_size] per-call dedup set: epoch << 32 | occurrence index
  int32_t* dset_row;         // [dset_size] row of the key that owns the dedup-set position
  Winner* win_list;          // [kWinLists * win_cap] elected occurrences
  uint32_t* win_cnt;         // [kWinLists * kWinStride] fill of each sub-list (zero between calls)
  uint64_t win_cap;
  unsigned long long* occupied;  // [capacity / 512, at least 1] one bit per bucket: set when a slot of the bucket is
                                 // taken; a clear bit proves the bucket empty (the sweep skips it), a set bit
                                 // proves nothing (the sweep clears it when it finds the bucket empty)
  uint32_t* sweep_list;      // [kWinLists * sweep_cap] slots found expired by the running sweep
  uint32_t* sweep_cnt;       // [kWinLists * kWinStride]
  uint64_t sweep_cap;
  uint64_t capacity;
  uint64_t n_buckets;        // per sub-table
  uint64_t n_filter;
  uint64_t dset_mask;
  uint64_t s_h0, s_h1, s_init, s_dedup;
  uint64_t s_filter[4];      // one salt per counter hash
  uint32_t bucket_shift;     // 64 - log2(n_buckets)   (64 means: single bucket)
  uint32_t filter_shift;     // 64 - log2(n_filter)
  uint32_t dim;
  uint32_t freq_threshold;
  uint32_t expire_steps;
  uint32_t bf16;
  uint32_t filter_hashes;    // counters per key (1..4); the key's count is their minimum
  uint32_t sync_epoch;       // current synchronisation window (>= 1); rows with touch == sync_epoch are "touched"
  unsigned long long* hwm_mail;  // pinned HOST word (or null): every lookup_or_insert leaves (its call tag << 32 | hwm)
                                 // there, so that the host can bound the sort's key width without waiting
};

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27;
  z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

// Rows that new keys may take when free_n rows are free.  The last 1/32 of the rows is held back:
// with buckets of eight slots, eviction chains grow steeply past a load of ~0.97 (measured: chains
// of 125 evictions at 0.965), and a chain that hits its bound costs a stash entry, then a resident.
// A table therefore stores at most capacity - capacity/32 keys: a call whose new keys do not ALL fit
// under that limit places none of them (counted in n_full), so that which keys are refused does not
// depend on the order in which the kernels happen to see them.
__host__ __device__ inline int64_t rows_on_offer(uint64_t capacity, int32_t free_n) {
  const int64_t offer = (int64_t)free_n - (int64_t)(capacity >> kReserveShift);
  return offer > 0 ? offer : 0;
}

constexpr int kSweepSlotsPerThread = 8;     // a wave of the sweep owns 64 buckets = one word of the occupancy bitmap
constexpr uint64_t kSweepSlotsPerBlock = 256ull * kSweepSlotsPerThread;
__host__ __device__ inline uint64_t occupancy_words(uint64_t capacity) { return (capacity + 511) / 512; }

__device__ inline uint64_t shr_or_zero(uint64_t h, uint32_t shift) { return shift >= 64 ? 0 : h >> shift; }

__device__ inline uint64_t bucket_index(const TableView& t, int side, uint64_t key) {
  uint64_t h = mix64(key ^ (side == 0 ? t.s_h0 : t.s_h1));
  return shr_or_zero(h, t.bucket_shift) + (side == 0 ? 0 : t.n_buckets);
}

__device__ inline uint64_t filter_index(const TableView& t, uint64_t key, uint32_t j = 0) {
  return shr_or_zero(mix64(key ^ t.s_filter[j]), t.filter_shift);
}

// Initial value of element j of the row of `key`: uniform on a 2^-27 grid in [-2^-4, 2^-4).
// `base` = mix64(key ^ s_init).  Only exact fp32 operations.
__device__ inline float init_value(uint64_t base, uint32_t j) {
  uint32_t u24 = (uint32_t)(mix64(base + (uint64_t)j) >> 40);
  return ((float)u24 * (1.0f / 8388608.0f) - 1.0f) * 0.0625f;
}

// bfloat16 <-> fp32 on bit patterns; round to nearest even.
__device__ inline uint16_t f32_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7F800000u) == 0x7F800000u) {
    if (u & 0x007FFFFFu) u |= 0x00400000u;
    return (uint16_t)(u >> 16);
  }
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// agent-scope relaxed atomics on table words (visible across all compute units of the device)
template <typename T>
__device__ inline T ld_agent(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ inline void st_agent(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline unsigned lane_id() { return __lane_id(); }
__device__ inline uint64_t lanes_below() { return (1ull << lane_id()) - 1ull; }

}  // namespace mono
