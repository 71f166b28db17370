// Expiry sweep (paper section 2.1, second heuristic: IDs inactive for a configured time are
// removed), plus the untimed maintenance kernels: initialisation, table dump (all keys, or only the
// keys trained in the current synchronisation window: section 2.2.3), counter dump and counter restore.
#include "common.h"
#include "kernels.h"

namespace mono {

__device__ inline bool is_expired(const TableView& t, uint32_t now, uint32_t seen) {
  return t.expire_steps > 0 && now >= seen && now - seen >= t.expire_steps;
}

// Sweep in four kernels:
//   sweep_begin  one thread: walks the (normally empty) stash; scratch[kSweepRemoved] = keys removed so far
//   sweep_find   eight slots per thread, only in buckets that the occupancy bitmap does not prove empty:
//                slots whose stamp is too old are appended to one of kWinLists lists (one atomic per
//                block, spread over the lists)
//   sweep_remove dense over the found slots: pushes the row on the free stack by rank, reports the
//                key, clears the slot
//   sweep_end    one thread settles the counters
__global__ void sweep_begin_kernel(TableView t, uint32_t now, int64_t* expired_keys, uint64_t max_expired) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  Control* c = t.ctl;
  unsigned long long removed = 0;
  uint32_t sn = c->stash_n < kStashCap ? c->stash_n : kStashCap;
  for (uint32_t s = 0; s < sn;) {
    if (is_expired(t, now, t.stash[s].seen)) {
      if (expired_keys && removed < max_expired) expired_keys[removed] = (int64_t)t.stash[s].key;
      t.free_rows[c->free_n] = t.stash[s].row;
      c->free_n += 1;
      t.stash[s] = t.stash[sn - 1];
      --sn;
      ++removed;
    } else {
      ++s;
    }
  }
  c->stash_n = sn;
  c->scratch[kSweepRemoved] = removed;
}

// A wave looks at 512 consecutive slots = 64 buckets = one word of the occupancy bitmap at a time; a lane
// looks at one slot of eight of those buckets (eight independent 8-byte loads, the eight lanes of a group
// covering a bucket's meta words as one 64-byte access), and only at buckets whose bit is set: a sweep
// over a sparsely filled table reads the bitmap and little else.  A bucket found empty gets its bit
// cleared.  A wave walks `iters` consecutive words (a large table would otherwise need 10^5 blocks that do
// next to nothing each) and asks for all of them at once, one per lane.  Waves never wait for each other:
// a wave that found expired slots reserves its room in a sub-list with one atomic of its own.
constexpr uint32_t kSweepMaxIters = 64;
__global__ __launch_bounds__(256) void sweep_find_kernel(TableView t, uint32_t now, uint32_t iters) {
  const uint32_t lane = lane_id(), grp = lane >> 3, l8 = lane & 7;
  const uint64_t n_words = occupancy_words(t.capacity);
  const uint64_t word0 = (((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * iters;
  if (word0 >= n_words) return;  // wave-uniform
  // a table that is at least a quarter full has hardly an empty bucket: its sweep does not wait for the
  // bitmap words before it asks for the buckets (and leaves the bitmap alone)
  const int32_t free_n = t.ctl->free_n;
  const bool dense = ((uint64_t)t.capacity - (uint64_t)(free_n < 0 ? 0 : free_n)) * 4 > t.capacity;
  unsigned long long mine = 0;  // lane i: the bitmap word of the wave's i-th turn
  if (lane < iters && word0 + lane < n_words) mine = dense ? ~0ull : t.occupied[word0 + lane];
#pragma unroll 1
  for (uint32_t i = 0; i < iters; ++i) {
    const unsigned long long bits = __shfl(mine, (int)i);
    if (bits == 0) continue;  // wave-uniform: no bucket of these 64 holds anything (or past the end)
    const uint64_t word = word0 + i;
    const uint64_t slot0 = word * 512;
    unsigned long long m[kSweepSlotsPerThread];
#pragma unroll
    for (int s = 0; s < kSweepSlotsPerThread; ++s) {
      const uint32_t bucket_here = 8u * (uint32_t)s + grp;
      const uint64_t slot = slot0 + (uint64_t)bucket_here * 8 + l8;
      m[s] = kNoMeta;
      if (((bits >> bucket_here) & 1ull) && slot < t.capacity) m[s] = t.buckets[slot >> 3].meta[l8];
    }
    uint64_t found[kSweepSlotsPerThread];
    unsigned long long now_empty = 0;  // buckets of this word that are flagged but hold nothing
    uint32_t total = 0;
#pragma unroll
    for (int s = 0; s < kSweepSlotsPerThread; ++s) {
      const bool live = meta_row(m[s]) != kNoRow;
      const uint64_t live_mask = __ballot(live);
      const uint32_t bucket_here = 8u * (uint32_t)s + grp;
      if (!dense && ((bits >> bucket_here) & 1ull) && ((live_mask >> (8 * grp)) & 0xFFull) == 0)
        now_empty |= 1ull << bucket_here;
      found[s] = __ballot(live && is_expired(t, now, meta_seen(m[s])));
      total += (uint32_t)__popcll(found[s]);
    }
    // every lane of a group computed the same verdict for its eight buckets: one lane clears for the wave
#pragma unroll
    for (int d = 8; d < 64; d <<= 1) now_empty |= __shfl_xor(now_empty, d);
    if (lane == 0 && now_empty) atomicAnd(&t.occupied[word], ~now_empty);
    if (total == 0) continue;  // wave-uniform
    const uint32_t list = (uint32_t)(word >> 2) & (kWinLists - 1);  // (the list of the 2048-slot chunk the word lies in)
    uint32_t p = 0;
    if (lane == 0) p = atomicAdd(&t.sweep_cnt[list * kWinStride], total);
    p = __shfl(p, 0);
#pragma unroll
    for (int s = 0; s < kSweepSlotsPerThread; ++s) {
      if ((found[s] >> lane) & 1ull) {
        const uint64_t slot = slot0 + (uint64_t)(8u * (uint32_t)s + grp) * 8 + l8;
        t.sweep_list[(uint64_t)list * t.sweep_cap + p + (uint32_t)__popcll(found[s] & lanes_below())] = (uint32_t)slot;
      }
      p += (uint32_t)__popcll(found[s]);
    }
  }
}

__global__ __launch_bounds__(256) void sweep_remove_kernel(TableView t, int64_t* expired_keys, uint64_t max_expired) {
  const uint32_t lane = lane_id();
  uint32_t inc = t.sweep_cnt[lane * kWinStride];
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t y = __shfl_up(inc, d);
    if ((int)lane >= d) inc += y;
  }
  const uint32_t total = __shfl(inc, 63);
  const int32_t free0 = t.ctl->free_n;                     // constant during this kernel
  const unsigned long long out0 = t.ctl->scratch[kSweepRemoved];       // keys already reported from the stash
  const uint32_t stride = gridDim.x * blockDim.x;
  for (uint32_t w0 = blockIdx.x * blockDim.x + (threadIdx.x & ~63u); w0 < total; w0 += stride) {
    const uint32_t w = w0 + lane;
    uint32_t lo = 0, hi = 64;
#pragma unroll
    for (int it = 0; it < 7; ++it) {  // 65 possible answers: seven halvings
      const uint32_t mid = (lo + hi) >> 1 < 63u ? (lo + hi) >> 1 : 63u;
      const uint32_t v = __shfl(inc, (int)mid);
      if (lo < hi) {
        if (v <= w) lo = mid + 1; else hi = mid;
      }
    }
    const uint32_t before = __shfl(inc, (int)(lo > 0 ? lo - 1 : 0));
    if (w < total) {
      const uint32_t p = w - (lo > 0 ? before : 0u);
      const uint32_t g = t.sweep_list[(uint64_t)lo * t.sweep_cap + p];
      Bucket* b = &t.buckets[g >> 3];
      const int l = (int)(g & 7);
      t.free_rows[free0 + (int32_t)w] = meta_row(b->meta[l]);
      if (expired_keys && out0 + w < max_expired) expired_keys[out0 + w] = (int64_t)b->key[l];
      b->meta[l] = kNoMeta;
      b->key[l] = kEmptyKey;
    }
  }
  // (which block finishes last cannot be known cheaply: the counters are settled by sweep_end)
}

__global__ void sweep_end_kernel(TableView t, uint64_t* n_expired) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  uint32_t total = 0;
  for (int l = 0; l < kWinLists; ++l) {
    total += t.sweep_cnt[l * kWinStride];
    t.sweep_cnt[l * kWinStride] = 0;
  }
  t.ctl->free_n += (int32_t)total;
  const unsigned long long removed = t.ctl->scratch[kSweepRemoved] + total;
  t.ctl->n_expired += removed;
  if (n_expired) *n_expired = removed;
}

__global__ void sweep_nothing_kernel(uint64_t* n_expired) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *n_expired = 0;
}

hipError_t launch_expire_sweep(const TableView& t, uint32_t now, uint64_t* d_n_expired, int64_t* d_expired_keys,
                               uint64_t max_expired, hipStream_t stream, Profiler* prof) {
  if (t.expire_steps == 0) {  // nothing ever expires: only the count is reported
    if (d_n_expired) MONO_LAUNCH(prof, K_SWEEP_END, stream, sweep_nothing_kernel, dim3(1), dim3(64), d_n_expired);
    return hipGetLastError();
  }
  MONO_LAUNCH(prof, K_SWEEP_BEGIN, stream, sweep_begin_kernel, dim3(1), dim3(64), t, now, d_expired_keys, max_expired);
  const uint64_t words = occupancy_words(t.capacity);
  uint64_t iters = (words + 32767) / 32768;  // about 32 K waves, at most kSweepMaxIters bitmap words each
  iters = iters < 1 ? 1 : (iters > kSweepMaxIters ? kSweepMaxIters : iters);
  const uint64_t waves = (words + iters - 1) / iters;
  const dim3 block(256), grid((unsigned)((waves + 3) / 4));
  MONO_LAUNCH(prof, K_SWEEP, stream, sweep_find_kernel, grid, block, t, now, (uint32_t)iters);
  MONO_LAUNCH(prof, K_SWEEP_REMOVE, stream, sweep_remove_kernel, dim3(grid.x < 2048u ? grid.x : 2048u), block, t,
              d_expired_keys, max_expired);
  MONO_LAUNCH(prof, K_SWEEP_END, stream, sweep_end_kernel, dim3(1), dim3(64), t, d_n_expired);
  return hipGetLastError();
}

// ---- dump --------------------------------------------------------------------------------------

__global__ void export_begin_kernel(TableView t) {
  if (blockIdx.x == 0 && threadIdx.x == 0) t.ctl->scratch[kExportCount] = 0;
}

constexpr int kExportBlock = 1024;

// touched_only: keep only the keys whose row was trained in the current synchronisation window
__global__ __launch_bounds__(kExportBlock) void export_kernel(TableView t, int64_t* keys, int32_t* rows,
                                                              uint32_t* last_seen, int64_t* slot, uint64_t max_n,
                                                              bool touched_only) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t total = t.capacity + kStashCap;
  bool live = false;
  uint64_t key = 0;
  uint32_t row = 0, seen = 0;
  int64_t where = -2;
  if (g < t.capacity) {
    const Bucket* b = &t.buckets[g >> 3];
    const int l = (int)(g & 7);
    const unsigned long long m = b->meta[l];
    row = meta_row(m);
    live = row != kNoRow;
    key = b->key[l];
    seen = meta_seen(m);
    where = (int64_t)g;
  } else if (g < total) {
    const uint32_t s = (uint32_t)(g - t.capacity);
    const uint32_t sn = t.ctl->stash_n < kStashCap ? t.ctl->stash_n : kStashCap;
    if (s < sn) {
      live = true;
      key = t.stash[s].key;
      row = t.stash[s].row;
      seen = t.stash[s].seen;
    }
  }
  if (live && touched_only) live = t.state[row].touch == t.sync_epoch;
  // one append per block: the waves' counts meet in LDS (a counter hit once per wave would serialise)
  __shared__ uint32_t wave_cnt[kExportBlock / 64];
  __shared__ unsigned long long block_base;
  const uint32_t wave = threadIdx.x >> 6;
  const uint64_t m = __ballot(live);
  if (lane_id() == 0) wave_cnt[wave] = (uint32_t)__popcll(m);
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t found = 0;
    for (int w = 0; w < kExportBlock / 64; ++w) found += wave_cnt[w];
    block_base = found ? atomicAdd(&t.ctl->scratch[kExportCount], (unsigned long long)found) : 0ull;
  }
  __syncthreads();
  if (live) {
    uint64_t o = block_base + __popcll(m & lanes_below());
    for (uint32_t w = 0; w < wave; ++w) o += wave_cnt[w];
    if (o < max_n) {
      if (keys) keys[o] = (int64_t)key;
      if (rows) rows[o] = (int32_t)row;
      if (last_seen) last_seen[o] = seen;
      if (slot) slot[o] = where;
    }
  }
}

hipError_t launch_export(const TableView& t, int64_t* d_keys, int32_t* d_row, uint32_t* d_last_seen, int64_t* d_slot,
                         uint64_t max_n, bool touched_only, hipStream_t stream) {
  hipLaunchKernelGGL(export_begin_kernel, dim3(1), dim3(64), 0, stream, t);
  const uint64_t total = t.capacity + kStashCap;
  hipLaunchKernelGGL(export_kernel, dim3((unsigned)((total + kExportBlock - 1) / kExportBlock)), dim3(kExportBlock), 0,
                     stream, t, d_keys, d_row, d_last_seen, d_slot, max_n, touched_only);
  return hipGetLastError();
}

// A group of lanes (dim / 4 rounded up to a power of two) copies one row, four elements per lane.
template <typename E>
__global__ __launch_bounds__(256) void export_values_kernel(TableView t, const int32_t* rows, uint64_t n, float* values,
                                                            float* acc, uint32_t group_log2) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t i = g >> group_log2;
  const uint32_t l = (uint32_t)g & ((1u << group_log2) - 1u);
  if (i >= n || l * 4 >= t.dim) return;
  const uint32_t r = (uint32_t)rows[i];
  const E* src = reinterpret_cast<const E*>(t.rows) + (uint64_t)r * t.dim + l * 4;
  if (values) {
    float4 v;
    if constexpr (sizeof(E) == 2) {
      const uint2 u = *reinterpret_cast<const uint2*>(src);
      v = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                      __uint_as_float(u.y & 0xFFFF0000u));
    } else {
      v = *reinterpret_cast<const float4*>(src);
    }
    *reinterpret_cast<float4*>(values + i * t.dim + l * 4) = v;
  }
  if (acc && l == 0) acc[i] = t.state[r].acc;
}

hipError_t launch_export_values(const TableView& t, const int32_t* d_row, uint64_t n, float* d_values, float* d_acc,
                                hipStream_t stream) {
  if (n == 0) return hipSuccess;
  uint32_t group_log2 = 0;
  while ((4u << group_log2) < t.dim) ++group_log2;
  const uint64_t total = n << group_log2;
  dim3 block(256), grid((unsigned)((total + 255) / 256));
  if (t.bf16)
    hipLaunchKernelGGL(export_values_kernel<uint16_t>, grid, block, 0, stream, t, d_row, n, d_values, d_acc, group_log2);
  else
    hipLaunchKernelGGL(export_values_kernel<float>, grid, block, 0, stream, t, d_row, n, d_values, d_acc, group_log2);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void filter_export_kernel(TableView t, uint32_t* words, uint64_t first,
                                                            uint64_t count) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= count) return;
  const unsigned long long w = t.filter[first + g];
  const uint32_t cnt = (uint32_t)w > 255u ? 255u : (uint32_t)w;
  words[g] = (((uint32_t)(w >> 32) & 0xFFFFFFu) << 8) | cnt;
}

hipError_t launch_filter_export(const TableView& t, uint32_t* d_words, uint64_t first, uint64_t count,
                                hipStream_t stream) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(filter_export_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, t, d_words,
                     first, count);
  return hipGetLastError();
}

// canonical word -> the table's own form (step << 32 | count)
__global__ __launch_bounds__(256) void filter_import_kernel(TableView t, const uint32_t* words, uint64_t first,
                                                            uint64_t count) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= count) return;
  const uint32_t w = words[g];
  t.filter[first + g] = ((unsigned long long)(w >> 8) << 32) | (unsigned long long)(w & 255u);
}

// Tables that never expire keys: a stored key stays counted.  Each of its counters inside
// [first, first + count) that the import left below the admission threshold is raised to it (a lookup
// of such a table reads a counter below the threshold as proof that the key is absent).  One thread
// per slot, then the stash.
__global__ __launch_bounds__(256) void filter_raise_kernel(TableView t, uint64_t first, uint64_t count) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint64_t key = kEmptyKey;
  if (g < t.capacity) {
    const Bucket* b = &t.buckets[g >> 3];
    if (meta_row(b->meta[g & 7]) != kNoRow) key = b->key[g & 7];
  } else if (g < t.capacity + kStashCap) {
    const uint32_t s = (uint32_t)(g - t.capacity);
    const uint32_t sn = t.ctl->stash_n < kStashCap ? t.ctl->stash_n : kStashCap;
    if (s < sn) key = t.stash[s].key;
  }
  if (key == kEmptyKey) return;
  const uint32_t least = t.freq_threshold > 1u ? t.freq_threshold : 1u;
  for (uint32_t j = 0; j < t.filter_hashes; ++j) {
    const uint64_t i = filter_index(t, key, j);
    if (i >= first && i - first < count) atomicMax(reinterpret_cast<uint32_t*>(&t.filter[i]), least);
  }
}

hipError_t launch_filter_import(const TableView& t, const uint32_t* d_words, uint64_t first, uint64_t count,
                                hipStream_t stream) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(filter_import_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, t, d_words,
                     first, count);
  if (t.expire_steps == 0) {  // (counters that age prove nothing about stored keys and stay as written)
    const uint64_t total = t.capacity + kStashCap;
    hipLaunchKernelGGL(filter_raise_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, t, first, count);
  }
  return hipGetLastError();
}

// ---- initialisation ------------------------------------------------------------------------------

// Free stack filled so that rows are handed out in ascending order: keys admitted early (the
// frequent ones) end up next to each other in memory.
__global__ __launch_bounds__(256) void init_free_rows_kernel(TableView t) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g < t.capacity) t.free_rows[g] = (uint32_t)(t.capacity - 1 - g);
  if (g == 0) t.ctl->free_n = (int32_t)t.capacity;
}

hipError_t launch_table_init(const TableView& t, uint64_t dset_size, hipStream_t stream) {
  hipError_t e;
  if ((e = hipMemsetAsync(t.buckets, 0xFF, 2 * t.n_buckets * sizeof(Bucket), stream)) != hipSuccess) return e;
  if ((e = hipMemsetAsync(t.filter, 0, t.n_filter * sizeof(unsigned long long), stream)) != hipSuccess) return e;
  if ((e = hipMemsetAsync(t.ctl, 0, sizeof(Control), stream)) != hipSuccess) return e;
  if ((e = hipMemsetAsync(t.win_cnt, 0, kWinLists * kWinStride * sizeof(uint32_t), stream)) != hipSuccess) return e;
  if ((e = hipMemsetAsync(t.sweep_cnt, 0, kWinLists * kWinStride * sizeof(uint32_t), stream)) != hipSuccess) return e;
  if ((e = hipMemsetAsync(t.occupied, 0, occupancy_words(t.capacity) * sizeof(unsigned long long), stream)) != hipSuccess)
    return e;
  if ((e = hipMemsetAsync(t.dset, 0, dset_size * sizeof(unsigned long long), stream)) != hipSuccess) return e;
  hipLaunchKernelGGL(init_free_rows_kernel, dim3((unsigned)((t.capacity + 255) / 256)), dim3(256), 0, stream, t);
  return hipGetLastError();
}

}  // namespace mono
