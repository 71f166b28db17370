// Expiry sweep (paper section 2.1, second heuristic: IDs inactive for a configured time are
// removed), plus the untimed maintenance kernels: initialisation, table dump, counter dump.
#include "common.h"
#include "kernels.h"

namespace mono {

__device__ inline bool is_expired(const TableView& t, uint32_t now, uint32_t seen) {
  return t.expire_steps > 0 && now >= seen && now - seen >= t.expire_steps;
}

// scratch[0] = keys removed by this call.  One thread also walks the (normally empty) stash.
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
  c->scratch[0] = removed;
}

// One thread per slot.  Only the second half of each bucket line (row, seen) is read; the key is
// read only for slots that expire.
__global__ __launch_bounds__(256) void sweep_kernel(TableView t, uint32_t now, int64_t* expired_keys,
                                                    uint64_t max_expired) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool expired = false;
  uint32_t row = kNoRow;
  Bucket* b = nullptr;
  int l = 0;
  if (g < t.capacity) {
    b = &t.buckets[g >> 3];
    l = (int)(g & 7);
    row = b->row[l];
    expired = row != kNoRow && is_expired(t, now, b->seen[l]);
  }
  const uint64_t m = __ballot(expired);
  if (m == 0) return;
  const int cnt = __popcll(m), leader = __ffsll((unsigned long long)m) - 1;
  int base = 0;
  unsigned long long obase = 0;
  if ((int)lane_id() == leader) {
    base = atomicAdd(&t.ctl->free_n, cnt);
    obase = atomicAdd(&t.ctl->scratch[0], (unsigned long long)cnt);
  }
  base = __shfl(base, leader);
  obase = __shfl(obase, leader);
  if (expired) {
    const int rank = __popcll(m & lanes_below());
    t.free_rows[base + rank] = row;
    if (expired_keys && obase + rank < max_expired) expired_keys[obase + rank] = (int64_t)b->key[l];
    b->row[l] = kNoRow;
    b->key[l] = kEmptyKey;
  }
}

__global__ void sweep_end_kernel(TableView t, uint64_t* n_expired) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  t.ctl->n_expired += t.ctl->scratch[0];
  if (n_expired) *n_expired = t.ctl->scratch[0];
}

hipError_t launch_expire_sweep(const TableView& t, uint32_t now, uint64_t* d_n_expired, int64_t* d_expired_keys,
                               uint64_t max_expired, hipStream_t stream) {
  hipLaunchKernelGGL(sweep_begin_kernel, dim3(1), dim3(64), 0, stream, t, now, d_expired_keys, max_expired);
  if (t.expire_steps > 0) {
    dim3 block(256), grid((unsigned)((t.capacity + 255) / 256));
    hipLaunchKernelGGL(sweep_kernel, grid, block, 0, stream, t, now, d_expired_keys, max_expired);
  }
  hipLaunchKernelGGL(sweep_end_kernel, dim3(1), dim3(64), 0, stream, t, d_n_expired);
  return hipGetLastError();
}

// ---- dump --------------------------------------------------------------------------------------

__global__ void export_begin_kernel(TableView t) {
  if (blockIdx.x == 0 && threadIdx.x == 0) t.ctl->scratch[1] = 0;
}

__global__ __launch_bounds__(256) void export_kernel(TableView t, int64_t* keys, int32_t* rows, uint32_t* last_seen,
                                                     int64_t* slot, uint64_t max_n) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t total = t.capacity + kStashCap;
  bool live = false;
  uint64_t key = 0;
  uint32_t row = 0, seen = 0;
  int64_t where = -2;
  if (g < t.capacity) {
    const Bucket* b = &t.buckets[g >> 3];
    const int l = (int)(g & 7);
    row = b->row[l];
    live = row != kNoRow;
    key = b->key[l];
    seen = b->seen[l];
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
  const uint64_t m = __ballot(live);
  if (m == 0) return;
  const int leader = __ffsll((unsigned long long)m) - 1;
  unsigned long long base = 0;
  if ((int)lane_id() == leader) base = atomicAdd(&t.ctl->scratch[1], (unsigned long long)__popcll(m));
  base = __shfl(base, leader);
  if (live) {
    const uint64_t o = base + __popcll(m & lanes_below());
    if (o < max_n) {
      if (keys) keys[o] = (int64_t)key;
      if (rows) rows[o] = (int32_t)row;
      if (last_seen) last_seen[o] = seen;
      if (slot) slot[o] = where;
    }
  }
}

hipError_t launch_export(const TableView& t, int64_t* d_keys, int32_t* d_row, uint32_t* d_last_seen, int64_t* d_slot,
                         uint64_t max_n, hipStream_t stream) {
  hipLaunchKernelGGL(export_begin_kernel, dim3(1), dim3(64), 0, stream, t);
  const uint64_t total = t.capacity + kStashCap;
  hipLaunchKernelGGL(export_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, t, d_keys, d_row,
                     d_last_seen, d_slot, max_n);
  return hipGetLastError();
}

template <typename E>
__global__ __launch_bounds__(256) void export_values_kernel(TableView t, const int32_t* rows, uint64_t n, float* values,
                                                            float* acc) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n * t.dim) return;
  const uint64_t i = g / t.dim;
  const uint32_t j = (uint32_t)(g % t.dim);
  const uint32_t r = (uint32_t)rows[i];
  const E* src = reinterpret_cast<const E*>(t.rows);
  if (values) {
    if constexpr (sizeof(E) == 2)
      values[g] = bf16_to_f32((uint16_t)src[(uint64_t)r * t.dim + j]);
    else
      values[g] = (float)src[(uint64_t)r * t.dim + j];
  }
  if (acc && j == 0) acc[i] = t.acc[r];
}

hipError_t launch_export_values(const TableView& t, const int32_t* d_row, uint64_t n, float* d_values, float* d_acc,
                                hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint64_t total = n * t.dim;
  dim3 block(256), grid((unsigned)((total + 255) / 256));
  if (t.bf16)
    hipLaunchKernelGGL(export_values_kernel<uint16_t>, grid, block, 0, stream, t, d_row, n, d_values, d_acc);
  else
    hipLaunchKernelGGL(export_values_kernel<float>, grid, block, 0, stream, t, d_row, n, d_values, d_acc);
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
  if ((e = hipMemsetAsync(t.dset, 0, dset_size * sizeof(unsigned long long), stream)) != hipSuccess) return e;
  hipLaunchKernelGGL(init_free_rows_kernel, dim3((unsigned)((t.capacity + 255) / 256)), dim3(256), 0, stream, t);
  return hipGetLastError();
}

}  // namespace mono
