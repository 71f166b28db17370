// lookup_or_insert: cuckoo probe, count-before-admit, insertion with bounded eviction chain,
// resolve (paper section 2.1; batch semantics of the build's contract).
//
// Three kernels per call, each one thread per occurrence:
//   probe_count   hit -> row index + last-seen stamp; miss -> touch the key's occurrence counter
//   admit_insert  (after ALL counts) miss with counter >= threshold -> elect one occurrence per
//                 distinct key through the per-call dedup set; the elected one takes a row from the
//                 free stack, inserts the key (CAS on 64-bit key slots, eviction chain), and its
//                 wave initialises the row cooperatively
//   resolve       duplicates of an admitted key pick up the row of the elected occurrence
//
// Slot protocol (no 128-bit atomics needed): a slot's `row` word doubles as its lock.
//   free slot:      key == EMPTY, row == kNoRow
//   claim:          CAS key EMPTY -> k; then seen, fence, row (publishing)
//   evict:          old = exch(row, kNoRow); old == kNoRow -> slot is free or mid-write, try another;
//                   else the caller owns the slot: read the victim's key/seen, write its own, fence,
//                   publish row.  The victim continues in its other sub-table.
// No thread ever waits for another one; every loop is bounded.
#include "common.h"
#include "kernels.h"

namespace mono {

__device__ inline int find_in_bucket(const Bucket* b, uint64_t k) {
  const ulonglong2* kp = reinterpret_cast<const ulonglong2*>(b->key);
  ulonglong2 a0 = kp[0], a1 = kp[1], a2 = kp[2], a3 = kp[3];
  int j = -1;
  j = a0.x == k ? 0 : j;
  j = a0.y == k ? 1 : j;
  j = a1.x == k ? 2 : j;
  j = a1.y == k ? 3 : j;
  j = a2.x == k ? 4 : j;
  j = a2.y == k ? 5 : j;
  j = a3.x == k ? 6 : j;
  j = a3.y == k ? 7 : j;
  return j;
}

__device__ inline void touch_counter(const TableView& t, uint64_t key, uint32_t step) {
  unsigned long long* w = &t.filter[filter_index(t, key)];
  unsigned long long cur = ld_agent(w);
  // first toucher of the batch ages the word and stamps the step; increments only ever follow it
  while ((uint32_t)(cur >> 32) != step) {
    uint32_t last = (uint32_t)(cur >> 32), cnt = (uint32_t)cur;
    if (t.expire_steps > 0 && step - last >= t.expire_steps) cnt = 0;
    unsigned long long want = ((unsigned long long)step << 32) | cnt;
    unsigned long long old = atomicCAS(w, cur, want);
    if (old == cur) break;
    cur = old;
  }
  atomicAdd(w, 1ull);  // unsaturated; read as min(count, 255)
}

__global__ __launch_bounds__(256) void probe_count_kernel(TableView t, const int64_t* __restrict__ keys, uint64_t n,
                                                          uint32_t step, int32_t* __restrict__ rows_out) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint64_t k = (uint64_t)keys[i];
  if (k == kEmptyKey) {
    rows_out[i] = kRowAbsent;
    return;
  }
  Bucket* b = &t.buckets[bucket_index(t, 0, k)];
  int j = find_in_bucket(b, k);
  if (j < 0) {
    b = &t.buckets[bucket_index(t, 1, k)];
    j = find_in_bucket(b, k);
  }
  if (j >= 0) {
    rows_out[i] = (int32_t)b->row[j];
    if (b->seen[j] != step) b->seen[j] = step;
    return;
  }
  uint32_t sn = t.ctl->stash_n;
  if (sn) {
    sn = sn < kStashCap ? sn : kStashCap;
    for (uint32_t s = 0; s < sn; ++s)
      if (t.stash[s].key == k) {
        rows_out[i] = (int32_t)t.stash[s].row;
        t.stash[s].seen = step;
        return;
      }
  }
  touch_counter(t, k, step);
  rows_out[i] = kRowMiss;
}

// ---- insertion ---------------------------------------------------------------------------------

__device__ inline bool try_claim(Bucket* b, uint64_t k, uint32_t row, uint32_t seen) {
#pragma unroll 1
  for (int l = 0; l < kBucket; ++l) {
    if (ld_agent(&b->key[l]) != kEmptyKey) continue;
    if (atomicCAS((unsigned long long*)&b->key[l], (unsigned long long)kEmptyKey, (unsigned long long)k) ==
        (unsigned long long)kEmptyKey) {
      st_agent(&b->seen[l], seen);
      __threadfence();
      st_agent(&b->row[l], row);
      return true;
    }
  }
  return false;
}

// Inserts (k, row, seen); k is not in the table and no other thread inserts the same key.
__device__ void cuckoo_insert(const TableView& t, uint64_t k, uint32_t row, uint32_t seen) {
  int side = 0;
  uint32_t chain = 0;
#pragma unroll 1
  for (int kick = 0; kick < kMaxKicks; ++kick) {
    Bucket* b = &t.buckets[bucket_index(t, side, k)];
    if (try_claim(b, k, row, seen)) goto done;
    if (kick == 0 && try_claim(&t.buckets[bucket_index(t, 1, k)], k, row, seen)) goto done;
    // evict: take the lock of a published slot
    uint32_t v0 = (uint32_t)(mix64(k + (uint64_t)kick) >> 61);
#pragma unroll 1
    for (int tries = 0; tries < kBucket; ++tries) {
      int l = (int)((v0 + (uint32_t)tries) & (kBucket - 1));
      uint32_t old = atomicExch(&b->row[l], kNoRow);
      if (old == kNoRow) continue;  // free or mid-write: not ours
      __threadfence();
      uint64_t vk = ld_agent(&b->key[l]);
      uint32_t vs = ld_agent(&b->seen[l]);
      st_agent(&b->key[l], k);
      st_agent(&b->seen[l], seen);
      __threadfence();
      st_agent(&b->row[l], row);
      k = vk;
      row = old;
      seen = vs;
      side = 1 - side;  // the victim continues in its other sub-table
      ++chain;
      break;
    }
  }
  {  // chain bound hit: keep the homeless element aside
    uint32_t s = atomicAdd(&t.ctl->stash_n, 1u);
    atomicAdd(&t.ctl->n_insert_failed, 1ull);
    if (s < kStashCap) {
      t.stash[s].key = k;
      t.stash[s].row = row;
      t.stash[s].seen = seen;
    } else {
      atomicAdd(&t.ctl->n_lost, 1ull);
    }
  }
done:
  if (chain) atomicMax(&t.ctl->max_chain, (unsigned long long)chain);
}

template <typename E>
__device__ inline void store_init(E* rows, uint64_t idx, float v);
template <>
__device__ inline void store_init<float>(float* rows, uint64_t idx, float v) { rows[idx] = v; }
template <>
__device__ inline void store_init<uint16_t>(uint16_t* rows, uint64_t idx, float v) { rows[idx] = f32_to_bf16(v); }

template <typename E>
__global__ __launch_bounds__(256) void admit_insert_kernel(TableView t, const int64_t* __restrict__ keys, uint64_t n,
                                                           uint32_t step, uint32_t epoch, int32_t* rows_out) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool miss = i < n && rows_out[i] == kRowMiss;
  bool winner = false;
  uint64_t k = 0, pos = 0;
  if (miss) {
    k = (uint64_t)keys[i];
    unsigned long long* w = &t.filter[filter_index(t, k)];
    unsigned long long word = *w;
    uint32_t cnt = (uint32_t)word;
    if (cnt > 255u) {  // keep the unsaturated count from ever wrapping
      atomicMin(w, (word & 0xFFFFFFFF00000000ull) | 255ull);
      cnt = 255u;
    }
    if (cnt < t.freq_threshold) {
      rows_out[i] = kRowAbsent;
    } else {
      // one occurrence per distinct key wins its position of the per-call dedup set
      pos = mix64(k ^ t.s_dedup) & t.dset_mask;
      const unsigned long long mine = ((unsigned long long)epoch << 32) | (unsigned long long)i;
      for (;;) {
        unsigned long long e = ld_agent(&t.dset[pos]);
        if ((uint32_t)(e >> 32) != epoch) {
          unsigned long long old = atomicCAS(&t.dset[pos], e, mine);
          if (old == e) {
            winner = true;
            break;
          }
          e = old;  // someone wrote this position in this call
          if ((uint32_t)(e >> 32) != epoch) continue;
        }
        if ((uint64_t)keys[(uint32_t)e] == k) break;  // duplicate of the owner
        pos = (pos + 1) & t.dset_mask;
      }
      if (!winner) rows_out[i] = -(int32_t)pos - 3;
    }
  }
  // winners take rows from the free stack, one atomic per wave
  const uint64_t wmask = __ballot(winner);
  if (wmask == 0) return;
  const int cnt = __popcll(wmask);
  const int leader = __ffsll((unsigned long long)wmask) - 1;
  int base = 0;
  if ((int)lane_id() == leader) base = atomicSub(&t.ctl->free_n, cnt);
  base = __shfl(base, leader);
  uint32_t row = kNoRow;
  if (winner) {
    int idx = base - 1 - __popcll(wmask & lanes_below());
    if (idx >= 0) row = t.free_rows[idx];
  }
  if ((int)lane_id() == leader) {
    int got = base < 0 ? 0 : (base < cnt ? base : cnt);
    if (got < cnt) {
      atomicAdd(&t.ctl->free_n, cnt - got);
      atomicAdd(&t.ctl->n_full, (unsigned long long)(cnt - got));
    }
    if (got) atomicAdd(&t.ctl->n_admitted, (unsigned long long)got);
  }
  if (winner) {
    t.dset_row[pos] = row == kNoRow ? kRowAbsent : (int32_t)row;
    rows_out[i] = row == kNoRow ? kRowAbsent : (int32_t)row;
    if (row != kNoRow) cuckoo_insert(t, k, row, step);
  }
  // the wave initialises the new rows together: coalesced stores, one mixer call per lane
  uint64_t imask = __ballot(winner && row != kNoRow);
  E* rows = reinterpret_cast<E*>(t.rows);
  while (imask) {
    int l = __ffsll((unsigned long long)imask) - 1;
    imask &= imask - 1;
    uint64_t kk = __shfl(k, l);
    uint32_t rr = __shfl(row, l);
    uint64_t base_h = mix64(kk ^ t.s_init);
    for (uint32_t j = lane_id(); j < t.dim; j += 64) store_init<E>(rows, (uint64_t)rr * t.dim + j, init_value(base_h, j));
    if (lane_id() == 0) t.acc[rr] = 0.0f;
  }
}

__global__ __launch_bounds__(256) void resolve_kernel(TableView t, uint64_t n, int32_t* rows_out) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int32_t v = rows_out[i];
  if (v <= -3) rows_out[i] = t.dset_row[(uint64_t)(-(v + 3))];
}

hipError_t launch_lookup_or_insert(const TableView& t, const int64_t* d_keys, uint64_t n, uint32_t step, uint32_t epoch,
                                   int32_t* d_rows_out, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  dim3 block(256), grid((unsigned)((n + 255) / 256));
  hipLaunchKernelGGL(probe_count_kernel, grid, block, 0, stream, t, d_keys, n, step, d_rows_out);
  if (t.bf16)
    hipLaunchKernelGGL(admit_insert_kernel<uint16_t>, grid, block, 0, stream, t, d_keys, n, step, epoch, d_rows_out);
  else
    hipLaunchKernelGGL(admit_insert_kernel<float>, grid, block, 0, stream, t, d_keys, n, step, epoch, d_rows_out);
  hipLaunchKernelGGL(resolve_kernel, grid, block, 0, stream, t, n, d_rows_out);
  return hipGetLastError();
}

}  // namespace mono
