// lookup_or_insert: cuckoo probe, count-before-admit, insertion with bounded eviction chain,
// resolve (paper section 2.1; batch semantics of the build's contract).
//
// Four kernels per call:
//   probe_count   (thread per occurrence) hit -> row index + last-seen stamp; miss -> touch the
//                 key's occurrence counter
//   admit_elect   (thread per occurrence, after ALL counts) miss with counter >= threshold -> one
//                 occurrence per distinct key is elected through the per-call dedup set and appended
//                 to one of kWinLists lists (one atomic per block, spread over the lists: a single
//                 append counter would serialise at ~12 ns per atomic on this machine)
//   insert        (dense, grid-stride over the elected occurrences) if all of them fit under the
//                 table's fill limit (else none is placed): take a row from the free stack by rank
//                 (no atomics), insert the key (CAS on 64-bit key slots, eviction chain), mark the
//                 bucket in the occupancy bitmap, initialise the row with the whole wave
//   resolve       duplicates of an admitted key pick up the row of the elected occurrence; one
//                 thread settles the counters and reports the high-water mark of rows to the host
//
// The same four kernels restore snapshot records (RestoreSource): every record is a forced
// admission whose row, accumulator and last-seen step come from the caller instead of from
// init(seed, key) / the current step; a record whose key is already stored is refused.  The
// migrate kernel re-inserts every stored element of one table into another (rehash / grow).
//
// Slot protocol (no 128-bit atomics, no fences): a slot's `meta` word doubles as its lock.
//   free slot:   key == EMPTY, meta == kNoMeta
//   claim:       CAS key EMPTY -> k (wait for the result); then store meta (publishes row + stamp)
//   evict:       old = exch(meta, kNoMeta); row(old) == kNoRow -> slot is free or mid-write, try
//                another; else the caller owns the slot: vk = exch(key, k) (wait), then store meta.
//                The victim (vk, old) continues in its other sub-table.
// Every access in the protocol is an agent-scope atomic performed at the coherence point, and each
// step consumes the result of the previous one, so no ordering fence is needed.  No thread ever
// waits for another one; every loop is bounded.
#include "common.h"
#include "kernels.h"

namespace mono {

// Counts are kept unsaturated in the low half of a counter word and read as min(count, 255).  Where
// counters age, the first touch of a batch cuts the count back to 255; where they do not, a reader
// does so once the count has passed kCountGuard (a batch adds less than 2^28).
constexpr uint32_t kCountGuard = 1u << 30;

// one counter word: `times` occurrences at `step`
__device__ inline void touch_word(const TableView& t, unsigned long long* w, uint32_t step, uint32_t times) {
  if (t.expire_steps == 0) {
    // nothing ever ages: the stamp only moves forward and the count only grows, so two atomics
    // whose results nobody waits for do it (low half = count, high half = last step)
    uint32_t* half = reinterpret_cast<uint32_t*>(w);
    atomicMax(half + 1, step);
    atomicAdd(half, times);
    return;
  }
  unsigned long long cur = ld_agent(w);
  for (;;) {
    if ((uint32_t)(cur >> 32) == step) {  // already touched in this batch: increments only
      atomicAdd(w, (unsigned long long)times);  // unsaturated; read as min(count, 255)
      return;
    }
    // first toucher of the batch: ages the word, stamps the step and adds its occurrences in one exchange
    uint32_t last = (uint32_t)(cur >> 32), cnt = (uint32_t)cur;
    if (cnt > 255u) cnt = 255u;  // the unsaturated count is cut back once per batch: it can never wrap
    if (step - last >= t.expire_steps) cnt = 0;
    const unsigned long long want = ((unsigned long long)step << 32) | (unsigned long long)(cnt + times);
    const unsigned long long old = atomicCAS(w, cur, want);
    if (old == cur) return;
    cur = old;
  }
}

// every counter of the key (section 2.1's probabilistic filter read as a counting filter with
// filter_hashes hashes; two hashes of a key that fall on one counter touch it twice, as the oracle does)
__device__ inline void touch_counter(const TableView& t, uint64_t key, uint32_t step, uint32_t times) {
  for (uint32_t j = 0; j < t.filter_hashes; ++j) touch_word(t, &t.filter[filter_index(t, key, j)], step, times);
}

// Cooperative probe.  A lane owns one key; the eight lanes of a group then visit the group's eight
// buckets one after another, each lane reading 16 bytes, so that a bucket line (eight keys + eight
// meta words) is ONE 128-byte access: lanes 0-3 of the group hold the keys two by two, lanes 4-7 the
// meta words.  (Four 16-byte loads by one lane on the same line cost ~2.5x more once the line comes
// from beyond the L2: measured.)  The eight loads of a lane are independent and in flight together.
// side = 0 probes T0 for the keys flagged `want`, side = 1 probes T1.
__device__ inline void probe_side(const TableView& t, uint64_t k, uint64_t bucket, bool want, uint32_t gi,
                                  uint32_t gbase, unsigned long long* meta_out, int* slot_out) {
  ulonglong2 d[kBucket];
#pragma unroll
  for (int r = 0; r < kBucket; ++r) {
    const int src = (int)gbase + r;
    const int need = __shfl((int)want, src);
    const uint64_t bb = __shfl(bucket, src);
    d[r] = make_ulonglong2(0ull, 0ull);
    if (need) d[r] = reinterpret_cast<const ulonglong2*>(t.buckets + bb)[gi];
  }
#pragma unroll
  for (int r = 0; r < kBucket; ++r) {
    const int src = (int)gbase + r;
    const int need = __shfl((int)want, src);
    const uint64_t kr = __shfl(k, src);
    const bool is_key_lane = gi < 4;
    const uint64_t m0 = __ballot(need && is_key_lane && d[r].x == kr);
    const uint64_t m1 = __ballot(need && is_key_lane && d[r].y == kr);
    const uint32_t g0 = (uint32_t)(m0 >> gbase) & 0xFu, g1 = (uint32_t)(m1 >> gbase) & 0xFu;
    const int s = g0 ? 2 * (__ffs((int)g0) - 1) : (g1 ? 2 * (__ffs((int)g1) - 1) + 1 : -1);
    const int ml = (int)gbase + 4 + ((s < 0 ? 0 : s) >> 1);
    const unsigned long long mx = __shfl(d[r].x, ml), my = __shfl(d[r].y, ml);
    if ((int)gi == r && s >= 0) {
      *meta_out = (s & 1) ? my : mx;
      *slot_out = s;
    }
  }
}

// Threads (= keys) per block of probe_count.  The block's missing keys are gathered in an LDS set with
// their multiplicities and each distinct one touches its counter once: a hot ID that is not (yet)
// admitted would otherwise hit one counter word with 10^5 atomics, which serialise at ~12 ns each.
// The larger the block, the fewer touches such a key makes (one per block that holds it), but a block
// lives as long as its slowest wave and the waves of a large block wait for each other at its barriers.
//   kProbeBlockStatic: tables that never expire keys.  A key misses only until it is admitted, so hot
//     missing keys are rare after the first steps (measured on the default workload: 0.200 ms per
//     launch with 256, 0.225 ms with 1024).
//   kProbeBlockAgeing: tables with expiry, whose counters age and whose hot set may drift: every step
//     brings hot IDs that are new (measured on the streaming workload: 0.55 ms with 1024, 1.5 ms with 256
//     from an empty table; 0.43 / 0.72 / 1.10 ms with 1024 / 512 / 256 on a table at load 0.77).
constexpr int kProbeBlockStatic = 256;
constexpr int kProbeBlockAgeing = 1024;
// Keys per thread on tables with expiry: two turns halve the touches of a hot missing key once more
// (streaming workload at load 0.77: 0.424 ms per launch with one key per thread, 0.380 with two, 0.391
// with four, whose 96 KB set of missing keys leaves one block per compute unit; blocks of 512 and 256
// threads with one key each take 0.72 and 1.10 ms: the kernel's time follows the number of blocks that
// touch the hottest counters, ~12 ns per touch of one word).
constexpr int kProbeTurnsAgeing = 2;

// restore != 0: the keys are snapshot records; a stored key is marked absent (its record is refused)
// and nothing is stamped or counted.
// kTurns: keys per thread.  A block owns kProbeBlock * kTurns consecutive keys and takes them in kTurns
// turns of one key per thread; the LDS set of missing keys spans all turns, so that a hot missing key
// costs one counter touch per kProbeBlock * kTurns keys.
template <int kProbeBlock, int kTurns>
__global__ __launch_bounds__(kProbeBlock) void probe_count_kernel(TableView t, const int64_t* __restrict__ keys,
                                                                  uint64_t n, uint32_t step,
                                                                  int32_t* __restrict__ rows_out, int restore) {
  constexpr int kMissSlots = 2 * kProbeBlock * kTurns;  // slots of the block's LDS set of missing keys
  __shared__ unsigned long long miss_key[kMissSlots];
  __shared__ uint32_t miss_cnt[kMissSlots];
  for (int s = threadIdx.x; s < kMissSlots; s += kProbeBlock) {
    miss_key[s] = kEmptyKey;
    miss_cnt[s] = 0;
  }
  __syncthreads();  // the LDS set is cleared
  const uint32_t lane = lane_id(), gi = lane & 7u, gbase = lane & ~7u;
  bool sparse = false;  // (tables with expiry) less than a quarter full: the occupancy bitmap is worth a look
  if (t.expire_steps != 0) {
    const int32_t free_n = t.ctl->free_n;
    sparse = ((uint64_t)t.capacity - (uint64_t)(free_n < 0 ? 0 : free_n)) * 4 <= t.capacity;
  }
#pragma unroll 1
  for (int turn = 0; turn < kTurns; ++turn) {
    const uint64_t i = ((uint64_t)blockIdx.x * kTurns + (uint64_t)turn) * kProbeBlock + threadIdx.x;
    const uint64_t k = i < n ? (uint64_t)keys[i] : kEmptyKey;
    const bool live = k != kEmptyKey;
    // Negative lookup through the admission counters.  When nothing ages (expire_steps == 0) a
    // counter never decreases, and a stored key reached freq_threshold on its counter when it was
    // admitted: a counter below the threshold proves the key absent, and both bucket probes are saved
    // (most misses are tail IDs seen once).  Counts added by this very batch can only make the test
    // err on the side of probing.
    bool maybe = live;
    if (t.expire_steps == 0 && live && !restore) {
      uint32_t cnt = 0xFFFFFFFFu;
      for (uint32_t j = 0; j < t.filter_hashes; ++j) {  // the key's count is the smallest of its counters
        uint32_t* w = reinterpret_cast<uint32_t*>(&t.filter[filter_index(t, k, j)]);
        const uint32_t c = *w;
        if (c > kCountGuard) atomicMin(w, 255u);  // an unsaturated count (read as min(count, 255)) must never wrap
        cnt = c < cnt ? c : cnt;
      }
      maybe = cnt >= (t.freq_threshold > 1u ? t.freq_threshold : 1u);
    }
    const uint64_t b0 = bucket_index(t, 0, k), b1 = bucket_index(t, 1, k);
    // Where counters age nothing above could prove a key absent.  On a sparsely filled table the
    // occupancy bitmap, which is small enough to stay in the caches, often proves a bucket empty: such a
    // bucket is not read.  (Where the counters do the proving, the bitmap would only add a dependent
    // access: measured, 4 % on the step.)
    bool look0 = maybe, look1 = maybe;
    if (sparse && maybe) {
      look0 = (t.occupied[b0 >> 6] >> (b0 & 63)) & 1ull;
      look1 = (t.occupied[b1 >> 6] >> (b1 & 63)) & 1ull;
    }
    unsigned long long m = kNoMeta;
    int slot = -1;
    uint64_t where = b0;
    if (__ballot(look0))  // wave-uniform
      probe_side(t, k, b0, look0, gi, gbase, &m, &slot);
    const bool again = look1 && slot < 0;
    if (__ballot(again)) {  // wave-uniform
      probe_side(t, k, b1, again, gi, gbase, &m, &slot);
      if (again) where = b1;
    }
    bool miss = false;
    if (i < n) {
      if (!live) {
        rows_out[i] = kRowAbsent;
      } else if (slot >= 0) {
        rows_out[i] = restore ? kRowAbsent : (int32_t)meta_row(m);
        if (!restore && meta_seen(m) != step)
          reinterpret_cast<uint32_t*>(&t.buckets[where].meta[slot])[1] = step;  // stamp
      } else {
        miss = true;
        const uint32_t sn = t.ctl->stash_n;
        if (sn) {
          const uint32_t lim = sn < kStashCap ? sn : kStashCap;
          for (uint32_t s = 0; s < lim && miss; ++s)
            if (t.stash[s].key == k) {
              rows_out[i] = restore ? kRowAbsent : (int32_t)t.stash[s].row;
              if (!restore) t.stash[s].seen = step;
              miss = false;
            }
        }
        if (miss) rows_out[i] = kRowMiss;
      }
    }
    if (miss && !restore) {  // (records of a restore call are not occurrences: nothing is counted)
      uint32_t pos = (uint32_t)(mix64(k ^ t.s_dedup) >> 40) & (kMissSlots - 1);
      for (;;) {  // at most half of the slots are ever taken: a free slot always turns up
        const unsigned long long old = atomicCAS(&miss_key[pos], (unsigned long long)kEmptyKey, (unsigned long long)k);
        if (old == kEmptyKey || old == k) break;
        pos = (pos + 1) & (kMissSlots - 1);
      }
      atomicAdd(&miss_cnt[pos], 1u);
    }
  }
  if (restore) return;  // block-uniform
  __syncthreads();
  for (int s = threadIdx.x; s < kMissSlots; s += kProbeBlock)
    if (miss_cnt[s]) touch_counter(t, miss_key[s], step, miss_cnt[s]);
}

// ---- election ------------------------------------------------------------------------------------

// kElectBlock: occurrences (= threads) per block.  256 on tables that never expire keys; 1024 on tables
// with expiry, where an ID that turns hot before it is admitted is led by one occurrence per block, and
// all those leaders meet at one position of the dedup set.
template <int kElectBlock>
__global__ __launch_bounds__(kElectBlock) void admit_elect_kernel(TableView t, const int64_t* __restrict__ keys,
                                                                  uint64_t n, uint32_t epoch, int32_t* rows_out,
                                                                  int restore) {
  constexpr int kElectSlots = 2 * kElectBlock;  // slots of a block's LDS set of missing keys
  constexpr int kElectWaves = kElectBlock / 64;
  __shared__ uint32_t wave_cnt[kElectWaves];
  __shared__ uint32_t block_base;
  // The block's occurrences of one missing key are represented by one of them (the leader): a key
  // that turns hot before it is admitted arrives here in thousands of occurrences, and each of them
  // re-reading the counter and competing for the same position of the dedup set serialised.
  __shared__ unsigned long long s_key[kElectSlots];
  __shared__ int32_t s_res[kElectSlots];  // what the leader found: kRowAbsent, or the dedup-set position as -(pos) - 3
  for (int s = threadIdx.x; s < kElectSlots; s += kElectBlock) s_key[s] = kEmptyKey;
  __syncthreads();
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool miss = i < n && rows_out[i] == kRowMiss;
  const uint64_t k = miss ? (uint64_t)keys[i] : kEmptyKey;
  bool leader = false;
  uint32_t ls = 0;
  if (miss) {
    ls = (uint32_t)(mix64(k ^ t.s_dedup) >> 32) & (kElectSlots - 1);
    for (;;) {  // at most half of the slots are ever taken: a free slot always turns up
      const unsigned long long old = atomicCAS(&s_key[ls], (unsigned long long)kEmptyKey, (unsigned long long)k);
      if (old == kEmptyKey) leader = true;
      if (old == kEmptyKey || old == k) break;
      ls = (ls + 1) & (kElectSlots - 1);
    }
  }
  bool winner = false;
  uint64_t pos = 0;
  if (leader) {
    // A snapshot record is admitted whatever its counter says, and with a threshold of 0 or 1 every
    // missing key is admissible (its count is at least 1 by now): no counter is read for either.
    uint32_t cnt = 255u;
    if (!restore && t.freq_threshold > 1u) {
      for (uint32_t j = 0; j < t.filter_hashes; ++j) {  // smallest of the key's counters
        const uint32_t c = reinterpret_cast<const uint32_t*>(&t.filter[filter_index(t, k, j)])[0];
        cnt = c < cnt ? c : cnt;  // (counts are kept unsaturated and read as min(count, 255))
      }
    }
    int32_t found = kRowAbsent;
    if (cnt >= t.freq_threshold) {
      // one occurrence per distinct key wins its position of the per-call dedup set
      pos = mix64(k ^ t.s_dedup) & t.dset_mask;
      const unsigned long long mine = ((unsigned long long)epoch << 32) | (unsigned long long)i;
      for (;;) {
        unsigned long long e = ld_agent(&t.dset[pos]);
        if ((uint32_t)(e >> 32) != epoch) {
          const unsigned long long old = atomicCAS(&t.dset[pos], e, mine);
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
      // (a second record of the same key in one restore call is refused like a stored key)
      found = restore ? kRowAbsent : -(int32_t)pos - 3;
    }
    s_res[ls] = found;
    if (!winner) rows_out[i] = found;  // the winner keeps kRowMiss until the insertion gives it its row
  }
  __syncthreads();
  if (miss && !leader) rows_out[i] = s_res[ls];
  // block-aggregated append to sub-list (blockIdx mod kWinLists)
  const uint32_t wave = threadIdx.x >> 6;
  const uint64_t wmask = __ballot(winner);
  if (lane_id() == 0) wave_cnt[wave] = (uint32_t)__popcll(wmask);
  __syncthreads();
  const uint32_t list = blockIdx.x & (kWinLists - 1);
  if (threadIdx.x == 0) {
    uint32_t total = 0;
    for (int w = 0; w < kElectWaves; ++w) total += wave_cnt[w];
    block_base = total ? atomicAdd(&t.win_cnt[list * kWinStride], total) : 0u;
  }
  __syncthreads();
  if (winner) {
    uint32_t p = block_base + (uint32_t)__popcll(wmask & lanes_below());
    for (uint32_t w = 0; w < wave; ++w) p += wave_cnt[w];
    t.win_list[(uint64_t)list * t.win_cap + p] = Winner{k, (uint32_t)i, (uint32_t)pos};
  }
}

// ---- insertion ---------------------------------------------------------------------------------

__device__ inline void wait_all_memory_ops() {
  __asm__ volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0);  // every load, store and atomic of this wave has been performed
  __asm__ volatile("" ::: "memory");
}

// The bucket's bit in the occupancy bitmap.  Read first, with an ordinary load: most buckets that take a
// key hold one already, and a stale copy can only show a bit as clear that another compute unit has set
// in this very kernel (bits are cleared by the sweep alone, in a kernel of its own), which costs one
// redundant atomic.
__device__ inline void mark_occupied(const TableView& t, const Bucket* b) {
  const uint64_t idx = (uint64_t)(b - t.buckets);
  unsigned long long* w = &t.occupied[idx >> 6];
  const unsigned long long bit = 1ull << (idx & 63);
  if (!(*w & bit)) atomicOr(w, bit);
}

__device__ inline bool try_claim(const TableView& t, Bucket* b, uint64_t k, unsigned long long meta) {
  // snapshot of the eight keys (may be stale: a slot seen free may be taken by now; the CAS decides)
  const ulonglong2* kp = reinterpret_cast<const ulonglong2*>(b->key);
  const ulonglong2 a0 = kp[0], a1 = kp[1], a2 = kp[2], a3 = kp[3];
  const uint64_t snap[kBucket] = {a0.x, a0.y, a1.x, a1.y, a2.x, a2.y, a3.x, a3.y};
#pragma unroll
  for (int l = 0; l < kBucket; ++l) {
    if (snap[l] != kEmptyKey) continue;
    if (atomicCAS((unsigned long long*)&b->key[l], (unsigned long long)kEmptyKey, (unsigned long long)k) ==
        (unsigned long long)kEmptyKey) {
      st_agent(&b->meta[l], meta);  // issued after the CAS has returned: publishes the slot
      mark_occupied(t, b);
      return true;
    }
  }
  return false;
}

__device__ inline bool has_empty_key(const Bucket* b) {
  const ulonglong2* kp = reinterpret_cast<const ulonglong2*>(b->key);
  const ulonglong2 a0 = kp[0], a1 = kp[1], a2 = kp[2], a3 = kp[3];
  return a0.x == kEmptyKey || a0.y == kEmptyKey || a1.x == kEmptyKey || a1.y == kEmptyKey || a2.x == kEmptyKey ||
         a2.y == kEmptyKey || a3.x == kEmptyKey || a3.y == kEmptyKey;
}

// Which resident of the full bucket b (in sub-table `side`) to evict.  A victim whose OTHER bucket has
// a free slot ends the chain after one move, so the other buckets of the eight residents are looked
// at first (eight independent line reads) and the first such resident from `start` on is chosen;
// if there is none, `start` itself.  Only a hint: the snapshot may be stale, the protocol decides.
// Measured on the streaming configuration at load 0.92: a random victim gave chains of up to 20
// evictions, each five dependent memory round trips long, and the slowest chain is the kernel's time.
__device__ inline uint32_t pick_victim(const TableView& t, const Bucket* b, int side, uint32_t start) {
  const ulonglong2* kp = reinterpret_cast<const ulonglong2*>(b->key);
  const ulonglong2 a0 = kp[0], a1 = kp[1], a2 = kp[2], a3 = kp[3];
  const uint64_t res[kBucket] = {a0.x, a0.y, a1.x, a1.y, a2.x, a2.y, a3.x, a3.y};
  uint32_t good = 0;  // bit l: resident l could move out at once
#pragma unroll
  for (int l = 0; l < kBucket; ++l) {
    if (res[l] == kEmptyKey) continue;
    if (has_empty_key(&t.buckets[bucket_index(t, 1 - side, res[l])])) good |= 1u << l;
  }
  if (good == 0) return start;
  const uint32_t rotated = ((good >> start) | (good << (kBucket - start))) & 0xFFu;  // bit 0 = slot `start`
  return (start + (uint32_t)__ffs((int)rotated) - 1u) & (kBucket - 1);
}

// Inserts (k, meta); k is not in the table and no other thread inserts the same key.
__device__ void cuckoo_insert(const TableView& t, uint64_t k, unsigned long long meta) {
  int side = 0;
  uint32_t chain = 0;
#pragma unroll 1
  for (int kick = 0; kick < kMaxKicks; ++kick) {
    Bucket* b = &t.buckets[bucket_index(t, side, k)];
    if (try_claim(t, b, k, meta)) goto done;
    if (kick == 0 && try_claim(t, &t.buckets[bucket_index(t, 1, k)], k, meta)) goto done;
    // evict: take the lock of a published slot
    const uint32_t v0 = pick_victim(t, b, side, (uint32_t)(mix64(k + (uint64_t)kick) >> 61));
#pragma unroll 1
    for (int tries = 0; tries < kBucket; ++tries) {
      const int l = (int)((v0 + (uint32_t)tries) & (kBucket - 1));
      const unsigned long long old = atomicExch(&b->meta[l], kNoMeta);
      if (meta_row(old) == kNoRow) continue;  // free or mid-write: not ours
      const uint64_t vk = atomicExch((unsigned long long*)&b->key[l], (unsigned long long)k);
      wait_all_memory_ops();  // the key exchange is performed before the slot is published again
      st_agent(&b->meta[l], meta);
      k = vk;
      meta = old;
      side = 1 - side;  // the victim continues in its other sub-table
      ++chain;
      break;
    }
  }
  {  // chain bound hit: keep the homeless element aside
    const uint32_t s = atomicAdd(&t.ctl->stash_n, 1u);
    atomicAdd(&t.ctl->n_insert_failed, 1ull);
    if (s < kStashCap) {
      t.stash[s].key = k;
      t.stash[s].row = meta_row(meta);
      t.stash[s].seen = meta_seen(meta);
    } else {
      atomicAdd(&t.ctl->n_lost, 1ull);
    }
  }
done:
  // (read first: an atomic on this one word from every insertion that evicted serialises at ~12 ns each,
  // which at load 0.8 was most of the kernel's time)
  if (chain && (unsigned long long)chain > ld_agent(&t.ctl->max_chain))
    atomicMax(&t.ctl->max_chain, (unsigned long long)chain);
}

template <typename E>
__device__ inline void store_init4(E* rows, uint64_t idx, float4 v);
template <>
__device__ inline void store_init4<float>(float* rows, uint64_t idx, float4 v) {
  *reinterpret_cast<float4*>(rows + idx) = v;
}
template <>
__device__ inline void store_init4<uint16_t>(uint16_t* rows, uint64_t idx, float4 v) {
  uint2 u;
  u.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
  u.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
  *reinterpret_cast<uint2*>(rows + idx) = u;
}

// Dense over the elected occurrences: winner number w of the call takes free_rows[free_n - 1 - w].
template <typename E>
__global__ __launch_bounds__(256) void insert_kernel(TableView t, uint32_t step, int32_t* rows_out,
                                                     RestoreSource src) {
  const uint32_t lane = lane_id();
  // inclusive prefix of the sub-list fills, one list per lane
  uint32_t inc = t.win_cnt[lane * kWinStride];
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t y = __shfl_up(inc, d);
    if ((int)lane >= d) inc += y;
  }
  const uint32_t total = __shfl(inc, 63);
  const int32_t free0 = t.ctl->free_n;  // settled by the resolve kernel, constant here
  // all of the call's new keys fit under the fill limit, or none of them is placed
  const bool room = (int64_t)total <= rows_on_offer(t.capacity, free0);
  E* rows = reinterpret_cast<E*>(t.rows);
  const uint32_t stride = gridDim.x * blockDim.x;
  for (uint32_t w0 = blockIdx.x * blockDim.x + (threadIdx.x & ~63u); w0 < total; w0 += stride) {
    const uint32_t w = w0 + lane;
    const bool valid = w < total;
    // sub-list of w: the first list whose inclusive prefix exceeds w
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
    uint64_t k = 0;
    uint32_t row = kNoRow, occ = 0;
    if (valid) {
      const uint32_t p = w - (lo > 0 ? before : 0u);
      const Winner e = t.win_list[(uint64_t)lo * t.win_cap + p];
      occ = e.occ;
      k = e.key;
      if (room) row = t.free_rows[free0 - 1 - (int32_t)w];
      t.dset_row[e.pos] = row == kNoRow ? kRowAbsent : (int32_t)row;
      rows_out[e.occ] = row == kNoRow ? kRowAbsent : (int32_t)row;
      if (row != kNoRow) {
        cuckoo_insert(t, k, make_meta(row, src.seen ? src.seen[e.occ] : step));
        if (src.values && t.expire_steps == 0) {
          // a restored key counts as seen freq_threshold times: its counters are raised to that
          // (records may come without their counters, and a counter below the threshold would
          // otherwise "prove" the key absent to the next lookup).  Counters that age prove nothing
          // and are left as they are: the restored table is then the snapshot, whatever the order
          // in which records and counter words arrive
          const uint32_t least = t.freq_threshold > 1u ? t.freq_threshold : 1u;
          for (uint32_t j = 0; j < t.filter_hashes; ++j)
            atomicMax(reinterpret_cast<uint32_t*>(&t.filter[filter_index(t, k, j)]), least);
        }
      }
    }
    // the wave initialises its new rows together: a group of dim/4 lanes per row (at most the whole
    // wave, which then walks the row in pieces of 256 elements), four elements per lane, 64/group rows
    // at a time, stored as whole 16-byte (fp32) or 8-byte (bf16) pieces
    uint32_t glog = 0;
    while (glog < 6 && (4u << glog) < t.dim) ++glog;
    const uint32_t group = 1u << glog, per_round = 64u >> glog, l = lane & (group - 1u), gi = lane >> glog;
    const int ok = valid && row != kNoRow;
    if (__ballot(ok) == 0) continue;  // wave-uniform
    for (uint32_t q = 0; q < group; ++q) {
      const int from = (int)(q * per_round + gi);
      const uint64_t kk = __shfl(k, from);
      const uint32_t rr = __shfl(row, from);
      const uint32_t oo = __shfl(occ, from);
      if (!__shfl(ok, from)) continue;
      for (uint32_t col = l * 4; col < t.dim; col += 256) {
        float4 v;
        if (src.values) {
          v = *reinterpret_cast<const float4*>(src.values + (uint64_t)oo * t.dim + col);
        } else {
          const uint64_t base_h = mix64(kk ^ t.s_init);
          v = make_float4(init_value(base_h, col), init_value(base_h, col + 1), init_value(base_h, col + 2),
                          init_value(base_h, col + 3));
        }
        store_init4<E>(rows, (uint64_t)rr * t.dim + col, v);
      }
      if (l == 0) t.state[rr] = RowState{src.acc ? src.acc[oo] : 0.0f, 0u};
    }
  }
}

__global__ __launch_bounds__(256) void resolve_kernel(TableView t, uint64_t n, int32_t* rows_out, uint32_t epoch) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const int32_t v = rows_out[i];
    if (v <= -3) rows_out[i] = t.dset_row[(uint64_t)(-(v + 3))];
  }
  if (i == 0) {  // settle the counters of this call (the insert kernel has finished)
    uint32_t total = 0;
    for (int l = 0; l < kWinLists; ++l) {
      total += t.win_cnt[l * kWinStride];
      t.win_cnt[l * kWinStride] = 0;
    }
    const int32_t free0 = t.ctl->free_n;
    const uint32_t offer = (uint32_t)rows_on_offer(t.capacity, free0);
    const uint32_t got = total <= offer ? total : 0u;  // all of the call's new keys or none
    t.ctl->free_n = free0 - (int32_t)got;
    const uint32_t in_use = (uint32_t)t.capacity - (uint32_t)(free0 - (int32_t)got);
    if (in_use > t.ctl->hwm) t.ctl->hwm = in_use;  // rows are handed out in ascending order
    if (t.hwm_mail)  // the host reads this word when it pleases; the mark only ever grows, so a stale value is a safe one
      __hip_atomic_store(t.hwm_mail, ((unsigned long long)epoch << 32) | (unsigned long long)t.ctl->hwm, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_SYSTEM);
    t.ctl->n_admitted += got;
    t.ctl->n_full += total - got;
  }
}

// Records of a restore call that were refused (rows_out < 0 after the resolve step) -> scratch slot.
__global__ __launch_bounds__(256) void count_refused_kernel(TableView t, uint64_t n, const int32_t* rows_out) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t m = __ballot(i < n && rows_out[i] < 0);
  if (m && lane_id() == 0) atomicAdd(&t.ctl->scratch[kRefusedRecords], (unsigned long long)__popcll(m));
}

hipError_t launch_lookup_or_insert(const TableView& t, const int64_t* d_keys, uint64_t n, uint32_t step, uint32_t epoch,
                                   int32_t* d_rows_out, const RestoreSource& src, hipStream_t stream, Profiler* prof) {
  if (n == 0) return hipSuccess;
  const int restore = src.values != nullptr;
  const dim3 block(256), grid((unsigned)((n + 255) / 256));
  const dim3 igrid(grid.x < 2048u ? grid.x : 2048u);
  if (t.expire_steps == 0)
    MONO_LAUNCH(prof, K_PROBE_COUNT, stream, (probe_count_kernel<kProbeBlockStatic, 1>),
                dim3((unsigned)((n + kProbeBlockStatic - 1) / kProbeBlockStatic)), dim3(kProbeBlockStatic), t, d_keys, n,
                step, d_rows_out, restore);
  else {
    constexpr uint64_t per_block = (uint64_t)kProbeBlockAgeing * kProbeTurnsAgeing;
    MONO_LAUNCH(prof, K_PROBE_COUNT, stream, (probe_count_kernel<kProbeBlockAgeing, kProbeTurnsAgeing>),
                dim3((unsigned)((n + per_block - 1) / per_block)), dim3(kProbeBlockAgeing), t, d_keys, n, step, d_rows_out,
                restore);
  }
  if (t.expire_steps == 0)
    MONO_LAUNCH(prof, K_ADMIT_ELECT, stream, admit_elect_kernel<256>, grid, block, t, d_keys, n, epoch, d_rows_out, restore);
  else
    MONO_LAUNCH(prof, K_ADMIT_ELECT, stream, admit_elect_kernel<1024>, dim3((unsigned)((n + 1023) / 1024)), dim3(1024), t,
                d_keys, n, epoch, d_rows_out, restore);
  if (t.bf16)
    MONO_LAUNCH(prof, K_INSERT, stream, insert_kernel<uint16_t>, igrid, block, t, step, d_rows_out, src);
  else
    MONO_LAUNCH(prof, K_INSERT, stream, insert_kernel<float>, igrid, block, t, step, d_rows_out, src);
  MONO_LAUNCH(prof, K_RESOLVE, stream, resolve_kernel, grid, block, t, n, d_rows_out, epoch);
  if (restore) hipLaunchKernelGGL(count_refused_kernel, grid, block, 0, stream, t, n, d_rows_out);
  return hipGetLastError();
}

// ---- rehash / grow -------------------------------------------------------------------------------

// Every stored element of `src` (slots, then the stash) is inserted into `dst` under dst's hash
// functions, with its row index and last-seen step unchanged (the rows themselves are copied
// separately, position for position).  Elements are distinct and none is in dst: the insertion
// protocol's preconditions hold.
__global__ __launch_bounds__(256) void migrate_kernel(TableView dst, TableView src) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g < src.capacity) {
    const Bucket* b = &src.buckets[g >> 3];
    const unsigned long long m = b->meta[g & 7];
    if (meta_row(m) != kNoRow) cuckoo_insert(dst, b->key[g & 7], m);
  } else if (g < src.capacity + kStashCap) {
    const uint32_t s = (uint32_t)(g - src.capacity);
    const uint32_t sn = src.ctl->stash_n < kStashCap ? src.ctl->stash_n : kStashCap;
    if (s < sn) cuckoo_insert(dst, src.stash[s].key, make_meta(src.stash[s].row, src.stash[s].seen));
  }
}

// Free stack of the grown table: the new rows at the bottom (handed out last, in ascending order),
// the free rows of the old table above them in their old order.
__global__ __launch_bounds__(256) void migrate_free_rows_kernel(TableView dst, TableView src, int32_t src_free_n) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t extra = dst.capacity - src.capacity;
  if (g < extra)
    dst.free_rows[g] = (uint32_t)(dst.capacity - 1 - g);
  else if (g < extra + (uint64_t)src_free_n)
    dst.free_rows[g] = src.free_rows[g - extra];
}

// Counter i of the grown array takes the value of the counter its keys used to share (top-bit
// addressing: old index = new index >> shift).
__global__ __launch_bounds__(256) void migrate_filter_kernel(TableView dst, TableView src, uint32_t shift) {
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g < dst.n_filter) dst.filter[g] = src.filter[g >> shift];
}

hipError_t launch_migrate(const TableView& dst, const TableView& src, int32_t src_free_n, hipStream_t stream) {
  uint32_t shift = 0;
  while ((src.capacity << shift) < dst.capacity) ++shift;
  const dim3 block(256);
  hipLaunchKernelGGL(migrate_filter_kernel, dim3((unsigned)((dst.n_filter + 255) / 256)), block, 0, stream, dst, src,
                     shift);
  hipLaunchKernelGGL(migrate_free_rows_kernel, dim3((unsigned)((dst.capacity + 255) / 256)), block, 0, stream, dst, src,
                     src_free_n);
  const uint64_t total = src.capacity + kStashCap;
  hipLaunchKernelGGL(migrate_kernel, dim3((unsigned)((total + 255) / 256)), block, 0, stream, dst, src);
  return hipGetLastError();
}

}  // namespace mono
