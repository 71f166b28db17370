// Stable LSD radix sort of (row index, bag) pairs, used to bring the occurrences of one embedding
// row together before the gradient reduction.
//
// The key width is decided ON THE DEVICE: row indices are handed out in ascending order, so every
// row in use is below the high-water mark `hwm` kept in the control block.  bit_length(hwm - 1)
// bits are sorted in the fewest passes of equal width that the call's shape allows (digits of at most eight
// bits in blocks of 2048 elements up to 16 M rows, of at most nine bits in blocks of 4096 elements beyond:
// either way a block's share of a bin leaves as pieces of eight elements on average); the host picks the
// shape and launches the passes that an upper bound of `hwm` needs (it keeps one without waiting for the
// device: see the table's host side) and the superfluous ones return at once.  Pass p reads buffer (p even ? a : b)
// and writes the other one.  Pass 0 reads the row indices as the caller holds them and finds the bag
// of every occurrence from the offsets (no array of bag numbers is ever written to memory); dropped
// occurrences (row -1) are left out by it, and it publishes the number of pairs that remain
// (kValidPairs slot of the control block's scratch).
//
// Unit of work: one block owns kItems consecutive elements, an equal share per wave.  Per pass:
//   hist     per-unit digit histogram (LDS atomics), written bin-major: hist[bin * units + unit]
//   scan     one block per bin: exclusive scan along the units; bin totals to `totals`
//   scatter  the block loads its elements into registers (all loads independent), counts the digits
//            per wave in LDS, turns the counts into start offsets inside the block, then every wave
//            ranks its elements 64 at a time by digit matching with ballots (stable: rank = number
//            of lower lanes with the same digit) and puts them IN ORDER into an LDS copy of the
//            block; the copy is then written out with neighbouring threads on neighbouring
//            elements of a bin.  (Scattering straight from the registers sends one 8-byte write
//            per element to the L2: measured, that request rate was what bounded the pass.)
// No kernel spins or waits for another block.
#include "common.h"
#include "kernels.h"

namespace mono {

// A kernel of the sort is compiled for one shape (see kernels.h): kBits = widest digit, kBlock = threads,
// kItems = elements owned by a block.
template <uint32_t kBits, int kBlock, uint32_t kItems>
struct Shape {
  static constexpr uint32_t kBins = 1u << kBits;
  static constexpr int kWaves = kBlock / 64;
  static constexpr int kScanWaves = (int)kBins / 64;  // the first kBins threads of a block own one bin each
  static constexpr uint32_t kPerWave = kItems / kWaves;
  static constexpr uint32_t kRounds = kPerWave / 64;
  static_assert(kBlock >= (int)kBins && kBlock % 64 == 0 && kItems % (uint32_t)kBlock == 0, "one thread per bin");
};

// Lanes of the wave that hold the same digit as this lane (among the lanes with valid == true).
__device__ inline uint64_t same_digit_lanes(uint32_t digit, uint32_t bits, bool valid) {
  uint64_t peers = __ballot(valid);
  for (uint32_t b = 0; b < bits; ++b) {
    const bool bit = (digit >> b) & 1u;
    const uint64_t vote = __ballot(bit);
    peers &= bit ? vote : ~vote;
  }
  return peers;
}

// key of occurrence i in pass 0: its row, or hwm if the occurrence was dropped
__device__ inline uint32_t first_key(const int32_t* rows, uint64_t i, uint32_t hwm) {
  const uint32_t r = (uint32_t)rows[i];
  return r < hwm ? r : hwm;
}

// An offset of the caller's, bounded to the n occurrences of the batch.
__device__ inline uint64_t bounded_offset(const int64_t* offsets, uint64_t b, uint64_t n) {
  const int64_t o = offsets[b];
  return o < 0 ? 0ull : ((uint64_t)o > n ? n : (uint64_t)o);
}

// The bag that holds occurrence `pos`: the last bag b with offsets[b] <= pos (offsets are non-decreasing
// and start at 0).  Run by a whole wave: 64 probes per step, four dependent steps for two million bags.
// Whatever the offsets hold, the answer is a bag index below n_bags and the loop ends.
__device__ inline uint32_t bag_holding(const int64_t* offsets, uint64_t n_bags, uint64_t n, uint64_t pos) {
  uint64_t lo = 0, hi = n_bags;
  while (hi - lo > 1) {
    const uint64_t step = (hi - lo + 63) / 64;
    const uint64_t p = lo + (uint64_t)(lane_id() + 1) * step;
    const bool ok = p < hi && bounded_offset(offsets, p, n) <= pos;
    const uint64_t m = __ballot(ok);
    const uint64_t k = m == ~0ull ? 64 : (uint64_t)(__ffsll((unsigned long long)~m) - 1);  // leading yes answers
    const uint64_t nlo = lo + k * step, nhi = lo + (k + 1) * step;
    lo = nlo;
    hi = nhi < hi ? nhi : hi;
  }
  return (uint32_t)lo;
}

// Pass 0 also notes, for the scatter kernel of the same pass, the bag that holds the unit's first
// occurrence (the last wave of the block searches while the others count).
template <uint32_t kBits, int kBlock, uint32_t kItems>
__global__ __launch_bounds__(kBlock) void sort_hist_kernel(const Control* __restrict__ ctl, uint32_t pass,
                                                               const int32_t* __restrict__ rows,
                                                               const uint2* __restrict__ src, uint64_t n,
                                                               uint64_t units, uint32_t* __restrict__ hist,
                                                               const int64_t* __restrict__ offsets, uint64_t n_bags,
                                                               uint32_t* __restrict__ unit_bag) {
  const SortPlan plan = make_sort_plan(ctl->hwm, kBits);
  if (pass >= plan.passes) return;
  using S = Shape<kBits, kBlock, kItems>;
  __shared__ uint32_t cnt[S::kBins];
  const uint64_t unit = blockIdx.x;
  const uint32_t shift = plan.shift(pass), nbins = 1u << plan.width(pass), mask = nbins - 1;
  for (uint32_t b = threadIdx.x; b < nbins; b += kBlock) cnt[b] = 0;
  __syncthreads();
  const uint64_t base = unit * kItems;
  if (pass > 0) n = ctl->scratch[kValidPairs];
  // every key of the thread is requested before the first one is counted (left to itself the compiler
  // keeps each load behind the LDS atomic before it: eight memory round trips in a row)
  constexpr uint32_t kPerThread = kItems / kBlock;
  uint32_t key[kPerThread];
#pragma unroll
  for (uint32_t r = 0; r < kPerThread; ++r) {
    const uint64_t i = base + (uint64_t)r * kBlock + threadIdx.x;
    key[r] = plan.hwm;
    if (i < n) key[r] = pass == 0 ? first_key(rows, i, plan.hwm) : src[i].x;
  }
#pragma unroll
  for (uint32_t r = 0; r < kPerThread; ++r)
    if (key[r] < plan.hwm) atomicAdd(&cnt[(key[r] >> shift) & mask], 1u);
  __syncthreads();
  for (uint32_t b = threadIdx.x; b < nbins; b += kBlock) hist[(uint64_t)b * units + unit] = cnt[b];
  if (pass == 0 && (threadIdx.x >> 6) == S::kWaves - 1) {  // wave-uniform; after the last barrier: nobody waits for it
    const uint32_t b0 = bag_holding(offsets, n_bags, n, unit * kItems);
    if (lane_id() == 0) unit_bag[unit] = b0;
  }
}

// exclusive scan of hist[bin * units + 0 .. units) in place; total of the bin to totals[bin].
// One block per bin; thread t owns a run of consecutive units (loaded at once, summed serially),
// the thread sums are scanned across the block, and the run is written back.
constexpr uint32_t kScanPerThread = 16;  // units per thread and round
template <uint32_t kBits>
__global__ __launch_bounds__(256) void sort_scan_kernel(const Control* __restrict__ ctl, uint32_t pass,
                                                        uint32_t* __restrict__ hist, uint64_t units,
                                                        uint32_t* __restrict__ totals) {
  const SortPlan plan = make_sort_plan(ctl->hwm, kBits);
  if (pass >= plan.passes || blockIdx.x >= (1u << plan.width(pass))) return;
  __shared__ uint32_t wave_sum[4];
  __shared__ uint32_t carry_s;
  uint32_t* row = hist + (uint64_t)blockIdx.x * units;
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (uint64_t t0 = 0; t0 < units; t0 += 256ull * kScanPerThread) {
    const uint64_t first = t0 + (uint64_t)threadIdx.x * kScanPerThread;
    uint32_t v[kScanPerThread];
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t j = 0; j < kScanPerThread; ++j) {
      v[j] = first + j < units ? row[first + j] : 0;
      sum += v[j];
    }
    uint32_t x = sum;  // inclusive wave scan of the thread sums
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t y = __shfl_up(x, d);
      if ((int)lane >= d) x += y;
    }
    if (lane == 63) wave_sum[wave] = x;
    __syncthreads();
    uint32_t run = carry_s + x - sum;
    for (uint32_t w = 0; w < wave; ++w) run += wave_sum[w];
#pragma unroll
    for (uint32_t j = 0; j < kScanPerThread; ++j) {
      if (first + j < units) row[first + j] = run;
      run += v[j];
    }
    __syncthreads();
    if (threadIdx.x == 255) carry_s = run;
    __syncthreads();
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry_s;
}

template <uint32_t kBits, int kBlock, uint32_t kItems>
__global__ __launch_bounds__(kBlock) void sort_scatter_kernel(Control* __restrict__ ctl, uint32_t pass,
                                                                  const int32_t* __restrict__ rows,
                                                                  const int64_t* __restrict__ offsets,
                                                                  uint64_t n_bags,
                                                                  const uint32_t* __restrict__ unit_bag,
                                                                  const uint2* __restrict__ src,
                                                                  uint64_t n, uint64_t units,
                                                                  const uint32_t* __restrict__ hist,
                                                                  const uint32_t* __restrict__ totals,
                                                                  uint2* __restrict__ dst) {
  const SortPlan plan = make_sort_plan(ctl->hwm, kBits);
  if (pass >= plan.passes) return;
  using S = Shape<kBits, kBlock, kItems>;
  __shared__ uint2 stage[kItems];          // the block's elements in sorted order
  __shared__ uint32_t lds[S::kWaves][S::kBins];   // per-wave digit counts, then local start offsets
  __shared__ uint32_t local_start[S::kBins];       // first position of a bin in `stage`
  __shared__ uint32_t global_start[S::kBins];      // where this block's part of a bin goes in dst
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint64_t unit = blockIdx.x;
  const uint32_t shift = plan.shift(pass), bits = plan.width(pass), nbins = 1u << bits, mask = nbins - 1;

  // 0. what step 3 needs from memory is asked for first: it arrives while the elements are loaded
  const bool bin_thread = threadIdx.x < S::kBins;
  const uint32_t bin = threadIdx.x;
  uint32_t tot = 0, before_me = 0;  // the bin in the whole batch / in the units before this one
  if (bin_thread && bin < nbins) {
    tot = totals[bin];
    before_me = hist[(uint64_t)bin * units + unit];
  }
  // 1. this wave's elements -> registers (independent, coalesced loads)
  if (pass > 0) n = ctl->scratch[kValidPairs];
  const uint64_t ubase = unit * kItems;
  const uint64_t base = ubase + (uint64_t)wave * S::kPerWave;
  uint2 kv[S::kRounds];
#pragma unroll
  for (uint32_t r = 0; r < S::kRounds; ++r) {
    const uint64_t i = base + (uint64_t)r * 64 + lane;
    kv[r] = make_uint2(0xFFFFFFFFu, 0u);
    if (i < n) kv[r] = pass == 0 ? make_uint2(first_key(rows, i, plan.hwm), 0u) : src[i];
    if (kv[r].x >= plan.hwm) kv[r].x = 0xFFFFFFFFu;  // dropped occurrence (or past the end): left out
  }
  for (uint32_t b = threadIdx.x; b < S::kBins; b += kBlock) {
#pragma unroll
    for (int w = 0; w < S::kWaves; ++w) lds[w][b] = 0;
  }
  if (pass == 0) {
    // The bag of every occurrence of the unit (the pooled gradient of bag b is the gradient of each of its
    // occurrences): the unit's bags are walked from the one that holds its first occurrence, and each
    // writes its number over its occurrences in an LDS array (the memory of `stage`, which is not needed
    // yet).  Whatever the offsets hold, every write stays inside the unit and every bag number that is
    // read is bounded to the bags of the batch.
    uint32_t* bag_here = reinterpret_cast<uint32_t*>(stage);
    const uint64_t uend = ubase + kItems < n ? ubase + kItems : n;
    constexpr uint32_t kBagsPerThread = 4;  // consecutive bags per thread and round (a unit holds ~500 bags of four IDs)
    // a thread stops at the first of its bags that starts at or after the end of the unit: offsets are
    // non-decreasing, so no later bag of its can reach into the unit (no barrier inside the loop)
    for (uint64_t b = (uint64_t)unit_bag[unit] + (uint64_t)threadIdx.x * kBagsPerThread; b < n_bags;
         b += (uint64_t)kBlock * kBagsPerThread) {
      uint64_t o[kBagsPerThread + 1];
#pragma unroll
      for (uint32_t q = 0; q <= kBagsPerThread; ++q) o[q] = b + q <= n_bags ? bounded_offset(offsets, b + q, n) : uend;
      if (o[0] >= uend) break;
#pragma unroll
      for (uint32_t q = 0; q < kBagsPerThread; ++q) {
        const uint64_t from = o[q] > ubase ? o[q] : ubase, to = o[q + 1] < uend ? o[q + 1] : uend;
        for (uint64_t i = from; i < to; ++i) bag_here[i - ubase] = (uint32_t)(b + q);
      }
    }
    __syncthreads();
    const uint32_t last_bag = (uint32_t)(n_bags - 1);  // (an occurrence outside every bag reads whatever the LDS held)
#pragma unroll
    for (uint32_t r = 0; r < S::kRounds; ++r) kv[r].y = min(bag_here[wave * S::kPerWave + r * 64 + lane], last_bag);
  }
  __syncthreads();
  // 2. per-wave digit counts
#pragma unroll
  for (uint32_t r = 0; r < S::kRounds; ++r) {
    if (kv[r].x != 0xFFFFFFFFu) atomicAdd(&lds[wave][(kv[r].x >> shift) & mask], 1u);
  }
  __syncthreads();
  // 3. thread b < S::kBins owns bin b: exclusive scans of the bin totals, once within the block
  //    (positions in `stage`) and once over all bins of the pass (start of the bin in dst)
  __shared__ uint32_t scan_sum[S::kScanWaves], scan_tot[S::kScanWaves];
  {
    uint32_t mine = 0;
    if (bin_thread && bin < nbins) {
#pragma unroll
      for (int w = 0; w < S::kWaves; ++w) mine += lds[w][bin];
    }
    uint32_t x = mine, y = tot;  // inclusive wave scans
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t xs = __shfl_up(x, d), ys = __shfl_up(y, d);
      if ((int)lane >= d) {
        x += xs;
        y += ys;
      }
    }
    if (bin_thread && lane == 63) {
      scan_sum[wave] = x;
      scan_tot[wave] = y;
    }
    __syncthreads();
    if (bin_thread) {
      uint32_t run = x - mine, run_tot = y - tot;  // first position of the bin in the block / in dst
      for (uint32_t w = 0; w < wave; ++w) {
        run += scan_sum[w];
        run_tot += scan_tot[w];
      }
      if (bin < nbins) {
        local_start[bin] = run;
        global_start[bin] = run_tot + before_me;
        uint32_t at = run;
#pragma unroll
        for (int w = 0; w < S::kWaves; ++w) {
          const uint32_t c = lds[w][bin];
          lds[w][bin] = at;
          at += c;
        }
      }
      if (pass == 0 && blockIdx.x == 0 && threadIdx.x == S::kBins - 1)
        ctl->scratch[kValidPairs] = run_tot + tot;  // pairs that remain
    }
  }
  __syncthreads();
  // 4. rank (stable) into `stage`, 64 elements at a time
  volatile uint32_t* off = lds[wave];
#pragma unroll
  for (uint32_t r = 0; r < S::kRounds; ++r) {
    const bool valid = kv[r].x != 0xFFFFFFFFu;
    const uint32_t digit = (kv[r].x >> shift) & mask;
    const uint64_t peers = same_digit_lanes(digit, bits, valid);
    if (valid) stage[off[digit] + (uint32_t)__popcll(peers & lanes_below())] = kv[r];
    __builtin_amdgcn_wave_barrier();
    if (valid && (peers & lanes_below()) == 0) off[digit] += (uint32_t)__popcll(peers);
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();
  // 5. out: neighbouring threads write neighbouring elements of a bin
  uint32_t total = 0;
#pragma unroll
  for (int w = 0; w < S::kScanWaves; ++w) total += scan_sum[w];
  for (uint32_t p = threadIdx.x; p < total; p += kBlock) {
    const uint2 e = stage[p];
    const uint32_t digit = (e.x >> shift) & mask;
    dst[global_start[digit] + (p - local_start[digit])] = e;
  }
}

template <uint32_t kBits, int kBlock, uint32_t kItems>
static void queue_sort_passes(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                              const int64_t* d_offsets, uint64_t n_bags, uint32_t passes, hipStream_t stream,
                              Profiler* prof) {
  const uint64_t units = sort_units(n, kItems);
  uint32_t* totals = ws.hist + (uint64_t)(1u << kBits) * units;
  const dim3 block(kBlock), grid((unsigned)units);
  for (uint32_t p = 0; p < passes; ++p) {
    const uint2* src = p % 2 == 0 ? ws.pair_a : ws.pair_b;
    uint2* dst = p % 2 == 0 ? ws.pair_b : ws.pair_a;
    MONO_LAUNCH(prof, K_SORT_HIST, stream, (sort_hist_kernel<kBits, kBlock, kItems>), grid, block, t.ctl, p, d_rows, src, n,
                units, ws.hist, d_offsets, n_bags, ws.unit_bag);
    MONO_LAUNCH(prof, K_SORT_SCAN, stream, sort_scan_kernel<kBits>, dim3(1u << kBits), dim3(256), t.ctl, p, ws.hist, units,
                totals);
    MONO_LAUNCH(prof, K_SORT_SCATTER, stream, (sort_scatter_kernel<kBits, kBlock, kItems>), grid, block, t.ctl, p, d_rows,
                d_offsets, n_bags, ws.unit_bag, src, n, units, ws.hist, totals, dst);
  }
}

hipError_t launch_sort_pairs(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                             const int64_t* d_offsets, uint64_t n_bags, uint32_t hwm_bound, uint32_t* launched,
                             uint32_t* max_bits, hipStream_t stream, Profiler* prof) {
  // the shape and as many passes as the largest high-water mark the table can have by now needs (the device
  // knows the real mark: passes beyond its plan return at once)
  const uint32_t bound = hwm_bound < (uint32_t)t.capacity ? hwm_bound : (uint32_t)t.capacity;
  const SortShape shape = sort_shape_for(bound);
  const SortPlan worst = make_sort_plan(bound, shape.max_bits);
  if (launched) *launched = worst.passes;
  if (max_bits) *max_bits = shape.max_bits;
  if (n == 0) return hipSuccess;
  if (shape.max_bits == kSortWide.max_bits)
    queue_sort_passes<kSortWide.max_bits, (int)kSortWide.block, kSortWide.items>(t, ws, d_rows, n, d_offsets, n_bags,
                                                                                 worst.passes, stream, prof);
  else
    queue_sort_passes<kSortNarrow.max_bits, (int)kSortNarrow.block, kSortNarrow.items>(t, ws, d_rows, n, d_offsets,
                                                                                       n_bags, worst.passes, stream, prof);
  return hipGetLastError();
}

}  // namespace mono
