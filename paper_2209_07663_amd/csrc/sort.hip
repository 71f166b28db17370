// Stable LSD radix sort of (row index, bag) pairs, used to bring the occurrences of one embedding
// row together before the gradient reduction.
//
// Unit of work: one wave owns kSortItemsPerWave consecutive elements.  Per pass:
//   hist     per-unit digit histogram (LDS atomics), written bin-major: hist[bin * units + unit]
//   scan     one block per bin: exclusive scan along the units; bin totals to `totals`
//   scatter  each wave turns totals into bin bases (wave scan), adds its own row of the scanned
//            histogram, then ranks its elements 64 at a time by digit matching with ballots
//            (stable: rank = number of lower lanes with the same digit) and scatters them.
// Waves never wait for each other; no kernel spins.
#include "common.h"
#include "kernels.h"

namespace mono {

constexpr int kSortBlock = 256;                      // 4 independent waves
constexpr int kSortWaves = kSortBlock / 64;
constexpr uint32_t kSortRounds = kSortItemsPerWave / 64;

__device__ inline uint32_t load_key(const uint32_t* keys, uint64_t i, uint32_t clamp) {
  uint32_t k = keys[i];
  return k < clamp ? k : clamp;
}

__global__ __launch_bounds__(kSortBlock) void sort_hist_kernel(const uint32_t* __restrict__ keys, uint32_t clamp,
                                                               uint64_t n, uint64_t units, uint32_t shift,
                                                               uint32_t bits, uint32_t* __restrict__ hist) {
  __shared__ uint32_t lds[kSortWaves][kSortMaxBins];
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint64_t unit = (uint64_t)blockIdx.x * kSortWaves + wave;
  const uint32_t nbins = 1u << bits, mask = nbins - 1;
  uint32_t* cnt = lds[wave];
  for (uint32_t b = lane; b < nbins; b += 64) cnt[b] = 0;
  __builtin_amdgcn_wave_barrier();
  if (unit < units) {
    const uint64_t base = unit * kSortItemsPerWave;
#pragma unroll 4
    for (uint32_t r = 0; r < kSortRounds; ++r) {
      const uint64_t i = base + (uint64_t)r * 64 + lane;
      if (i < n) atomicAdd(&cnt[(load_key(keys, i, clamp) >> shift) & mask], 1u);
    }
    __builtin_amdgcn_wave_barrier();
    for (uint32_t b = lane; b < nbins; b += 64) hist[(uint64_t)b * units + unit] = cnt[b];
  }
}

// exclusive scan of hist[bin * units + 0 .. units) in place; total of the bin to totals[bin]
__global__ __launch_bounds__(256) void sort_scan_kernel(uint32_t* __restrict__ hist, uint64_t units,
                                                        uint32_t* __restrict__ totals) {
  __shared__ uint32_t wave_sum[4];
  __shared__ uint32_t carry_s;
  uint32_t* row = hist + (uint64_t)blockIdx.x * units;
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (uint64_t t0 = 0; t0 < units; t0 += 256) {
    const uint64_t i = t0 + threadIdx.x;
    const uint32_t v = i < units ? row[i] : 0;
    uint32_t x = v;  // inclusive wave scan
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      uint32_t y = __shfl_up(x, d);
      if ((int)lane >= d) x += y;
    }
    if (lane == 63) wave_sum[wave] = x;
    __syncthreads();
    uint32_t before = carry_s;
    for (uint32_t w = 0; w < wave; ++w) before += wave_sum[w];
    if (i < units) row[i] = before + x - v;
    __syncthreads();
    if (threadIdx.x == 255) carry_s = before + x;
    __syncthreads();
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry_s;
}

__global__ __launch_bounds__(kSortBlock) void sort_scatter_kernel(
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, uint32_t clamp, uint64_t n, uint64_t units,
    uint32_t shift, uint32_t bits, const uint32_t* __restrict__ hist, const uint32_t* __restrict__ totals,
    uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out) {
  __shared__ uint32_t lds[kSortWaves][kSortMaxBins];
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint64_t unit = (uint64_t)blockIdx.x * kSortWaves + wave;
  if (unit >= units) return;
  const uint32_t nbins = 1u << bits, mask = nbins - 1;
  volatile uint32_t* off = lds[wave];
  // bin bases: exclusive scan of the totals over the bins, `per` consecutive bins per lane
  {
    const uint32_t per = (nbins + 63) / 64;
    uint32_t local[kSortMaxBins / 64];
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t q = 0; q < kSortMaxBins / 64; ++q) {
      const uint32_t b = lane * per + q;
      local[q] = (q < per && b < nbins) ? totals[b] : 0;
      sum += local[q];
    }
    uint32_t x = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      uint32_t y = __shfl_up(x, d);
      if ((int)lane >= d) x += y;
    }
    uint32_t run = x - sum;
#pragma unroll
    for (uint32_t q = 0; q < kSortMaxBins / 64; ++q) {
      const uint32_t b = lane * per + q;
      if (q < per && b < nbins) {
        off[b] = run + hist[(uint64_t)b * units + unit];
        run += local[q];
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
  const uint64_t base = unit * kSortItemsPerWave;
#pragma unroll 2
  for (uint32_t r = 0; r < kSortRounds; ++r) {
    const uint64_t i = base + (uint64_t)r * 64 + lane;
    const bool valid = i < n;
    uint32_t k = 0, v = 0;
    if (valid) {
      k = load_key(keys, i, clamp);
      v = vals[i];
    }
    const uint32_t digit = (k >> shift) & mask;
    uint64_t peers = __ballot(valid);
    if (peers == 0) break;
    for (uint32_t b = 0; b < bits; ++b) {
      const bool bit = (digit >> b) & 1u;
      const uint64_t vote = __ballot(bit);
      peers &= bit ? vote : ~vote;
    }
    if (valid) {
      const uint32_t rank = __popcll(peers & lanes_below());
      const uint32_t dst = off[digit] + rank;
      keys_out[dst] = k;
      vals_out[dst] = v;
    }
    __builtin_amdgcn_wave_barrier();
    if (valid && (peers & lanes_below()) == 0) off[digit] += __popcll(peers);
    __builtin_amdgcn_wave_barrier();
  }
}

hipError_t launch_sort_pairs(const UpdateWorkspace& ws, const uint32_t* keys_in, uint32_t clamp, uint64_t n,
                             uint32_t bits, int* result_in_b, hipStream_t stream, Profiler* prof) {
  *result_in_b = 0;
  if (n == 0 || bits == 0) return hipSuccess;
  const uint64_t units = sort_units(n);
  const uint32_t passes = (bits + kSortMaxBits - 1) / kSortMaxBits;
  const uint32_t per = (bits + passes - 1) / passes;
  uint32_t* totals = ws.hist + (uint64_t)kSortMaxBins * sort_units(n);
  const uint32_t* src_k = keys_in ? keys_in : ws.key_a;
  const uint32_t* src_v = ws.val_a;
  uint32_t* dst_k = ws.key_b;
  uint32_t* dst_v = ws.val_b;
  dim3 block(kSortBlock), grid((unsigned)((units + kSortWaves - 1) / kSortWaves));
  uint32_t shift = 0;
  for (uint32_t p = 0; p < passes; ++p) {
    const uint32_t b = bits - shift < per ? bits - shift : per;
    const uint32_t cl = p == 0 ? clamp : 0xFFFFFFFFu;
    MONO_LAUNCH(prof, K_SORT_HIST, stream, sort_hist_kernel, grid, block, src_k, cl, n, units, shift, b, ws.hist);
    MONO_LAUNCH(prof, K_SORT_SCAN, stream, sort_scan_kernel, dim3(1u << b), dim3(256), ws.hist, units, totals);
    MONO_LAUNCH(prof, K_SORT_SCATTER, stream, sort_scatter_kernel, grid, block, src_k, src_v, cl, n, units, shift, b, ws.hist,
                       totals, dst_k, dst_v);
    shift += b;
    // ping-pong; after the first pass the source is always one of the workspace pairs
    if (p % 2 == 0) {
      src_k = ws.key_b; src_v = ws.val_b; dst_k = ws.key_a; dst_v = ws.val_a;
    } else {
      src_k = ws.key_a; src_v = ws.val_a; dst_k = ws.key_b; dst_v = ws.val_b;
    }
    *result_in_b = p % 2 == 0 ? 1 : 0;
  }
  return hipGetLastError();
}

}  // namespace mono
