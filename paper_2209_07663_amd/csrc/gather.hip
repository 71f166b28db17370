// gather_pool: embedding-row gather with per-bag sum pooling.
//
// A wave owns 64 consecutive bags.  First every lane loads the bounds and the first kIdsInRegs row
// indices of ONE bag (coalesced: the bags of a wave are neighbours in `offsets` and in `rows`).
// Then the wave walks its bags in rounds: a group of lanes (dim/4 rounded up to a power of two)
// takes one bag per round, gets the bag's row indices from the owner lane by shuffle, reads the
// rows (one coalesced dim*sizeof(E) access per row, kIdsInRegs of them in flight) and writes the
// pooled row once, in full lines.  The few bags longer than kIdsInRegs read their remaining
// indices from memory.  A wave whose bags all hold at most two IDs (one-hot slots) issues four rounds
// of row reads together instead (81 -> 69 us on the workload with one ID per bag).
// Measured on MI355X the earlier one-group-per-bag kernel spent half its time
// on the dependent offset -> index -> row chain issued by eight times as many waves.
// Summation is in occurrence order, in fp32.
#include "common.h"
#include "kernels.h"

namespace mono {

constexpr int kIdsInRegs = 8;

template <typename E>
__device__ inline float4 load4(const E* rows, uint32_t row, uint32_t dim, uint32_t lane4);

template <>
__device__ inline float4 load4<float>(const float* rows, uint32_t row, uint32_t dim, uint32_t lane4) {
  return *reinterpret_cast<const float4*>(rows + (uint64_t)row * dim + lane4 * 4);
}
template <>
__device__ inline float4 load4<uint16_t>(const uint16_t* rows, uint32_t row, uint32_t dim, uint32_t lane4) {
  uint2 u = *reinterpret_cast<const uint2*>(rows + (uint64_t)row * dim + lane4 * 4);
  float4 v;
  v.x = __uint_as_float(u.x << 16);
  v.y = __uint_as_float(u.x & 0xFFFF0000u);
  v.z = __uint_as_float(u.y << 16);
  v.w = __uint_as_float(u.y & 0xFFFF0000u);
  return v;
}

__device__ inline void add4(float4& a, const float4& b) {
  a.x += b.x;
  a.y += b.y;
  a.z += b.z;
  a.w += b.w;
}

template <typename E>
__global__ __launch_bounds__(256) void gather_pool_kernel(const E* __restrict__ rows, const int32_t* __restrict__ idx,
                                                          const int64_t* __restrict__ offsets, uint64_t n_bags,
                                                          uint64_t n, uint32_t cap, uint32_t dim,
                                                          uint32_t group_log2, float* __restrict__ out) {
  const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const uint64_t bag_base = wave * 64;
  if (bag_base >= n_bags) return;  // wave-uniform
  const uint32_t lane = lane_id();
  // phase 1: lane <-> bag
  const bool mine = bag_base + lane < n_bags;
  // offsets and row indices are the caller's: both are bounded (to the n indices, to the table's
  // rows) so that a malformed input gives zeros, not an access out of range
  int64_t s = mine ? offsets[bag_base + lane] : 0;
  int64_t e = mine ? offsets[bag_base + lane + 1] : 0;
  s = s < 0 ? 0 : s;
  e = e > (int64_t)n ? (int64_t)n : e;
  const int len = e > s ? (int)(e - s > 0x7FFFFFFF ? 0x7FFFFFFF : e - s) : 0;
  int32_t id[kIdsInRegs];
#pragma unroll
  for (int j = 0; j < kIdsInRegs; ++j) id[j] = j < len ? idx[s + j] : -1;
  // phase 2: group <-> bag, one bag per group and round
  const uint32_t group = 1u << group_log2, l = lane & (group - 1u), g = lane >> group_log2;
  const uint32_t bags_per_round = 64u >> group_log2;
  const bool active = l * 4 < dim;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  // Short bags (one or two IDs each, as in one-hot slots): a round keeps only one or two rows per
  // lane in flight, so four rounds are issued together instead.
  constexpr int kShort = 2, kRoundsTogether = kIdsInRegs / kShort;
  int longest = len;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) longest = max(longest, __shfl_xor(longest, d));
  if (longest <= kShort) {  // wave-uniform
    for (uint32_t q0 = 0; q0 < group; q0 += kRoundsTogether) {
      float4 v[kRoundsTogether][kShort];
#pragma unroll
      for (int rr = 0; rr < kRoundsTogether; ++rr) {
        const int src = (int)((q0 + rr) * bags_per_round + g) & 63;
#pragma unroll
        for (int j = 0; j < kShort; ++j) {
          const int32_t r = __shfl(id[j], src);
          v[rr][j] = (q0 + rr < group && (uint32_t)r < cap && active) ? load4<E>(rows, (uint32_t)r, dim, l) : zero;
        }
      }
#pragma unroll
      for (int rr = 0; rr < kRoundsTogether; ++rr) {
        float4 acc = v[rr][0];
        add4(acc, v[rr][1]);
        const uint64_t bag = bag_base + (q0 + rr) * bags_per_round + g;
        if (q0 + rr < group && bag < n_bags && active) *reinterpret_cast<float4*>(out + bag * dim + l * 4) = acc;
      }
    }
    return;
  }
  for (uint32_t q = 0; q < group; ++q) {
    const int src = (int)(q * bags_per_round + g);
    const int blen = __shfl(len, src);
    const int64_t bs = __shfl(s, src);
    float4 v[kIdsInRegs];
#pragma unroll
    for (int j = 0; j < kIdsInRegs; ++j) {
      const int32_t r = __shfl(id[j], src);
      v[j] = ((uint32_t)r < cap && active) ? load4<E>(rows, (uint32_t)r, dim, l) : zero;
    }
    float4 acc = zero;
#pragma unroll
    for (int j = 0; j < kIdsInRegs; ++j) add4(acc, v[j]);
    for (int j = kIdsInRegs; j < blen; ++j) {  // long bag: the rest of its indices straight from memory
      const int32_t r = idx[bs + j];
      if ((uint32_t)r < cap && active) add4(acc, load4<E>(rows, (uint32_t)r, dim, l));
    }
    const uint64_t bag = bag_base + (uint32_t)src;
    if (bag < n_bags && active) *reinterpret_cast<float4*>(out + bag * dim + l * 4) = acc;
  }
}

hipError_t launch_gather_pool(const TableView& t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets,
                              uint64_t n_bags, float* d_out, hipStream_t stream, Profiler* prof) {
  if (n_bags == 0) return hipSuccess;
  uint32_t group_log2 = 0;
  while ((4u << group_log2) < t.dim) ++group_log2;
  const uint64_t waves = (n_bags + 63) / 64;
  const dim3 block(256), grid((unsigned)((waves + 3) / 4));
  if (t.bf16)
    MONO_LAUNCH(prof, K_GATHER_POOL, stream, gather_pool_kernel<uint16_t>, grid, block, (const uint16_t*)t.rows, d_rows,
                d_offsets, n_bags, n, (uint32_t)t.capacity, t.dim, group_log2, d_out);
  else
    MONO_LAUNCH(prof, K_GATHER_POOL, stream, gather_pool_kernel<float>, grid, block, (const float*)t.rows, d_rows,
                d_offsets, n_bags, n, (uint32_t)t.capacity, t.dim, group_log2, d_out);
  return hipGetLastError();
}

}  // namespace mono
