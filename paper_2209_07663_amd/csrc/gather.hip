// gather_pool: embedding-row gather with per-bag sum pooling.
//
// A wave owns 64 consecutive bags.  First every lane loads the bounds and the first kIdsInRegs
// indices of ONE bag (coalesced: the bags of a wave are neighbours in `offsets` and in the index
// array).  Then the wave walks its bags in rounds: a group of lanes (dim/4 rounded up to a power of
// two, at most the whole wave) takes one bag per round, gets the bag's indices from the owner lane by
// shuffle, reads the rows (one coalesced access per row, kIdsInRegs of them in flight) and writes the
// pooled row once, in full lines.  Rows wider than 256 elements are walked in segments of 256 by the
// whole wave.  The few bags longer than kIdsInRegs read their remaining indices from memory.  A wave
// whose bags all hold at most two IDs (one-hot slots) issues four rounds of row reads together instead
// (81 -> 69 us on the workload with one ID per bag).
// Measured on MI355X the earlier one-group-per-bag kernel spent half its time
// on the dependent offset -> index -> row chain issued by eight times as many waves.
// Summation is in occurrence order, in fp32.
//
// Where the rows come from is a policy of the kernel:
//   TableRows       int32 row indices into one table (what lookup_or_insert hands out); an index
//                   outside the table counts as absent
//   QuotRemRows     int64 IDs into the two dense tables of the quotient-remainder decomposition
//                   (the paper's hashing baseline, section 3.1): E = E_r[ID mod 2^m] + E_q[ID div 2^m];
//                   an ID outside [0, 2^(2m)) counts as absent
#include "common.h"
#include "kernels.h"

namespace mono {

constexpr int kIdsInRegs = 8;

template <typename E>
__device__ inline float4 load4(const E* rows, uint64_t row, uint32_t dim, uint32_t col);

template <>
__device__ inline float4 load4<float>(const float* rows, uint64_t row, uint32_t dim, uint32_t col) {
  return *reinterpret_cast<const float4*>(rows + row * dim + col);
}
template <>
__device__ inline float4 load4<uint16_t>(const uint16_t* rows, uint64_t row, uint32_t dim, uint32_t col) {
  uint2 u = *reinterpret_cast<const uint2*>(rows + row * dim + col);
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
struct TableRows {
  using Id = int32_t;
  const E* rows;
  const int32_t* idx;
  uint32_t cap;
  __device__ Id none() const { return -1; }
  __device__ Id at(int64_t i) const { return idx[i]; }
  __device__ bool present(Id r) const { return (uint32_t)r < cap; }
  __device__ float4 fetch(Id r, uint32_t dim, uint32_t col) const { return load4<E>(rows, (uint32_t)r, dim, col); }
};

template <typename E>
struct QuotRemRows {
  using Id = int64_t;
  const E* rem;    // E_r: 2^m rows
  const E* quot;   // E_q: 2^m rows
  const int64_t* ids;
  uint32_t m;
  __device__ Id none() const { return -1; }
  __device__ Id at(int64_t i) const { return ids[i]; }
  __device__ bool present(Id id) const { return ((uint64_t)id >> (2 * m)) == 0; }
  __device__ float4 fetch(Id id, uint32_t dim, uint32_t col) const {
    float4 a = load4<E>(rem, (uint64_t)id & ((1ull << m) - 1), dim, col);
    add4(a, load4<E>(quot, (uint64_t)id >> m, dim, col));
    return a;
  }
};

template <typename Src>
__global__ __launch_bounds__(256) void gather_pool_kernel(Src src, const int64_t* __restrict__ offsets,
                                                          uint64_t n_bags, uint64_t n, uint32_t dim,
                                                          uint32_t group_log2, float* __restrict__ out) {
  using Id = typename Src::Id;
  const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const uint64_t bag_base = wave * 64;
  if (bag_base >= n_bags) return;  // wave-uniform
  const uint32_t lane = lane_id();
  // phase 1: lane <-> bag
  const bool mine = bag_base + lane < n_bags;
  // offsets and indices are the caller's: both are bounded (to the n indices, to the table's
  // rows) so that a malformed input gives zeros, not an access out of range
  int64_t s = mine ? offsets[bag_base + lane] : 0;
  int64_t e = mine ? offsets[bag_base + lane + 1] : 0;
  s = s < 0 ? 0 : s;
  e = e > (int64_t)n ? (int64_t)n : e;
  const int len = e > s ? (int)(e - s > 0x7FFFFFFF ? 0x7FFFFFFF : e - s) : 0;
  Id id[kIdsInRegs];
#pragma unroll
  for (int j = 0; j < kIdsInRegs; ++j) id[j] = j < len ? src.at(s + j) : src.none();
  // phase 2: group <-> bag, one bag per group and round
  const uint32_t group = 1u << group_log2, l = lane & (group - 1u), g = lane >> group_log2;
  const uint32_t bags_per_round = 64u >> group_log2;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  // Short bags (one or two IDs each, as in one-hot slots): a round keeps only one or two rows per
  // lane in flight, so four rounds are issued together instead.
  constexpr int kShort = 2, kRoundsTogether = kIdsInRegs / kShort;
  int longest = len;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) longest = max(longest, __shfl_xor(longest, d));
  if (longest <= kShort && dim <= 256) {  // wave-uniform
    const bool active = l * 4 < dim;
    for (uint32_t q0 = 0; q0 < group; q0 += kRoundsTogether) {
      float4 v[kRoundsTogether][kShort];
#pragma unroll
      for (int rr = 0; rr < kRoundsTogether; ++rr) {
        const int from = (int)((q0 + rr) * bags_per_round + g) & 63;
#pragma unroll
        for (int j = 0; j < kShort; ++j) {
          const Id r = __shfl(id[j], from);
          v[rr][j] = (q0 + rr < group && src.present(r) && active) ? src.fetch(r, dim, l * 4) : zero;
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
    const int from = (int)(q * bags_per_round + g);
    const int blen = __shfl(len, from);
    const int64_t bs = __shfl(s, from);
    Id rid[kIdsInRegs];
#pragma unroll
    for (int j = 0; j < kIdsInRegs; ++j) rid[j] = __shfl(id[j], from);
    const uint64_t bag = bag_base + (uint32_t)from;
    for (uint32_t col = l * 4; col < dim; col += 256) {  // one trip for rows of at most 256 elements
      float4 v[kIdsInRegs];
#pragma unroll
      for (int j = 0; j < kIdsInRegs; ++j) v[j] = src.present(rid[j]) ? src.fetch(rid[j], dim, col) : zero;
      float4 acc = zero;
#pragma unroll
      for (int j = 0; j < kIdsInRegs; ++j) add4(acc, v[j]);
      for (int j = kIdsInRegs; j < blen; ++j) {  // long bag: the rest of its indices straight from memory
        const Id r = src.at(bs + j);
        if (src.present(r)) add4(acc, src.fetch(r, dim, col));
      }
      if (bag < n_bags) *reinterpret_cast<float4*>(out + bag * dim + col) = acc;
    }
  }
}

static uint32_t lane_group_log2(uint32_t dim) {
  uint32_t g = 0;
  while (g < 6 && (4u << g) < dim) ++g;
  return g;
}

hipError_t launch_gather_pool(const TableView& t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets,
                              uint64_t n_bags, float* d_out, hipStream_t stream, Profiler* prof) {
  if (n_bags == 0) return hipSuccess;
  const uint32_t group_log2 = lane_group_log2(t.dim);
  const uint64_t waves = (n_bags + 63) / 64;
  const dim3 block(256), grid((unsigned)((waves + 3) / 4));
  if (t.bf16) {
    const TableRows<uint16_t> src{(const uint16_t*)t.rows, d_rows, (uint32_t)t.capacity};
    MONO_LAUNCH(prof, K_GATHER_POOL, stream, gather_pool_kernel<TableRows<uint16_t>>, grid, block, src, d_offsets, n_bags,
                n, t.dim, group_log2, d_out);
  } else {
    const TableRows<float> src{(const float*)t.rows, d_rows, (uint32_t)t.capacity};
    MONO_LAUNCH(prof, K_GATHER_POOL, stream, gather_pool_kernel<TableRows<float>>, grid, block, src, d_offsets, n_bags, n,
                t.dim, group_log2, d_out);
  }
  return hipGetLastError();
}

hipError_t launch_qr_gather_pool(const void* d_rem, const void* d_quot, uint32_t log2_rows, uint32_t dim, bool bf16,
                                 const int64_t* d_ids, uint64_t n, const int64_t* d_offsets, uint64_t n_bags,
                                 float* d_out, hipStream_t stream) {
  if (n_bags == 0) return hipSuccess;
  const uint32_t group_log2 = lane_group_log2(dim);
  const uint64_t waves = (n_bags + 63) / 64;
  const dim3 block(256), grid((unsigned)((waves + 3) / 4));
  if (bf16) {
    const QuotRemRows<uint16_t> src{(const uint16_t*)d_rem, (const uint16_t*)d_quot, d_ids, log2_rows};
    hipLaunchKernelGGL(gather_pool_kernel<QuotRemRows<uint16_t>>, grid, block, 0, stream, src, d_offsets, n_bags, n, dim,
                       group_log2, d_out);
  } else {
    const QuotRemRows<float> src{(const float*)d_rem, (const float*)d_quot, d_ids, log2_rows};
    hipLaunchKernelGGL(gather_pool_kernel<QuotRemRows<float>>, grid, block, 0, stream, src, d_offsets, n_bags, n, dim,
                       group_log2, d_out);
  }
  return hipGetLastError();
}

}  // namespace mono
