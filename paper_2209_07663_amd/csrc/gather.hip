// gather_pool: embedding-row gather with per-bag sum pooling.
//
// A group of lanes (dim/4 rounded up to a power of two) owns one bag; each lane keeps four
// consecutive elements of the pooled row in registers, so one row read is one coalesced
// dim*sizeof(E) access of the group and the pooled row is written once, in full lines.  Up to four
// row reads of a bag are in flight per lane.  Summation is in occurrence order, in fp32.
#include "common.h"
#include "kernels.h"

namespace mono {

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
                                                          uint32_t dim, uint32_t group_log2, float* __restrict__ out) {
  const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t bag = tid >> group_log2;
  const uint32_t l = (uint32_t)tid & ((1u << group_log2) - 1u);
  if (bag >= n_bags || l * 4 >= dim) return;
  const int64_t s = offsets[bag], e = offsets[bag + 1];
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const float4 zero = acc;
  for (int64_t i = s; i < e; i += 4) {
    int32_t r0 = idx[i];
    int32_t r1 = i + 1 < e ? idx[i + 1] : -1;
    int32_t r2 = i + 2 < e ? idx[i + 2] : -1;
    int32_t r3 = i + 3 < e ? idx[i + 3] : -1;
    float4 v0 = r0 >= 0 ? load4<E>(rows, (uint32_t)r0, dim, l) : zero;
    float4 v1 = r1 >= 0 ? load4<E>(rows, (uint32_t)r1, dim, l) : zero;
    float4 v2 = r2 >= 0 ? load4<E>(rows, (uint32_t)r2, dim, l) : zero;
    float4 v3 = r3 >= 0 ? load4<E>(rows, (uint32_t)r3, dim, l) : zero;
    add4(acc, v0);
    add4(acc, v1);
    add4(acc, v2);
    add4(acc, v3);
  }
  *reinterpret_cast<float4*>(out + bag * dim + l * 4) = acc;
}

hipError_t launch_gather_pool(const TableView& t, const int32_t* d_rows, const int64_t* d_offsets, uint64_t n_bags,
                              float* d_out, hipStream_t stream, Profiler* prof) {
  if (n_bags == 0) return hipSuccess;
  uint32_t group_log2 = 0;
  while ((4u << group_log2) < t.dim) ++group_log2;
  uint64_t threads = n_bags << group_log2;
  dim3 block(256), grid((unsigned)((threads + 255) / 256));
  if (t.bf16)
    MONO_LAUNCH(prof, K_GATHER_POOL, stream, gather_pool_kernel<uint16_t>, grid, block, (const uint16_t*)t.rows, d_rows, d_offsets,
                       n_bags, t.dim, group_log2, d_out);
  else
    MONO_LAUNCH(prof, K_GATHER_POOL, stream, gather_pool_kernel<float>, grid, block, (const float*)t.rows, d_rows, d_offsets,
                       n_bags, t.dim, group_log2, d_out);
  return hipGetLastError();
}

}  // namespace mono
