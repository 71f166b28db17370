// apply_grad_adagrad: duplicate-ID gradient scatter-reduce + row-wise Adagrad.
//
//   expand       bag index of every occurrence (the pooled gradient of bag b is the gradient of each
//                of its occurrences)
//   sort         stable radix sort of (row, bag) by row: the occurrences of a row become one run;
//                dropped occurrences (row -1) sort behind everything under the key `capacity`
//   seg_reduce   the sorted sequence is cut into chunks of kChunk; a lane group (dim/4 lanes, four
//                elements each) walks one chunk, summing grad[bag] along each run.  A run that lies
//                inside the chunk is complete: Adagrad is applied at once.  A run that crosses a
//                chunk border leaves a partial sum
//   combine      one wave per run that crosses borders: adds its partials (tree over lane groups)
//                and applies Adagrad.  Long runs (hot IDs) are thus reduced pairwise, not serially.
// Everything is deterministic: no floating-point atomics.
#include "common.h"
#include "kernels.h"

namespace mono {

constexpr uint32_t kHeadFlag = 0x80000000u;  // partial belongs to a run that starts in its chunk

__global__ __launch_bounds__(256) void expand_bags_kernel(const int64_t* __restrict__ offsets, uint64_t n_bags,
                                                          uint32_t* __restrict__ bag_of) {
  const uint64_t b = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= n_bags) return;
  const int64_t s = offsets[b], e = offsets[b + 1];
  for (int64_t i = s; i < e; ++i) bag_of[i] = (uint32_t)b;
}

template <typename E>
__device__ inline float4 load_row4(const E* rows, uint32_t row, uint32_t dim, uint32_t l);
template <>
__device__ inline float4 load_row4<float>(const float* rows, uint32_t row, uint32_t dim, uint32_t l) {
  return *reinterpret_cast<const float4*>(rows + (uint64_t)row * dim + l * 4);
}
template <>
__device__ inline float4 load_row4<uint16_t>(const uint16_t* rows, uint32_t row, uint32_t dim, uint32_t l) {
  uint2 u = *reinterpret_cast<const uint2*>(rows + (uint64_t)row * dim + l * 4);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xFFFF0000u));
}
template <typename E>
__device__ inline void store_row4(E* rows, uint32_t row, uint32_t dim, uint32_t l, float4 v);
template <>
__device__ inline void store_row4<float>(float* rows, uint32_t row, uint32_t dim, uint32_t l, float4 v) {
  *reinterpret_cast<float4*>(rows + (uint64_t)row * dim + l * 4) = v;
}
template <>
__device__ inline void store_row4<uint16_t>(uint16_t* rows, uint32_t row, uint32_t dim, uint32_t l, float4 v) {
  uint2 u;
  u.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
  u.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
  *reinterpret_cast<uint2*>(rows + (uint64_t)row * dim + l * 4) = u;
}

// Row-wise Adagrad on one row by one lane group; g = this lane's four gradient elements (zero in
// lanes beyond dim).  acc += mean_j g_j^2; w_j -= lr * g_j / (sqrt(acc) + eps).
template <typename E>
__device__ inline void adagrad_row(const TableView& t, uint32_t row, float4 g, bool active, uint32_t l,
                                   uint32_t group, float lr, float eps) {
  float ss = g.x * g.x + g.y * g.y + g.z * g.z + g.w * g.w;
  for (uint32_t d = 1; d < group; d <<= 1) ss += __shfl_xor(ss, (int)d);
  const float acc = t.acc[row] + ss / (float)t.dim;
  const float denom = sqrtf(acc) + eps;
  if (active) {
    E* rows = reinterpret_cast<E*>(t.rows);
    float4 w = load_row4<E>(rows, row, t.dim, l);
    w.x -= lr * g.x / denom;
    w.y -= lr * g.y / denom;
    w.z -= lr * g.z / denom;
    w.w -= lr * g.w / denom;
    store_row4<E>(rows, row, t.dim, l, w);
  }
  if (l == 0) t.acc[row] = acc;
}

__device__ inline void acc4(float4& a, const float4& b) {
  a.x += b.x;
  a.y += b.y;
  a.z += b.z;
  a.w += b.w;
}

template <typename E>
__global__ __launch_bounds__(256) void seg_reduce_kernel(TableView t, const uint32_t* __restrict__ sk,
                                                         const uint32_t* __restrict__ sv, uint64_t n,
                                                         const float* __restrict__ grad, float lr, float eps,
                                                         float* __restrict__ part, uint32_t* __restrict__ part_row,
                                                         uint32_t group_log2) {
  const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t c = tid >> group_log2;
  const uint32_t group = 1u << group_log2;
  const uint32_t l = (uint32_t)tid & (group - 1u);
  const uint64_t n_chunks = (n + kChunk - 1) / kChunk;
  if (c >= n_chunks) return;
  const bool active = l * 4 < t.dim;
  const uint32_t cap = (uint32_t)t.capacity;
  const uint64_t cs = c * kChunk, ce = cs + kChunk < n ? cs + kChunk : n;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  const float4* g4 = reinterpret_cast<const float4*>(grad);
  const uint32_t dim4 = t.dim >> 2;

  uint32_t a_row = kNoRow, b_row = kNoRow;
  uint32_t run = sk[cs];
  bool head_in = cs == 0 || sk[cs - 1] != run;
  float4 sum = zero;

  auto flush = [&](bool tail_in) {
    if (run >= cap) return;  // dropped occurrences
    if (head_in && tail_in) {
      adagrad_row<E>(t, run, sum, active, l, group, lr, eps);
    } else if (tail_in) {  // started in an earlier chunk, ends here
      a_row = run;
      if (active) *reinterpret_cast<float4*>(part + (2 * c) * t.dim + l * 4) = sum;
    } else {  // continues in the next chunk
      b_row = run | (head_in ? kHeadFlag : 0u);
      if (active) *reinterpret_cast<float4*>(part + (2 * c + 1) * t.dim + l * 4) = sum;
    }
  };

  for (uint64_t i = cs; i < ce; i += 4) {
    // four occurrences in flight
    uint32_t r[4], bg[4];
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool ok = i + u < ce;
      r[u] = ok ? sk[i + u] : kNoRow;
      bg[u] = ok ? sv[i + u] : 0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = (r[u] < cap && active) ? g4[(uint64_t)bg[u] * dim4 + l] : zero;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (i + u >= ce) break;
      if (r[u] != run) {
        flush(true);
        run = r[u];
        head_in = true;
        sum = zero;
      }
      acc4(sum, v[u]);
    }
  }
  flush(!(ce < n && sk[ce] == run));
  if (l == 0) {
    part_row[2 * c] = a_row;
    part_row[2 * c + 1] = b_row;
  }
}

// One wave per chunk; only the wave whose chunk holds the head of a border-crossing run works.
template <typename E>
__global__ __launch_bounds__(256) void combine_kernel(TableView t, uint64_t n_chunks, const float* __restrict__ part,
                                                      const uint32_t* __restrict__ part_row, float lr, float eps,
                                                      uint32_t group_log2) {
  const uint64_t c = (uint64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (c >= n_chunks) return;
  const uint32_t head = part_row[2 * c + 1];
  if (head == kNoRow || !(head & kHeadFlag)) return;
  const uint32_t row = head & ~kHeadFlag;
  const uint32_t lane = lane_id();
  // number of chunks after c that lie entirely inside the run
  uint64_t mid = 0;
  for (;;) {
    const uint64_t cc = c + 1 + mid + lane;
    const bool is_mid = cc < n_chunks && part_row[2 * cc + 1] == row;
    const uint64_t m = __ballot(is_mid);
    if (m == ~0ull) {
      mid += 64;
      continue;
    }
    mid += (uint64_t)(__ffsll((unsigned long long)~m) - 1);
    break;
  }
  const uint64_t tail = c + 1 + mid;
  const bool has_tail = tail < n_chunks && part_row[2 * tail] == row;
  const uint64_t pieces = 1 + mid + (has_tail ? 1 : 0);
  const uint32_t group = 1u << group_log2, l = lane & (group - 1u), gi = lane >> group_log2, ng = 64u >> group_log2;
  const bool active = l * 4 < t.dim;
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  if (active)
    for (uint64_t p = gi; p < pieces; p += ng) {
      const uint64_t slot = p <= mid ? 2 * (c + p) + 1 : 2 * tail;
      acc4(sum, *reinterpret_cast<const float4*>(part + slot * t.dim + l * 4));
    }
  for (uint32_t d = group; d < 64; d <<= 1) {
    sum.x += __shfl_xor(sum.x, (int)d);
    sum.y += __shfl_xor(sum.y, (int)d);
    sum.z += __shfl_xor(sum.z, (int)d);
    sum.w += __shfl_xor(sum.w, (int)d);
  }
  if (gi == 0) adagrad_row<E>(t, row, sum, active, l, group, lr, eps);
}

hipError_t launch_apply_grad_adagrad(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                                     const int64_t* d_offsets, uint64_t n_bags, const float* d_grad, float lr, float eps,
                                     hipStream_t stream, Profiler* prof) {
  if (n == 0 || n_bags == 0) return hipSuccess;
  MONO_LAUNCH(prof, K_EXPAND_BAGS, stream, expand_bags_kernel, dim3((unsigned)((n_bags + 255) / 256)), dim3(256), d_offsets, n_bags,
                     ws.val_a);
  uint32_t bits = 1;  // keys are rows in [0, capacity) plus `capacity` itself for dropped occurrences
  while ((1ull << bits) <= t.capacity) ++bits;
  int in_b = 0;
  hipError_t e = launch_sort_pairs(ws, reinterpret_cast<const uint32_t*>(d_rows), (uint32_t)t.capacity, n, bits, &in_b,
                                   stream, prof);
  if (e != hipSuccess) return e;
  const uint32_t* sk = in_b ? ws.key_b : ws.key_a;
  const uint32_t* sv = in_b ? ws.val_b : ws.val_a;
  uint32_t group_log2 = 0;
  while ((4u << group_log2) < t.dim) ++group_log2;
  const uint64_t n_chunks = reduce_chunks(n);
  const uint64_t threads = n_chunks << group_log2;
  const dim3 block(256), grid((unsigned)((threads + 255) / 256)), cgrid((unsigned)((n_chunks + 3) / 4));
  if (t.bf16) {
    MONO_LAUNCH(prof, K_SEG_REDUCE, stream, seg_reduce_kernel<uint16_t>, grid, block, t, sk, sv, n, d_grad, lr, eps, ws.part,
                       ws.part_row, group_log2);
    MONO_LAUNCH(prof, K_COMBINE, stream, combine_kernel<uint16_t>, cgrid, block, t, n_chunks, ws.part, ws.part_row, lr, eps,
                       group_log2);
  } else {
    MONO_LAUNCH(prof, K_SEG_REDUCE, stream, seg_reduce_kernel<float>, grid, block, t, sk, sv, n, d_grad, lr, eps, ws.part,
                       ws.part_row, group_log2);
    MONO_LAUNCH(prof, K_COMBINE, stream, combine_kernel<float>, cgrid, block, t, n_chunks, ws.part, ws.part_row, lr, eps,
                       group_log2);
  }
  return hipGetLastError();
}

}  // namespace mono
