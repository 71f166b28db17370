// apply_grad_adagrad: duplicate-ID gradient scatter-reduce + row-wise Adagrad.
//
//   expand       bag index of every occurrence (the pooled gradient of bag b is the gradient of each
//                of its occurrences)
//   sort         stable radix sort of (row, bag) by row: the occurrences of a row become one run;
//                dropped occurrences (row -1) sort behind everything
//   seg_reduce   the sorted sequence is cut into chunks of kChunk; a lane group (dim/4 lanes, four
//                elements each) walks one chunk, summing grad[bag] along each run.  A run that lies
//                inside the chunk is complete: Adagrad is applied at once.  A run that crosses a
//                chunk border leaves a partial sum in LDS; the groups of a block then join the
//                partials of runs that stay inside the block's tile (Adagrad again) and only runs
//                that cross a BLOCK border leave partials in global memory (at most two per block)
//   combine      one block per run that crosses block borders: adds its partials (lane groups in
//                parallel, then across groups) and applies Adagrad
// A hot ID with 10^5..10^6 occurrences is thus reduced as chunk sums -> tile sums -> total, never
// serially, and everything is deterministic: no floating-point atomics.
//
// Partial-slot convention (same at chunk level in LDS and at tile level in global memory): unit u
// has slot A = 2u ("run that started before this unit and ends inside it") and slot B = 2u + 1
// ("run that continues past the end of this unit"; flag kHeadFlag if it also starts inside it).
#include "common.h"
#include "kernels.h"

namespace mono {

constexpr uint32_t kHeadFlag = 0x80000000u;

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
  const uint2 u = *reinterpret_cast<const uint2*>(rows + (uint64_t)row * dim + l * 4);
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
__global__ __launch_bounds__(256) void seg_reduce_kernel(TableView t, const uint2* __restrict__ pair_a,
                                                         const uint2* __restrict__ pair_b, uint64_t n,
                                                         const float* __restrict__ grad, float lr, float eps,
                                                         float* __restrict__ part, uint32_t* __restrict__ part_row,
                                                         uint32_t group_log2) {
  extern __shared__ float4 s_mem[];  // [2 * groups_per_block][dim / 4] vectors, then the slot rows
  const SortPlan plan = make_sort_plan(t.ctl->hwm);
  const uint2* __restrict__ sp = plan.passes % 2 ? pair_b : pair_a;  // where the sort left its result
  const uint32_t hwm = plan.hwm;
  const uint32_t group = 1u << group_log2, gpb = 256u >> group_log2;  // groups (= chunks) per block
  const uint32_t g = threadIdx.x >> group_log2, l = threadIdx.x & (group - 1u);
  const uint32_t dim4 = t.dim >> 2;
  float4* s_vec = s_mem;
  uint32_t* s_row = reinterpret_cast<uint32_t*>(s_mem + 2 * gpb * dim4);
  const uint64_t n_chunks = (n + kChunk - 1) / kChunk;
  const uint64_t c0 = (uint64_t)blockIdx.x * gpb;  // first chunk of this block's tile
  const uint64_t c = c0 + g;
  const uint32_t chunks_here = (uint32_t)(n_chunks - c0 < gpb ? n_chunks - c0 : gpb);
  const bool active = l < dim4;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  const float4* g4 = reinterpret_cast<const float4*>(grad);

  // ---- phase 1: every group reduces the runs of its chunk -------------------------------------
  uint32_t a_row = kNoRow, b_row = kNoRow;
  if (c < n_chunks) {
    const uint64_t cs = c * kChunk, ce = cs + kChunk < n ? cs + kChunk : n;
    uint32_t run = sp[cs].x;
    bool head_in = cs == 0 || sp[cs - 1].x != run;
    float4 sum = zero;
    auto flush = [&](bool tail_in) {
      if (run >= hwm) return;  // dropped occurrences
      if (head_in && tail_in) {
        adagrad_row<E>(t, run, sum, active, l, group, lr, eps);
      } else if (tail_in) {  // started in an earlier chunk, ends here
        a_row = run;
        if (active) s_vec[(2 * g) * dim4 + l] = sum;
      } else {  // continues in the next chunk
        b_row = run | (head_in ? kHeadFlag : 0u);
        if (active) s_vec[(2 * g + 1) * dim4 + l] = sum;
      }
    };
    for (uint64_t i = cs; i < ce; i += 4) {  // four occurrences in flight
      uint2 kv[4];
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) kv[u] = i + u < ce ? sp[i + u] : make_uint2(kNoRow, 0u);
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = (kv[u].x < hwm && active) ? g4[(uint64_t)kv[u].y * dim4 + l] : zero;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (i + u >= ce) break;
        if (kv[u].x != run) {
          flush(true);
          run = kv[u].x;
          head_in = true;
          sum = zero;
        }
        acc4(sum, v[u]);
      }
    }
    flush(!(ce < n && sp[ce].x == run));
  }
  if (l == 0) {
    s_row[2 * g] = a_row;
    s_row[2 * g + 1] = b_row;
  }
  if (threadIdx.x == 0) {
    part_row[2 * (uint64_t)blockIdx.x] = kNoRow;
    part_row[2 * (uint64_t)blockIdx.x + 1] = kNoRow;
  }
  __syncthreads();

  // ---- phase 2: join the chunk partials of runs inside this tile -------------------------------
  // The group holding the first piece of a run within the tile walks the following chunks.
  const bool walker = c < n_chunks && b_row != kNoRow && ((b_row & kHeadFlag) || g == 0);
  if (walker) {
    const uint32_t row = b_row & ~kHeadFlag;
    const bool head_in_tile = (b_row & kHeadFlag) != 0;
    float4 sum = active ? s_vec[(2 * g + 1) * dim4 + l] : zero;
    uint32_t cc = g + 1;
    bool tail = false;
    while (cc < chunks_here) {
      if (s_row[2 * cc] == row) {  // the run ends in chunk cc
        if (active) acc4(sum, s_vec[(2 * cc) * dim4 + l]);
        tail = true;
        break;
      }
      if (s_row[2 * cc + 1] != row) break;  // (cannot happen for consistent slots)
      if (active) acc4(sum, s_vec[(2 * cc + 1) * dim4 + l]);
      ++cc;
    }
    if (tail && head_in_tile) {
      adagrad_row<E>(t, row, sum, active, l, group, lr, eps);
    } else {
      const uint64_t slot = 2 * (uint64_t)blockIdx.x + (tail ? 0 : 1);
      if (active) *reinterpret_cast<float4*>(part + slot * t.dim + l * 4) = sum;
      if (l == 0) part_row[slot] = tail ? row : (row | (head_in_tile ? kHeadFlag : 0u));
    }
  }
  // a run that entered the tile from before and ends in chunk 0 is the tile's A partial as it stands
  if (g == 0 && c < n_chunks && a_row != kNoRow) {
    if (active) *reinterpret_cast<float4*>(part + (2 * (uint64_t)blockIdx.x) * t.dim + l * 4) = s_vec[l];
    if (l == 0) part_row[2 * (uint64_t)blockIdx.x] = a_row;
  }
}

// One block per tile; only the block whose tile holds the head of a border-crossing run works.
template <typename E>
__global__ __launch_bounds__(256) void combine_kernel(TableView t, uint64_t n_tiles, const float* __restrict__ part,
                                                      const uint32_t* __restrict__ part_row, float lr, float eps,
                                                      uint32_t group_log2) {
  extern __shared__ float4 s_mem[];  // [groups_per_block][dim / 4]
  const uint64_t c = blockIdx.x;
  const uint32_t head = part_row[2 * c + 1];
  if (head == kNoRow || !(head & kHeadFlag)) return;  // block-uniform
  const uint32_t row = head & ~kHeadFlag;
  // number of tiles after c that lie entirely inside the run
  uint64_t mid = 0;
  for (;;) {
    const uint64_t cc = c + 1 + mid + (threadIdx.x & 63);
    const bool is_mid = cc < n_tiles && part_row[2 * cc + 1] == row;
    const uint64_t m = __ballot(is_mid);
    if (m == ~0ull) {
      mid += 64;
      continue;
    }
    mid += (uint64_t)(__ffsll((unsigned long long)~m) - 1);
    break;
  }
  const uint64_t tail = c + 1 + mid;
  const bool has_tail = tail < n_tiles && part_row[2 * tail] == row;
  const uint64_t pieces = 1 + mid + (has_tail ? 1 : 0);
  const uint32_t group = 1u << group_log2, gpb = 256u >> group_log2;
  const uint32_t g = threadIdx.x >> group_log2, l = threadIdx.x & (group - 1u);
  const uint32_t dim4 = t.dim >> 2;
  const bool active = l < dim4;
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  if (active)
    for (uint64_t p = g; p < pieces; p += gpb) {
      const uint64_t slot = p <= mid ? 2 * (c + p) + 1 : 2 * tail;
      acc4(sum, *reinterpret_cast<const float4*>(part + slot * t.dim + l * 4));
    }
  if (active) s_mem[g * dim4 + l] = sum;
  __syncthreads();
  if (g == 0) {
    float4 total = make_float4(0.f, 0.f, 0.f, 0.f);
    const uint32_t used = pieces < gpb ? (uint32_t)pieces : gpb;
    if (active)
      for (uint32_t q = 0; q < used; ++q) acc4(total, s_mem[q * dim4 + l]);
    adagrad_row<E>(t, row, total, active, l, group, lr, eps);
  }
}

hipError_t launch_apply_grad_adagrad(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                                     const int64_t* d_offsets, uint64_t n_bags, const float* d_grad, float lr, float eps,
                                     hipStream_t stream, Profiler* prof) {
  if (n == 0 || n_bags == 0) return hipSuccess;
  MONO_LAUNCH(prof, K_EXPAND_BAGS, stream, expand_bags_kernel, dim3((unsigned)((n_bags + 255) / 256)), dim3(256),
              d_offsets, n_bags, ws.bag_of);
  hipError_t e = launch_sort_pairs(t, ws, d_rows, n, stream, prof);
  if (e != hipSuccess) return e;
  uint32_t group_log2 = 0;
  while ((4u << group_log2) < t.dim) ++group_log2;
  const uint32_t gpb = 256u >> group_log2;
  const uint64_t n_tiles = (reduce_chunks(n) + gpb - 1) / gpb;
  const dim3 block(256), grid((unsigned)n_tiles);
  const size_t lds_reduce = 2 * gpb * (t.dim / 4) * sizeof(float4) + 2 * gpb * sizeof(uint32_t);
  const size_t lds_combine = gpb * (t.dim / 4) * sizeof(float4);
  if (t.bf16) {
    MONO_LAUNCH_SMEM(prof, K_SEG_REDUCE, stream, seg_reduce_kernel<uint16_t>, grid, block, lds_reduce, t, ws.pair_a,
                     ws.pair_b, n, d_grad, lr, eps, ws.part, ws.part_row, group_log2);
    MONO_LAUNCH_SMEM(prof, K_COMBINE, stream, combine_kernel<uint16_t>, grid, block, lds_combine, t, n_tiles, ws.part,
                     ws.part_row, lr, eps, group_log2);
  } else {
    MONO_LAUNCH_SMEM(prof, K_SEG_REDUCE, stream, seg_reduce_kernel<float>, grid, block, lds_reduce, t, ws.pair_a,
                     ws.pair_b, n, d_grad, lr, eps, ws.part, ws.part_row, group_log2);
    MONO_LAUNCH_SMEM(prof, K_COMBINE, stream, combine_kernel<float>, grid, block, lds_combine, t, n_tiles, ws.part,
                     ws.part_row, lr, eps, group_log2);
  }
  return hipGetLastError();
}

}  // namespace mono
