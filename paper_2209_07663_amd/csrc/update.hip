// apply_grad_adagrad: duplicate-ID gradient scatter-reduce + row-wise Adagrad.
//
//   sort         stable radix sort of (row, bag) by row: the occurrences of a row become one run (the
//                pooled gradient of bag b is the gradient of each of its occurrences; the first pass
//                finds the bag of every occurrence from the offsets); dropped occurrences (row -1) are
//                left out
//   seg_reduce   the sorted sequence is cut into chunks of 16 pairs per lane of a lane group (dim/4
//                lanes, four elements each); the group loads its chunk's pairs at once, then walks
//                them with eight gradient rows in flight, summing grad[bag] along each run.  A run that lies
//                inside the chunk is complete: Adagrad is applied at once.  A run that crosses a
//                chunk border leaves a partial sum in LDS; the groups of a block then join the
//                partials of runs that stay inside the block's tile (Adagrad again) and only runs
//                that cross a BLOCK border leave partials in global memory (at most two per block)
//   combine      one block per run that crosses block borders: adds its partials (lane groups in
//                parallel, then across groups) and applies Adagrad
// A hot ID with 10^5..10^6 occurrences is thus reduced as chunk sums -> tile sums -> total, never
// serially, and everything is deterministic: no floating-point atomics.
// The store that writes a row's new accumulator also carries the number of the current
// synchronisation window: that is the row's "touched" mark (paper section 2.2.3), at no extra cost.
//
// Partial-slot convention (same at chunk level in LDS and at tile level in global memory): unit u
// has slot A = 2u ("run that started before this unit and ends inside it") and slot B = 2u + 1
// ("run that continues past the end of this unit"; flag kHeadFlag if it also starts inside it).
#include "common.h"
#include "kernels.h"

namespace mono {

constexpr uint32_t kHeadFlag = 0x80000000u;

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

// lr / (sqrt(acc) + eps) with the hardware square root and reciprocal (1 ulp each: the update is
// compared at 1e-5, and this runs once per distinct row inside the serial walk of seg_reduce)
__device__ inline float step_scale(float acc, float lr, float eps) {
  return lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(acc) + eps);
}

// A lane's share of a row: SEG pieces of four elements, piece q at elements (q * 64 + l) * 4.  Rows of
// at most 256 elements have one piece per lane (SEG = 1, lane groups of up to 64 lanes); wider rows
// (512, 768, 1024 elements) are held by the whole wave with SEG = 2, 3, 4.
template <int SEG>
struct RowVec {
  float4 v[SEG];
  __device__ inline void zero() {
#pragma unroll
    for (int q = 0; q < SEG; ++q) v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ inline void add(const RowVec& o) {
#pragma unroll
    for (int q = 0; q < SEG; ++q) {
      v[q].x += o.v[q].x;
      v[q].y += o.v[q].y;
      v[q].z += o.v[q].z;
      v[q].w += o.v[q].w;
    }
  }
  __device__ inline float sum_sq() const {
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < SEG; ++q) ss += v[q].x * v[q].x + v[q].y * v[q].y + v[q].z * v[q].z + v[q].w * v[q].w;
    return ss;
  }
};

// piece q of a vector of dim4 float4 (dim4 = dim / 4) held by lane l; `p` points at the vector
template <int SEG>
__device__ inline RowVec<SEG> load_vec(const float4* p, uint32_t l, bool active) {
  RowVec<SEG> r;
#pragma unroll
  for (int q = 0; q < SEG; ++q) r.v[q] = active ? p[q * 64 + l] : make_float4(0.f, 0.f, 0.f, 0.f);
  return r;
}
template <int SEG>
__device__ inline void store_vec(float4* p, uint32_t l, bool active, const RowVec<SEG>& r) {
#pragma unroll
  for (int q = 0; q < SEG; ++q)
    if (active) p[q * 64 + l] = r.v[q];
}
template <typename E, int SEG>
__device__ inline RowVec<SEG> load_row(const E* rows, uint32_t row, uint32_t dim, uint32_t l, bool active) {
  RowVec<SEG> r;
#pragma unroll
  for (int q = 0; q < SEG; ++q)
    r.v[q] = active ? load_row4<E>(rows, row, dim, q * 64 + l) : make_float4(0.f, 0.f, 0.f, 0.f);
  return r;
}

// w -= scale * g on the lane's share of row `row`
template <typename E, int SEG>
__device__ inline void update_row(E* rows, uint32_t row, uint32_t dim, uint32_t l, const RowVec<SEG>& w,
                                  const RowVec<SEG>& g, float scale) {
#pragma unroll
  for (int q = 0; q < SEG; ++q) {
    float4 nw = w.v[q];
    nw.x = fmaf(-scale, g.v[q].x, nw.x);
    nw.y = fmaf(-scale, g.v[q].y, nw.y);
    nw.z = fmaf(-scale, g.v[q].z, nw.z);
    nw.w = fmaf(-scale, g.v[q].w, nw.w);
    store_row4<E>(rows, row, dim, q * 64 + l, nw);
  }
}

// Row-wise Adagrad on one row by one lane group; g = this lane's share of the gradient (zero in
// lanes beyond dim).  acc += mean_j g_j^2; w_j -= lr * g_j / (sqrt(acc) + eps).
template <typename E, int SEG>
__device__ inline void adagrad_row(const TableView& t, uint32_t row, const RowVec<SEG>& g, bool active, uint32_t l,
                                   uint32_t group, float lr, float eps) {
  float ss = g.sum_sq();
  for (uint32_t d = 1; d < group; d <<= 1) ss += __shfl_xor(ss, (int)d);
  const float acc = t.state[row].acc + ss / (float)t.dim;
  const float scale = step_scale(acc, lr, eps);
  if (active) {
    E* rows = reinterpret_cast<E*>(t.rows);
    const RowVec<SEG> w = load_row<E, SEG>(rows, row, t.dim, l, true);
    update_row<E, SEG>(rows, row, t.dim, l, w, g, scale);
  }
  if (l == 0) t.state[row] = RowState{acc, t.sync_epoch};  // trained in this window
}

// GLOG = log2(lanes per row), SEG = pieces of four elements per lane (1 unless GLOG == 6).  A group
// owns ppl << GLOG consecutive sorted pairs (ppl = pairs per lane, at most kPairsPerLane), so a block of
// 256 threads always owns a tile of 256 * ppl pairs; the host picks ppl so that small batches still
// fill the machine.
template <typename E, int GLOG, int SEG>
__global__ __launch_bounds__(256) void seg_reduce_kernel(TableView t, const uint2* __restrict__ pair_a,
                                                         const uint2* __restrict__ pair_b, uint64_t n,
                                                         const float* __restrict__ grad, float lr, float eps,
                                                         float* __restrict__ part, uint32_t* __restrict__ part_row,
                                                         uint32_t ppl, uint32_t launched, uint32_t max_bits) {
  static_assert(SEG == 1 || GLOG == 6, "rows wider than 256 elements are held by a whole wave");
  extern __shared__ float4 s_mem[];  // [2 * groups_per_block][dim / 4] vectors, then the slot rows
  using Vec = RowVec<SEG>;
  constexpr uint32_t group = 1u << GLOG, gpb = 256u >> GLOG;  // groups (= chunks) per block
  const uint32_t chunk = ppl << GLOG, tile = 256u * ppl;
  constexpr int kWide = (int)group < 8 ? (int)group : 8;
  constexpr int kBatch = kWide / SEG > 0 ? kWide / SEG : 1;   // gradient rows in flight per lane
  const SortPlan plan = make_sort_plan(t.ctl->hwm, max_bits);
  if (plan.passes > launched) {  // the host's bound on the high-water mark was too low: nothing is sorted, nothing is touched
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(&t.ctl->n_lost, 1ull);
    if (threadIdx.x == 0) {
      part_row[2 * (uint64_t)blockIdx.x] = kNoRow;
      part_row[2 * (uint64_t)blockIdx.x + 1] = kNoRow;
    }
    return;
  }
  const uint2* __restrict__ sp = plan.passes % 2 ? pair_b : pair_a;  // where the sort left its result
  const uint32_t hwm = plan.hwm;
  n = t.ctl->scratch[kValidPairs];  // the sort left the dropped occurrences out
  const uint32_t g = threadIdx.x >> GLOG, l = threadIdx.x & (group - 1u);
  const uint32_t dim4 = t.dim >> 2;
  float4* s_vec = s_mem;
  uint32_t* s_row = reinterpret_cast<uint32_t*>(s_mem + 2 * gpb * dim4);
  const uint64_t n_chunks = (n + chunk - 1) / chunk;
  const uint64_t c0 = (uint64_t)blockIdx.x * gpb;  // first chunk of this block's tile
  const uint64_t c = c0 + g;
  const uint32_t chunks_here = (uint32_t)(n_chunks - c0 < gpb ? n_chunks - c0 : gpb);
  const bool active = l < dim4;
  const float4* g4 = reinterpret_cast<const float4*>(grad);

  // ---- phase 0: the tile's sorted pairs -> LDS (coalesced) ---------------------------------------
  __shared__ uint2 s_pairs[SEG > 1 ? kReduceTile / 2 : kReduceTile];  // (wide rows: half the pairs, see the launcher)
  {
    const uint64_t t0 = (uint64_t)blockIdx.x * tile;
#pragma unroll
    for (int m = 0; m < kPairsPerLane; ++m) {
      const uint32_t j = (uint32_t)m * 256u + threadIdx.x;
      if ((uint32_t)m < ppl) s_pairs[j] = t0 + j < n ? sp[t0 + j] : make_uint2(kNoRow, 0u);
    }
  }
  __syncthreads();

  // ---- phase 1: every group reduces the runs of its chunk -------------------------------------
  uint32_t a_row = kNoRow, b_row = kNoRow;
  if (c < n_chunks) {
    const uint64_t cs = c * chunk;
    const uint32_t count = (uint32_t)(n - cs < chunk ? n - cs : chunk);
    const uint2* mine = s_pairs + g * chunk;  // this group's chunk
    const uint32_t before = cs > 0 ? sp[cs - 1].x : kNoRow;
    const uint32_t after = cs + count < n ? sp[cs + count].x : kNoRow;
    const uint32_t first = mine[0].x;
    const bool first_head_in = cs == 0 || before != first;
    uint32_t run = first;
    bool head_in = first_head_in;
    Vec sum;
    sum.zero();
    E* rows = reinterpret_cast<E*>(t.rows);
    const float inv_dim = 1.0f / (float)t.dim;
    for (uint32_t p0 = 0; p0 < count; p0 += kBatch) {  // position of the batch in the chunk
      uint32_t kx[kBatch + 1], ky[kBatch];
      Vec v[kBatch], w[kBatch];
      float a[kBatch];
      bool tail[kBatch], apply[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const uint2 kv = p0 + (uint32_t)u < chunk ? mine[p0 + u] : make_uint2(kNoRow, 0u);
        kx[u] = kv.x;
        ky[u] = kv.y;
      }
      kx[kBatch] = p0 + kBatch < count ? mine[p0 + kBatch].x : after;
      // everything the batch needs from memory is requested before anything is consumed: the
      // gradient row of every pair and, for every run that ends in the batch and lies inside the
      // chunk, its embedding row and accumulator
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const bool in = p0 + (uint32_t)u < count;
        const uint32_t next = p0 + (uint32_t)u + 1 < count ? kx[u + 1] : after;
        tail[u] = in && next != kx[u];
        apply[u] = tail[u] && kx[u] < hwm && (kx[u] != first || first_head_in);
        v[u] = load_vec<SEG>(g4 + (uint64_t)ky[u] * dim4, l, in && kx[u] < hwm && active);
        w[u] = load_row<E, SEG>(rows, kx[u], t.dim, l, apply[u] && active);
        a[u] = apply[u] ? t.state[kx[u]].acc : 0.f;
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (p0 + (uint32_t)u < count) {
          if (kx[u] != run) {
            run = kx[u];
            head_in = true;
            sum.zero();
          }
          sum.add(v[u]);
          if (tail[u]) {
            if (apply[u]) {  // the run lies inside the chunk: row-wise Adagrad at once
              float ss = sum.sum_sq();
#pragma unroll
              for (uint32_t d = 1; d < group; d <<= 1) ss += __shfl_xor(ss, (int)d);
              const float acc = a[u] + ss * inv_dim;
              const float scale = step_scale(acc, lr, eps);
              if (active) update_row<E, SEG>(rows, run, t.dim, l, w[u], sum, scale);
              if (l == 0) t.state[run] = RowState{acc, t.sync_epoch};
            } else if (run < hwm) {  // started in an earlier chunk, ends here
              a_row = run;
              store_vec<SEG>(s_vec + (2 * g) * dim4, l, active, sum);
            }
          }
        }
      }
    }
    if (after == run && run < hwm) {  // the last run continues in the next chunk
      b_row = run | (head_in ? kHeadFlag : 0u);
      store_vec<SEG>(s_vec + (2 * g + 1) * dim4, l, active, sum);
    }
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
  float4* part4 = reinterpret_cast<float4*>(part);
  const bool walker = c < n_chunks && b_row != kNoRow && ((b_row & kHeadFlag) || g == 0);
  if (walker) {
    const uint32_t row = b_row & ~kHeadFlag;
    const bool head_in_tile = (b_row & kHeadFlag) != 0;
    Vec sum = load_vec<SEG>(s_vec + (2 * g + 1) * dim4, l, active);
    uint32_t cc = g + 1;
    bool tail = false;
    while (cc < chunks_here) {
      if (s_row[2 * cc] == row) {  // the run ends in chunk cc
        sum.add(load_vec<SEG>(s_vec + (2 * cc) * dim4, l, active));
        tail = true;
        break;
      }
      if (s_row[2 * cc + 1] != row) break;  // (cannot happen for consistent slots)
      sum.add(load_vec<SEG>(s_vec + (2 * cc + 1) * dim4, l, active));
      ++cc;
    }
    if (tail && head_in_tile) {
      adagrad_row<E, SEG>(t, row, sum, active, l, group, lr, eps);
    } else {
      const uint64_t slot = 2 * (uint64_t)blockIdx.x + (tail ? 0 : 1);
      store_vec<SEG>(part4 + slot * dim4, l, active, sum);
      if (l == 0) part_row[slot] = tail ? row : (row | (head_in_tile ? kHeadFlag : 0u));
    }
  }
  // a run that entered the tile from before and ends in chunk 0 is the tile's A partial as it stands
  if (g == 0 && c < n_chunks && a_row != kNoRow) {
    store_vec<SEG>(part4 + (2 * (uint64_t)blockIdx.x) * dim4, l, active, load_vec<SEG>(s_vec, l, active));
    if (l == 0) part_row[2 * (uint64_t)blockIdx.x] = a_row;
  }
}

// One block per tile; only the block whose tile holds the head of a border-crossing run works.
template <typename E, int SEG>
__global__ __launch_bounds__(256) void combine_kernel(TableView t, uint64_t n_tiles, const float* __restrict__ part,
                                                      const uint32_t* __restrict__ part_row, float lr, float eps,
                                                      uint32_t group_log2) {
  extern __shared__ float4 s_mem[];  // [groups_per_block][dim / 4]
  using Vec = RowVec<SEG>;
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
  const float4* part4 = reinterpret_cast<const float4*>(part);
  Vec sum;
  sum.zero();
  for (uint64_t p = g; p < pieces; p += gpb) {
    const uint64_t slot = p <= mid ? 2 * (c + p) + 1 : 2 * tail;
    sum.add(load_vec<SEG>(part4 + slot * dim4, l, active));
  }
  store_vec<SEG>(s_mem + g * dim4, l, active, sum);
  __syncthreads();
  if (g == 0) {
    Vec total;
    total.zero();
    const uint32_t used = pieces < gpb ? (uint32_t)pieces : gpb;
    for (uint32_t q = 0; q < used; ++q) total.add(load_vec<SEG>(s_mem + q * dim4, l, active));
    adagrad_row<E, SEG>(t, row, total, active, l, group, lr, eps);
  }
}

hipError_t launch_apply_grad_adagrad(const TableView& t, const UpdateWorkspace& ws, const int32_t* d_rows, uint64_t n,
                                     const int64_t* d_offsets, uint64_t n_bags, const float* d_grad, float lr, float eps,
                                     uint32_t hwm_bound, hipStream_t stream, Profiler* prof) {
  if (n == 0 || n_bags == 0) return hipSuccess;
  uint32_t launched = 0, max_bits = 0;
  hipError_t e = launch_sort_pairs(t, ws, d_rows, n, d_offsets, n_bags, hwm_bound, &launched, &max_bits, stream, prof);
  if (e != hipSuccess) return e;
  uint32_t group_log2 = 0;
  while (group_log2 < 6 && (4u << group_log2) < t.dim) ++group_log2;
  const uint32_t seg = t.dim > 256 ? t.dim / 256 : 1;  // pieces of four elements per lane
  const uint32_t gpb = 256u >> group_log2;
  // pairs per lane: fewer for small batches (at least ~2048 tiles), and at most half the maximum for rows wider
  // than 256 elements, whose partial sums take the LDS that the pairs would
  uint32_t ppl = seg > 1 ? kPairsPerLane / 2 : kPairsPerLane;
  while (ppl > 1 && (n + 256ull * ppl - 1) / (256ull * ppl) < 2048) ppl >>= 1;
  const uint64_t n_tiles = (n + 256ull * ppl - 1) / (256ull * ppl);
  const dim3 block(256), grid((unsigned)n_tiles);
  const size_t lds_reduce = 2 * gpb * (t.dim / 4) * sizeof(float4) + 2 * gpb * sizeof(uint32_t);
  const size_t lds_combine = gpb * (t.dim / 4) * sizeof(float4);
#define MONO_SEG_REDUCE(E, GLOG, SEG)                                                                                  \
  MONO_LAUNCH_SMEM(prof, K_SEG_REDUCE, stream, (seg_reduce_kernel<E, GLOG, SEG>), grid, block, lds_reduce, t, ws.pair_a, \
                   ws.pair_b, n, d_grad, lr, eps, ws.part, ws.part_row, ppl, launched, max_bits)
#define MONO_COMBINE(E, SEG)                                                                                     \
  MONO_LAUNCH_SMEM(prof, K_COMBINE, stream, (combine_kernel<E, SEG>), grid, block, lds_combine, t, n_tiles, ws.part, \
                   ws.part_row, lr, eps, group_log2)
#define MONO_SEG_REDUCE_ALL(E)                                          \
  switch (seg) {                                                        \
    case 2: MONO_SEG_REDUCE(E, 6, 2); MONO_COMBINE(E, 2); break;        \
    case 3: MONO_SEG_REDUCE(E, 6, 3); MONO_COMBINE(E, 3); break;        \
    case 4: MONO_SEG_REDUCE(E, 6, 4); MONO_COMBINE(E, 4); break;        \
    default:                                                            \
      switch (group_log2) {                                             \
        case 0: MONO_SEG_REDUCE(E, 0, 1); break;                        \
        case 1: MONO_SEG_REDUCE(E, 1, 1); break;                        \
        case 2: MONO_SEG_REDUCE(E, 2, 1); break;                        \
        case 3: MONO_SEG_REDUCE(E, 3, 1); break;                        \
        case 4: MONO_SEG_REDUCE(E, 4, 1); break;                        \
        case 5: MONO_SEG_REDUCE(E, 5, 1); break;                        \
        default: MONO_SEG_REDUCE(E, 6, 1); break;                       \
      }                                                                 \
      MONO_COMBINE(E, 1);                                               \
  }
  if (t.bf16) {
    MONO_SEG_REDUCE_ALL(uint16_t)
  } else {
    MONO_SEG_REDUCE_ALL(float)
  }
#undef MONO_COMBINE
#undef MONO_SEG_REDUCE_ALL
#undef MONO_SEG_REDUCE
  return hipGetLastError();
}

}  // namespace mono
