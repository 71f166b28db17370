// Host side of the C ABI declared in include/monotable.h: argument checks, arena layout, launches.
#include <mutex>
#include <new>

#include "../../include/monotable.h"
#include "common.h"
#include "kernels.h"

using namespace mono;

struct mono_table {
  TableView view;
  UpdateWorkspace ws;
  void* owned_arena = nullptr;  // non-null when the library allocated the arena
  uint64_t max_ids = 0, max_bags = 0, dset_size = 0;
  uint32_t epoch = 0;       // per-call tag of the dedup set
  uint32_t last_step = 0;
  uint64_t seed = 0;
  uint32_t generation = 0;  // rehash generation of the placement hashes h0 / h1
  int device = 0;
  hipStream_t last_stream = nullptr;  // stream of the latest call that queued work for this table
  bool used_stream = false;
  // Bound on the device's high-water mark of rows, kept without waiting for the device: every
  // lookup_or_insert leaves (its call tag << 32 | mark) in a pinned host word when it ends, and the host
  // remembers how many keys each of its latest calls held (a call hands out at most one row per key).
  unsigned long long* h_mail = nullptr;       // pinned; null: no bound is kept (the capacity is used)
  static constexpr uint32_t kRecentCalls = 256;
  uint32_t recent_tag[kRecentCalls] = {0};    // call tags, by tag % kRecentCalls (0 = unused)
  uint64_t recent_n[kRecentCalls] = {0};      // keys of that call
  bool tags_wrapped = false;                  // the 32-bit call tag has wrapped: the bound is given up
  Profiler prof;
};

// Fixed workspace of mono_apply_grad_adagrad_noalloc: one copy per GPU the library runs on, held until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the address the
// kernels get is the per-device pointer that static_workspace() keeps.
constexpr uint64_t kStaticMaxIds = MONO_NOALLOC_MAX_IDS;  // largest batch of the allocation-free entry point
constexpr uint32_t kStaticMaxDim = 1024;
constexpr size_t static_part(size_t bytes) { return (bytes + 255) & ~(size_t)255; }
constexpr size_t kStaticScratchBytes =
    static_part(kStaticMaxIds * 4) + 2 * static_part(kStaticMaxIds * sizeof(uint2)) +
    static_part((size_t)512 * ((kStaticMaxIds + 2047) / 2048 + 1) * 4) +  // (at least sort_hist_words: checked below)
    static_part(2 * ((kStaticMaxIds + 255) / 256) * kStaticMaxDim * sizeof(float)) +
    static_part(2 * ((kStaticMaxIds + 255) / 256) * sizeof(uint32_t));
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

bool is_pow2(uint64_t v) { return v && !(v & (v - 1)); }
int log2u(uint64_t v) {
  int lg = 0;
  while ((1ull << lg) < v) ++lg;
  return lg;
}
size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// salt i of a seed: output i + 1 of the SplitMix64 sequence started at the seed
uint64_t salt(uint64_t seed, int i) { return mix64(seed + (uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull); }
// The placement hashes of rehash generation g are salted from seed + g * (an odd constant);
// generation 0 is the table as created.  Counter, initial-value and dedup hashes never change.
uint64_t placement_seed(uint64_t seed, uint32_t generation) {
  return seed + (uint64_t)generation * 0xD1B54A32D192ED03ull;
}

// embedding dimension: a multiple of 4 up to 256 (one lane group per row), or a multiple of 256 up to 1024
// (the whole wave walks the row in segments of 256 elements)
bool valid_dim(uint32_t dim) { return dim >= 4 && dim % 4 == 0 && (dim <= 256 || (dim <= 1024 && dim % 256 == 0)); }

bool valid_shape(uint64_t capacity, uint32_t dim, uint32_t flags, uint64_t max_ids, uint64_t max_bags) {
  return is_pow2(capacity) && capacity >= 16 && capacity <= (1ull << 30) && valid_dim(dim) &&
         flags <= MONO_ROWS_BF16 && max_ids >= 1 && max_ids <= (1ull << 28) && max_bags >= 1 && max_bags <= max_ids + 1;
}

// number of occurrence counters: 2^filter_log2, or 4 * capacity when filter_log2 == 0
uint64_t filter_size(uint64_t capacity, uint32_t filter_log2) {
  return filter_log2 ? 1ull << filter_log2 : 4 * capacity;
}
bool valid_filter(uint64_t capacity, uint32_t filter_hashes, uint32_t filter_log2) {
  (void)capacity;
  return filter_hashes >= 1 && filter_hashes <= 4 && (filter_log2 == 0 || (filter_log2 >= 4 && filter_log2 <= 34));
}

uint64_t dedup_size(uint64_t max_ids) {
  uint64_t s = 64;
  while (s < 2 * max_ids) s <<= 1;
  return s;
}

// Carves the arena; with base == nullptr only measures.  Returns the bytes used.
size_t layout(mono_table* t, char* base, uint64_t capacity, uint32_t dim, uint32_t flags, uint64_t max_ids,
              uint64_t max_bags, uint64_t n_filter) {
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes);
    return p;
  };
  const uint64_t n_buckets = capacity / 2 / kBucket, dset = dedup_size(max_ids);
  const size_t esize = flags == MONO_ROWS_BF16 ? 2 : 4;
  char* buckets = take(2 * n_buckets * sizeof(Bucket));
  char* filter = take(n_filter * sizeof(unsigned long long));
  char* rows = take(capacity * dim * esize);
  char* state = take(capacity * sizeof(RowState));
  char* free_rows = take(capacity * sizeof(uint32_t));
  char* ctl = take(sizeof(Control));
  char* stash = take(kStashCap * sizeof(StashEntry));
  char* dset_p = take(dset * sizeof(unsigned long long));
  char* dset_row = take(dset * sizeof(int32_t));
  // a sub-list takes the winners of every kWinLists-th block of the election kernel, whose blocks hold 256 or
  // 1024 occurrences: sized for the larger, which also covers the smaller
  const uint64_t win_cap = ((max_ids + 1023) / 1024 + kWinLists - 1) / kWinLists * 1024;
  const uint64_t sweep_blocks = (capacity + kSweepSlotsPerBlock - 1) / kSweepSlotsPerBlock;
  const uint64_t sweep_cap = (sweep_blocks + kWinLists - 1) / kWinLists * kSweepSlotsPerBlock;
  char* win_list = take(kWinLists * win_cap * sizeof(Winner));
  char* win_cnt = take(kWinLists * kWinStride * sizeof(uint32_t));
  char* occupied = take(occupancy_words(capacity) * sizeof(unsigned long long));
  char* sweep_list = take(kWinLists * sweep_cap * sizeof(uint32_t));
  char* sweep_cnt = take(kWinLists * kWinStride * sizeof(uint32_t));
  const uint64_t tiles = reduce_tiles(max_ids);
  char* unit_bag = take(max_ids * 4);
  char* pair_a = take(max_ids * sizeof(uint2));
  char* pair_b = take(max_ids * sizeof(uint2));
  char* hist = take(sort_hist_words(max_ids) * 4);
  char* part = take(2 * tiles * dim * sizeof(float));
  char* part_row = take(2 * tiles * sizeof(uint32_t));
  (void)max_bags;
  if (t && base) {
    TableView& v = t->view;
    v.buckets = (Bucket*)buckets;
    v.filter = (unsigned long long*)filter;
    v.rows = rows;
    v.state = (RowState*)state;
    v.free_rows = (uint32_t*)free_rows;
    v.ctl = (Control*)ctl;
    v.stash = (StashEntry*)stash;
    v.dset = (unsigned long long*)dset_p;
    v.dset_row = (int32_t*)dset_row;
    v.win_list = (Winner*)win_list;
    v.win_cnt = (uint32_t*)win_cnt;
    v.win_cap = win_cap;
    v.occupied = (unsigned long long*)occupied;
    v.sweep_list = (uint32_t*)sweep_list;
    v.sweep_cnt = (uint32_t*)sweep_cnt;
    v.sweep_cap = sweep_cap;
    t->ws.unit_bag = (uint32_t*)unit_bag;
    t->ws.pair_a = (uint2*)pair_a;
    t->ws.pair_b = (uint2*)pair_b;
    t->ws.hist = (uint32_t*)hist;
    t->ws.part = (float*)part;
    t->ws.part_row = (uint32_t*)part_row;
  }
  return off;
}

// The per-device address of `scratch`, resolved once per device with that device current.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mutex;

hipError_t static_workspace(int device, uint32_t dim, UpdateWorkspace* ws) {
  if (sort_hist_words(kStaticMaxIds) > (size_t)512 * ((kStaticMaxIds + 2047) / 2048 + 1)) return hipErrorInvalidValue;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
      int current = -1;
      hipError_t e = hipGetDevice(&current);
      if (e != hipSuccess) return e;
      if (current != device) return hipErrorInvalidDevice;  // the table's device must be the current one
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (!p) return hipErrorInvalidSymbol;
      g_scratch_ptr[device] = p;
    }
    base = g_scratch_ptr[device];
  }
  char* at = (char*)base;
  auto take = [&](size_t bytes) {
    char* p = at;
    at += static_part(bytes);
    return p;
  };
  const uint64_t tiles = reduce_tiles(kStaticMaxIds);
  ws->unit_bag = (uint32_t*)take(kStaticMaxIds * 4);
  ws->pair_a = (uint2*)take(kStaticMaxIds * sizeof(uint2));
  ws->pair_b = (uint2*)take(kStaticMaxIds * sizeof(uint2));
  ws->hist = (uint32_t*)take(sort_hist_words(kStaticMaxIds) * 4);
  ws->part = (float*)take(2 * tiles * dim * sizeof(float));
  ws->part_row = (uint32_t*)((char*)base + kStaticScratchBytes - static_part(2 * tiles * sizeof(uint32_t)));
  return hipSuccess;
}

void note_call(mono_table* t, uint32_t tag, uint64_t n) {
  t->recent_tag[tag % mono_table::kRecentCalls] = tag;
  t->recent_n[tag % mono_table::kRecentCalls] = n;
}

// A number that the table's high-water mark cannot exceed when work queued now runs: the mark that the
// device reported last, plus the keys of every call queued after the one that reported it.  A stale report
// only makes the bound larger (the mark never shrinks).
uint32_t hwm_bound(const mono_table* t) {
  const uint64_t capacity = t->view.capacity;
  if (!t->h_mail || t->tags_wrapped) return (uint32_t)capacity;
  const unsigned long long mail = *(volatile const unsigned long long*)t->h_mail;
  const uint32_t tag = (uint32_t)(mail >> 32);
  uint64_t bound = (uint32_t)mail;
  if (t->epoch < tag || t->epoch - tag >= mono_table::kRecentCalls) return (uint32_t)capacity;
  for (uint32_t c = tag + 1; c <= t->epoch && c != 0; ++c) {
    if (t->recent_tag[c % mono_table::kRecentCalls] != c) return (uint32_t)capacity;  // not on record
    bound += t->recent_n[c % mono_table::kRecentCalls];
    if (bound >= capacity) return (uint32_t)capacity;
  }
  return (uint32_t)(bound < capacity ? bound : capacity);
}

void note_stream(mono_table* t, void* stream) {
  t->last_stream = (hipStream_t)stream;
  t->used_stream = true;
}

}  // namespace

extern "C" {

const char* mono_strerror(int err) {
  switch (err) {
    case MONO_OK: return "ok";
    case MONO_EINVAL: return "invalid argument";
    case MONO_ENOMEM: return "out of device memory";
    case MONO_EHIP: return "HIP runtime error";
    case MONO_ELIMIT: return "batch exceeds the fixed workspace of the allocation-free entry point";
    default: return "unknown error";
  }
}

size_t mono_table_bytes_ex(uint64_t capacity, uint32_t dim, uint32_t flags, uint64_t max_ids, uint64_t max_bags,
                           uint32_t filter_log2) {
  if (!valid_shape(capacity, dim, flags, max_ids, max_bags) || !valid_filter(capacity, 1, filter_log2)) return 0;
  return layout(nullptr, nullptr, capacity, dim, flags, max_ids, max_bags, filter_size(capacity, filter_log2));
}

size_t mono_table_bytes(uint64_t capacity, uint32_t dim, uint32_t flags, uint64_t max_ids, uint64_t max_bags) {
  return mono_table_bytes_ex(capacity, dim, flags, max_ids, max_bags, 0);
}

int mono_table_create(mono_table** out, uint64_t capacity, uint32_t dim, uint64_t seed, uint32_t freq_threshold,
                      uint32_t expire_steps, uint32_t flags, uint64_t max_ids, uint64_t max_bags, void* d_arena,
                      size_t arena_bytes, void* stream) {
  return mono_table_create_ex(out, capacity, dim, seed, freq_threshold, expire_steps, flags, max_ids, max_bags, 1, 0,
                              d_arena, arena_bytes, stream);
}

int mono_table_create_ex(mono_table** out, uint64_t capacity, uint32_t dim, uint64_t seed, uint32_t freq_threshold,
                         uint32_t expire_steps, uint32_t flags, uint64_t max_ids, uint64_t max_bags,
                         uint32_t filter_hashes, uint32_t filter_log2, void* d_arena, size_t arena_bytes, void* stream) {
  if (!out) return MONO_EINVAL;
  *out = nullptr;
  if (!valid_shape(capacity, dim, flags, max_ids, max_bags) || freq_threshold > 255 || expire_steps >= (1u << 24) ||
      !valid_filter(capacity, filter_hashes, filter_log2))
    return MONO_EINVAL;
  const uint64_t n_filter = filter_size(capacity, filter_log2);
  const size_t need = layout(nullptr, nullptr, capacity, dim, flags, max_ids, max_bags, n_filter);
  if (d_arena && (arena_bytes < need || ((uintptr_t)d_arena & 255))) return MONO_EINVAL;
  mono_table* t = new (std::nothrow) mono_table();
  if (!t) return MONO_ENOMEM;
  if (hipGetDevice(&t->device) != hipSuccess) {
    delete t;
    return MONO_EHIP;
  }
  char* base = (char*)d_arena;
  if (!base) {
    if (hipMalloc((void**)&base, need) != hipSuccess) {
      (void)hipGetLastError();
      delete t;
      return MONO_ENOMEM;
    }
    t->owned_arena = base;
  }
  layout(t, base, capacity, dim, flags, max_ids, max_bags, n_filter);
  TableView& v = t->view;
  v.capacity = capacity;
  v.n_buckets = capacity / 2 / kBucket;
  v.n_filter = n_filter;
  v.filter_hashes = filter_hashes;
  t->dset_size = dedup_size(max_ids);
  v.dset_mask = t->dset_size - 1;
  uint64_t s[5];
  for (int i = 0; i < 5; ++i) s[i] = salt(seed, i);
  t->seed = seed;
  v.s_h0 = s[0];
  v.s_h1 = s[1];
  v.s_filter[0] = s[2];
  for (int j = 1; j < 4; ++j) v.s_filter[j] = salt(seed, 7 + j);
  v.s_init = s[3];
  v.s_dedup = s[4];
  v.bucket_shift = 64u - (uint32_t)log2u(v.n_buckets);
  v.filter_shift = 64u - (uint32_t)log2u(v.n_filter);
  v.dim = dim;
  v.freq_threshold = freq_threshold;
  v.expire_steps = expire_steps;
  v.bf16 = flags == MONO_ROWS_BF16;
  v.sync_epoch = 1;
  t->max_ids = max_ids;
  t->max_bags = max_bags;
  {  // (pinned host memory is allocated, never registered; without it the sort is simply sized for the capacity)
    void* mail = nullptr;
    void* mail_dev = nullptr;
    if (hipHostMalloc(&mail, sizeof(unsigned long long), hipHostMallocMapped) == hipSuccess && mail &&
        hipHostGetDevicePointer(&mail_dev, mail, 0) == hipSuccess && mail_dev) {
      t->h_mail = (unsigned long long*)mail;
      *t->h_mail = 0;  // call tag 0, mark 0: an empty table
      v.hwm_mail = (unsigned long long*)mail_dev;
    } else {
      (void)hipGetLastError();
      if (mail) (void)hipHostFree(mail);
      v.hwm_mail = nullptr;
    }
  }
  note_stream(t, stream);
  if (launch_table_init(v, t->dset_size, (hipStream_t)stream) != hipSuccess) {
    if (t->owned_arena) (void)hipFree(t->owned_arena);
    if (t->h_mail) (void)hipHostFree(t->h_mail);
    delete t;
    return MONO_EHIP;
  }
  *out = t;
  return MONO_OK;
}

int mono_table_destroy(mono_table* t) {
  if (!t) return MONO_EINVAL;
  int rc = MONO_OK;
  // the calls of a table go to one stream in order: waiting for the latest one is waiting for all of them
  if ((t->used_stream ? hipStreamSynchronize(t->last_stream) : hipDeviceSynchronize()) != hipSuccess) rc = MONO_EHIP;
  if (t->owned_arena && hipFree(t->owned_arena) != hipSuccess) rc = MONO_EHIP;
  if (t->h_mail && hipHostFree(t->h_mail) != hipSuccess) rc = MONO_EHIP;
  for (auto& r : t->prof.recs) {  // timings nobody read
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  delete t;
  return rc;
}

int mono_lookup_or_insert(mono_table* t, const int64_t* d_keys, uint64_t n, uint32_t step, int32_t* d_rows_out,
                          void* stream) {
  if (!t || n > t->max_ids || step >= (1u << 24) || step < t->last_step) return MONO_EINVAL;
  if (n == 0) return MONO_OK;
  if (!d_keys || !d_rows_out) return MONO_EINVAL;
  note_stream(t, stream);
  uint32_t epoch = t->epoch + 1;
  if (epoch == 0) {  // the 32-bit call tag wrapped: forget every old tag
    if (hipMemsetAsync(t->view.dset, 0, t->dset_size * sizeof(unsigned long long), (hipStream_t)stream) != hipSuccess)
      return MONO_EHIP;
    epoch = 1;
    t->tags_wrapped = true;
  }
  const RestoreSource none = {nullptr, nullptr, nullptr};
  if (launch_lookup_or_insert(t->view, d_keys, n, step, epoch, d_rows_out, none, (hipStream_t)stream, &t->prof) != hipSuccess)
    return MONO_EHIP;  // (the table's step and call tag move on only when the call was queued)
  t->epoch = epoch;
  t->last_step = step;
  note_call(t, epoch, n);
  return MONO_OK;
}

int mono_gather_pool(mono_table* t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets, uint64_t n_bags,
                     float* d_out, void* stream) {
  if (!t || n > t->max_ids || n_bags > t->max_bags) return MONO_EINVAL;
  note_stream(t, stream);
  if (n_bags == 0) return MONO_OK;
  if (!d_offsets || !d_out || (n && !d_rows)) return MONO_EINVAL;
  return launch_gather_pool(t->view, d_rows, n, d_offsets, n_bags, d_out, (hipStream_t)stream, &t->prof) == hipSuccess ? MONO_OK
                                                                                                           : MONO_EHIP;
}

int mono_qr_gather_pool(const void* d_table_r, const void* d_table_q, uint32_t log2_rows, uint32_t dim, uint32_t flags,
                        const int64_t* d_ids, uint64_t n, const int64_t* d_offsets, uint64_t n_bags, float* d_out,
                        void* stream) {
  if (log2_rows < 1 || log2_rows > 30 || !valid_dim(dim) || flags > MONO_ROWS_BF16 || n > (1ull << 40)) return MONO_EINVAL;
  if (n_bags == 0) return MONO_OK;
  if (!d_table_r || !d_table_q || !d_offsets || !d_out || (n && !d_ids)) return MONO_EINVAL;
  return launch_qr_gather_pool(d_table_r, d_table_q, log2_rows, dim, flags == MONO_ROWS_BF16, d_ids, n, d_offsets, n_bags,
                               d_out, (hipStream_t)stream) == hipSuccess
             ? MONO_OK
             : MONO_EHIP;
}

int mono_apply_grad_adagrad(mono_table* t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets,
                            uint64_t n_bags, const float* d_grad, float lr, float eps, void* stream) {
  if (!t || n > t->max_ids || n_bags > t->max_bags) return MONO_EINVAL;
  note_stream(t, stream);
  if (n == 0 || n_bags == 0) return MONO_OK;
  if (!d_rows || !d_offsets || !d_grad) return MONO_EINVAL;
  return launch_apply_grad_adagrad(t->view, t->ws, d_rows, n, d_offsets, n_bags, d_grad, lr, eps, hwm_bound(t),
                                   (hipStream_t)stream, &t->prof) == hipSuccess
             ? MONO_OK
             : MONO_EHIP;
}

uint64_t mono_noalloc_max_ids(void) { return kStaticMaxIds; }

int mono_apply_grad_adagrad_noalloc(mono_table* t, const int32_t* d_rows, uint64_t n, const int64_t* d_offsets,
                                    uint64_t n_bags, const float* d_grad, float lr, float eps, void* stream) {
  if (!t) return MONO_EINVAL;
  note_stream(t, stream);
  if (n > kStaticMaxIds || n_bags > kStaticMaxIds + 1 || t->view.dim > kStaticMaxDim) return MONO_ELIMIT;
  if (n == 0 || n_bags == 0) return MONO_OK;
  if (!d_rows || !d_offsets || !d_grad) return MONO_EINVAL;
  UpdateWorkspace ws;
  if (static_workspace(t->device, t->view.dim, &ws) != hipSuccess) return MONO_EHIP;
  // (no per-kernel events here: creating one may allocate)
  return launch_apply_grad_adagrad(t->view, ws, d_rows, n, d_offsets, n_bags, d_grad, lr, eps, hwm_bound(t),
                                   (hipStream_t)stream, nullptr) == hipSuccess
             ? MONO_OK
             : MONO_EHIP;
}

int mono_expire_sweep(mono_table* t, uint32_t now, uint64_t* d_n_expired, int64_t* d_expired_keys,
                      uint64_t max_expired, void* stream) {
  if (!t || now >= (1u << 24)) return MONO_EINVAL;
  note_stream(t, stream);
  return launch_expire_sweep(t->view, now, d_n_expired, d_expired_keys, d_expired_keys ? max_expired : 0,
                             (hipStream_t)stream, &t->prof) == hipSuccess
             ? MONO_OK
             : MONO_EHIP;
}

int mono_table_stats(mono_table* t, mono_stats* h_out, void* stream) {
  if (!t || !h_out) return MONO_EINVAL;
  Control c;
  if (hipMemcpyAsync(&c, t->view.ctl, sizeof(Control), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess ||
      hipStreamSynchronize((hipStream_t)stream) != hipSuccess)
    return MONO_EHIP;
  // (if that was the table's own stream, everything queued for the table has run: the mark just read is exact)
  if (t->h_mail && !t->tags_wrapped && t->used_stream && (hipStream_t)stream == t->last_stream)
    *t->h_mail = ((unsigned long long)t->epoch << 32) | (unsigned long long)c.hwm;
  h_out->capacity = t->view.capacity;
  h_out->size = t->view.capacity - (uint64_t)(c.free_n < 0 ? 0 : c.free_n);
  h_out->n_admitted = c.n_admitted;
  h_out->n_expired = c.n_expired;
  h_out->n_insert_failed = c.n_insert_failed;
  h_out->n_lost = c.n_lost;
  h_out->n_full = c.n_full;
  h_out->stash_size = c.stash_n < kStashCap ? c.stash_n : kStashCap;
  h_out->max_chain = c.max_chain;
  return MONO_OK;
}

int mono_table_export(mono_table* t, int64_t* d_keys, int32_t* d_row, uint32_t* d_last_seen, int64_t* d_slot,
                      float* d_values, float* d_acc, uint64_t max_n, uint64_t* h_n, void* stream) {
  if (!t || !h_n) return MONO_EINVAL;
  if ((d_values || d_acc) && !d_row) return MONO_EINVAL;  // values are gathered through the row indices
  hipStream_t s = (hipStream_t)stream;
  if (launch_export(t->view, d_keys, d_row, d_last_seen, d_slot, max_n, false, s) != hipSuccess) return MONO_EHIP;
  unsigned long long n = 0;
  if (hipMemcpyAsync(&n, &t->view.ctl->scratch[kExportCount], sizeof(n), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return MONO_EHIP;
  *h_n = n;
  const uint64_t wrote = n < max_n ? n : max_n;
  if ((d_values || d_acc) && wrote) {
    if (launch_export_values(t->view, d_row, wrote, d_values, d_acc, s) != hipSuccess) return MONO_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return MONO_EHIP;
  }
  return MONO_OK;
}

int mono_export_touched(mono_table* t, int64_t* d_keys, int32_t* d_row, float* d_values, float* d_acc, uint64_t max_n,
                        uint64_t* h_n, void* stream) {
  if (!t || !h_n) return MONO_EINVAL;
  if ((d_values || d_acc) && !d_row) return MONO_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (launch_export(t->view, d_keys, d_row, nullptr, nullptr, max_n, true, s) != hipSuccess) return MONO_EHIP;
  unsigned long long n = 0;
  if (hipMemcpyAsync(&n, &t->view.ctl->scratch[kExportCount], sizeof(n), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return MONO_EHIP;
  *h_n = n;
  if (n > max_n) return MONO_OK;  // the caller's buffers are too small: the window stays open
  if ((d_values || d_acc) && n) {
    if (launch_export_values(t->view, d_row, n, d_values, d_acc, s) != hipSuccess) return MONO_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return MONO_EHIP;
  }
  t->view.sync_epoch += 1;  // a new window: nothing is touched any more, and no memory was cleared for it
  return MONO_OK;
}

int mono_table_import(mono_table* t, const int64_t* d_keys, const float* d_values, const float* d_acc,
                      const uint32_t* d_last_seen, uint64_t n, uint64_t* h_refused, void* stream) {
  if (!t || n > t->max_ids) return MONO_EINVAL;
  note_stream(t, stream);
  if (h_refused) *h_refused = 0;
  if (n == 0) return MONO_OK;
  if (!d_keys || !d_values || !d_acc || !d_last_seen) return MONO_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (++t->epoch == 0) {
    if (hipMemsetAsync(t->view.dset, 0, t->dset_size * sizeof(unsigned long long), s) != hipSuccess) return MONO_EHIP;
    t->epoch = 1;
    t->tags_wrapped = true;
  }
  note_call(t, t->epoch, n);
  if (hipMemsetAsync(&t->view.ctl->scratch[kRefusedRecords], 0, sizeof(unsigned long long), s) != hipSuccess)
    return MONO_EHIP;
  const RestoreSource src = {d_values, d_acc, d_last_seen};
  // the per-occurrence result array of the four kernels lives in the update workspace (max_ids words)
  if (launch_lookup_or_insert(t->view, d_keys, n, 0, t->epoch, (int32_t*)t->ws.unit_bag, src, s, &t->prof) != hipSuccess)
    return MONO_EHIP;
  if (h_refused) {
    unsigned long long r = 0;
    if (hipMemcpyAsync(&r, &t->view.ctl->scratch[kRefusedRecords], sizeof(r), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
      return MONO_EHIP;
    *h_refused = r;
  }
  return MONO_OK;
}

int mono_filter_import(mono_table* t, const uint32_t* d_words, uint64_t first, uint64_t count, void* stream) {
  if (!t || first + count > t->view.n_filter || (count && !d_words)) return MONO_EINVAL;
  note_stream(t, stream);
  return launch_filter_import(t->view, d_words, first, count, (hipStream_t)stream) == hipSuccess ? MONO_OK : MONO_EHIP;
}

int mono_table_migrate(mono_table* dst, mono_table* src, uint32_t generation, void* stream) {
  if (!dst || !src || dst == src) return MONO_EINVAL;
  const TableView& a = src->view;
  TableView& b = dst->view;
  if (b.capacity < a.capacity || b.dim != a.dim || b.bf16 != a.bf16 || dst->seed != src->seed ||
      b.freq_threshold != a.freq_threshold || b.expire_steps != a.expire_steps || dst->epoch != 0 ||
      dst->last_step != 0 || b.filter_hashes != a.filter_hashes ||
      b.n_filter < a.n_filter ||
      b.n_filter / a.n_filter != b.capacity / a.capacity)  // the counter array grows with the table (powers of two)
    return MONO_EINVAL;  // dst must be a fresh table with the same parameters
  hipStream_t s = (hipStream_t)stream;
  note_stream(dst, stream);
  Control c;
  if (hipMemcpyAsync(&c, a.ctl, sizeof(Control), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return MONO_EHIP;
  b.s_h0 = salt(placement_seed(dst->seed, generation), 0);
  b.s_h1 = salt(placement_seed(dst->seed, generation), 1);
  b.sync_epoch = a.sync_epoch;
  dst->generation = generation;
  dst->last_step = src->last_step;
  dst->epoch = 1;  // dst counts as used from here on (a second migration into it is refused)
  if (dst->h_mail) *dst->h_mail = (1ull << 32) | (unsigned long long)c.hwm;  // rows keep their indices: so does the mark
  // rows and their state keep their indices: copied position for position up to the high-water mark
  const size_t esize = a.bf16 ? 2 : 4;
  if (c.hwm) {
    if (hipMemcpyAsync(b.rows, a.rows, (size_t)c.hwm * a.dim * esize, hipMemcpyDeviceToDevice, s) != hipSuccess ||
        hipMemcpyAsync(b.state, a.state, (size_t)c.hwm * sizeof(RowState), hipMemcpyDeviceToDevice, s) != hipSuccess)
      return MONO_EHIP;
  }
  Control d = c;
  d.stash_n = 0;  // stash elements get a new chance under the new hash functions
  d.free_n = c.free_n + (int32_t)(b.capacity - a.capacity);
  for (auto& x : d.scratch) x = 0;
  if (hipMemcpyAsync(b.ctl, &d, sizeof(Control), hipMemcpyHostToDevice, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)  // `d` is a local: the copy must have left it
    return MONO_EHIP;
  return launch_migrate(b, a, c.free_n, s) == hipSuccess ? MONO_OK : MONO_EHIP;
}

int mono_filter_export(mono_table* t, uint32_t* d_words, uint64_t first, uint64_t count, void* stream) {
  if (!t || first + count > t->view.n_filter || (count && !d_words)) return MONO_EINVAL;
  if (launch_filter_export(t->view, d_words, first, count, (hipStream_t)stream) != hipSuccess) return MONO_EHIP;
  return hipStreamSynchronize((hipStream_t)stream) == hipSuccess ? MONO_OK : MONO_EHIP;
}

int mono_profile_enable(mono_table* t, int on) {
  if (!t) return MONO_EINVAL;
  t->prof.on = on != 0;
  return MONO_OK;
}

int mono_profile_read(mono_table* t, const char** h_names, double* h_ms, uint64_t* h_launches, uint32_t max_kernels,
                      uint32_t* h_n) {
  if (!t || !h_n) return MONO_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return MONO_EHIP;
  double ms[K_COUNT] = {0};
  uint64_t cnt[K_COUNT] = {0};
  for (auto& r : t->prof.recs) {
    float e = 0.f;
    if (hipEventElapsedTime(&e, r.start, r.stop) == hipSuccess) {
      ms[r.id] += e;
      cnt[r.id] += 1;
    }
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  t->prof.recs.clear();
  uint32_t k = 0;
  for (int id = 0; id < K_COUNT && k < max_kernels; ++id) {
    if (!cnt[id]) continue;
    if (h_names) h_names[k] = kernel_name(id);
    if (h_ms) h_ms[k] = ms[id];
    if (h_launches) h_launches[k] = cnt[id];
    ++k;
  }
  *h_n = k;
  return MONO_OK;
}

}  // extern "C"
