// Optional per-kernel timing with HIP events (benchmark instrumentation, off by default).
#pragma once

#include <hip/hip_runtime.h>

#include <vector>

namespace mono {

enum KernelId {
  K_PROBE_COUNT = 0,
  K_ADMIT_ELECT,
  K_INSERT,
  K_RESOLVE,
  K_GATHER_POOL,
  K_SORT_HIST,
  K_SORT_SCAN,
  K_SORT_SCATTER,
  K_SEG_REDUCE,
  K_COMBINE,
  K_SWEEP_BEGIN,
  K_SWEEP,
  K_SWEEP_REMOVE,
  K_SWEEP_END,
  K_COUNT
};

inline const char* kernel_name(int id) {
  static const char* names[K_COUNT] = {"probe_count", "admit_elect", "insert", "resolve", "gather_pool",
                                       "sort_hist",   "sort_scan",    "sort_scatter", "seg_reduce",  "combine",
                                       "sweep_begin", "sweep_find", "sweep_remove", "sweep_end"};
  return id >= 0 && id < K_COUNT ? names[id] : "?";
}

struct Profiler {
  struct Rec {
    int id;
    hipEvent_t start, stop;
  };
  bool on = false;
  std::vector<Rec> recs;
};

// Brackets one kernel launch with two events on its stream when profiling is on.
class ProfScope {
 public:
  ProfScope(Profiler* p, int id, hipStream_t s) : p_(p && p->on ? p : nullptr), s_(s) {
    if (!p_) return;
    rec_.id = id;
    if (hipEventCreate(&rec_.start) != hipSuccess) {
      p_ = nullptr;
      return;
    }
    if (hipEventCreate(&rec_.stop) != hipSuccess) {
      (void)hipEventDestroy(rec_.start);
      p_ = nullptr;
      return;
    }
    (void)hipEventRecord(rec_.start, s_);
  }
  ~ProfScope() {
    if (!p_) return;
    (void)hipEventRecord(rec_.stop, s_);
    p_->recs.push_back(rec_);
  }

 private:
  Profiler* p_;
  hipStream_t s_;
  Profiler::Rec rec_{};
};

}  // namespace mono

#define MONO_LAUNCH_SMEM(prof, id, stream, kernel, grid, block, smem, ...)      \
  do {                                                                       \
    ::mono::ProfScope mono_ps_((prof), (id), (stream));                      \
    hipLaunchKernelGGL(kernel, (grid), (block), (smem), (stream), __VA_ARGS__); \
  } while (0)

#define MONO_LAUNCH(prof, id, stream, kernel, grid, block, ...)              \
  do {                                                                       \
    ::mono::ProfScope mono_ps_((prof), (id), (stream));                      \
    hipLaunchKernelGGL(kernel, (grid), (block), 0, (stream), __VA_ARGS__);   \
  } while (0)
