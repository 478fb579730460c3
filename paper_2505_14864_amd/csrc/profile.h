// Per-kernel timing with HIP events, the library's counterpart of the paper's
// profiling step (per-layer execution time feeds the "by Time" balancers).
#pragma once

#include <atomic>

#include "common.h"

namespace dynmo {

enum KernelId {
  K_ROUTE_TOPK = 0,
  K_ROUTE_CAPACITY,
  K_ROUTE_ACTIVE,
  K_ROUTE_TOPK_BWD,
  K_ROUTE_CAPACITY_BWD,
  K_ROUTE_DROP,
  K_PERMUTE_COUNT,
  K_PERMUTE_SCAN,
  K_PERMUTE_SCATTER,
  K_PERMUTE_ROWS,
  K_PERMUTE_BWD,
  K_COMBINE,
  K_COMBINE_BWD,
  K_FFN_GATEUP,
  K_FFN_DOWN,
  K_FFN_DA,
  K_FFN_DX,
  K_FFN_DWD,
  K_FFN_DWG,
  K_FFN_DWU,
  K_COUNT
};

extern std::atomic<bool> g_profile_on;
// profile_begin records the start event of a new pair for kernel role `id` and returns the
// pair's stop event (nullptr if no pair could be made: too many pending, or no event);
// profile_end records exactly that stop event, so concurrent launches of one role from
// several host threads cannot mix up each other's pairs.
hipEvent_t profile_begin(KernelId id, hipStream_t st);
void profile_end(hipEvent_t stop, hipStream_t st);

// Brackets one kernel launch with an event pair when profiling is enabled.
struct ProfScope {
  hipStream_t st;
  hipEvent_t stop;
  ProfScope(KernelId id, hipStream_t st_) : st(st_), stop(nullptr) {
    if (g_profile_on.load(std::memory_order_relaxed)) stop = profile_begin(id, st);
  }
  ~ProfScope() {
    if (stop) profile_end(stop, st);
  }
};

}  // namespace dynmo

// Launches one kernel inside a ProfScope and checks the launch.
#define DYNMO_TIMED_LAUNCH(id, st, ...)          \
  {                                              \
    ::dynmo::ProfScope _prof((id), (st));        \
    __VA_ARGS__;                                 \
  }                                              \
  DYNMO_LAUNCH_CHECK()
