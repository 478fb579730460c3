// Per-kernel timing with HIP events, the library's counterpart of the paper's
// profiling step (per-layer execution time feeds the "by Time" balancers).
#pragma once

#include "common.h"

namespace dynmo {

enum KernelId {
  K_ROUTE_TOPK = 0,
  K_ROUTE_CAPACITY,
  K_ROUTE_ACTIVE,
  K_ROUTE_TOPK_BWD,
  K_ROUTE_CAPACITY_BWD,
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

extern bool g_profile_on;
void profile_begin(KernelId id, hipStream_t st);
void profile_end(KernelId id, hipStream_t st);

// Brackets one kernel launch with an event pair when profiling is enabled.
struct ProfScope {
  KernelId id;
  hipStream_t st;
  bool on;
  ProfScope(KernelId id_, hipStream_t st_) : id(id_), st(st_), on(g_profile_on) {
    if (on) profile_begin(id, st);
  }
  ~ProfScope() {
    if (on) profile_end(id, st);
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
