#include "profile.h"

#include <mutex>
#include <vector>

namespace dynmo {

std::atomic<bool> g_profile_on{false};

namespace {
struct Slot {
  std::vector<hipEvent_t> start, stop;
  double total_ms = 0.0;
  int64_t launches = 0;
};
Slot g_slots[K_COUNT];
std::vector<hipEvent_t> g_free;
std::mutex g_mu;
constexpr size_t kMaxPending = 1 << 16;

const char* const kNames[K_COUNT] = {
    "route_topk",    "route_capacity", "route_active", "route_topk_bwd", "route_capacity_bwd",
    "route_drop",
    "permute_count", "permute_scan",   "permute_scatter", "permute_rows", "permute_bwd",
    "combine",       "combine_bwd",    "ffn_gateup",   "ffn_down",       "ffn_dA",
    "ffn_dX",        "ffn_dWd",        "ffn_dWg",      "ffn_dWu"};

hipEvent_t get_event() {
  if (!g_free.empty()) {
    hipEvent_t e = g_free.back();
    g_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Folds finished event pairs of one slot into its totals.  Waits for each stop event.
int32_t drain(Slot& s) {
  for (size_t i = 0; i < s.stop.size(); ++i) {
    DYNMO_HIP_TRY(hipEventSynchronize(s.stop[i]));
    float ms = 0.f;
    DYNMO_HIP_TRY(hipEventElapsedTime(&ms, s.start[i], s.stop[i]));
    s.total_ms += ms;
    s.launches += 1;
    g_free.push_back(s.start[i]);
    g_free.push_back(s.stop[i]);
  }
  s.start.clear();
  s.stop.clear();
  return DYNMO_OK;
}
}  // namespace

hipEvent_t profile_begin(KernelId id, hipStream_t st) {
  std::lock_guard<std::mutex> lk(g_mu);
  Slot& s = g_slots[id];
  if (s.start.size() >= kMaxPending) return nullptr;
  hipEvent_t a = get_event(), b = get_event();
  if (!a || !b) {
    if (a) g_free.push_back(a);
    if (b) g_free.push_back(b);
    return nullptr;
  }
  s.start.push_back(a);
  s.stop.push_back(b);
  (void)hipEventRecord(a, st);
  return b;
}

void profile_end(hipEvent_t stop, hipStream_t st) { (void)hipEventRecord(stop, st); }

}  // namespace dynmo

using namespace dynmo;

extern "C" int32_t dynmo_profile_enable(int32_t on) {
  g_profile_on.store(on != 0);
  return DYNMO_OK;
}

extern "C" int32_t dynmo_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (int i = 0; i < K_COUNT; ++i) {
    int32_t rc = drain(g_slots[i]);
    if (rc) return rc;
    g_slots[i].total_ms = 0.0;
    g_slots[i].launches = 0;
  }
  return DYNMO_OK;
}

extern "C" int32_t dynmo_profile_kernel_count(void) { return K_COUNT; }

extern "C" const char* dynmo_profile_kernel_name(int32_t id) {
  return (id >= 0 && id < K_COUNT) ? kNames[id] : nullptr;
}

extern "C" int32_t dynmo_profile_read(int32_t id, double* total_ms_host, int64_t* launches_host) {
  if (id < 0 || id >= K_COUNT || !total_ms_host || !launches_host) return DYNMO_EINVAL;
  std::lock_guard<std::mutex> lk(g_mu);
  int32_t rc = drain(g_slots[id]);
  if (rc) return rc;
  *total_ms_host = g_slots[id].total_ms;
  *launches_host = g_slots[id].launches;
  return DYNMO_OK;
}
