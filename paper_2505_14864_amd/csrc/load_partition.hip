// Load export (device -> host) and the host-side Partition balancer.
#include <math.h>

#include <vector>

#include "common.h"

using namespace dynmo;

extern "C" int32_t dynmo_layer_load(const dynmo_desc* d, const int32_t* seg_offsets, double cost_per_row,
                                    int32_t* counts_host, double* load_host, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!seg_offsets || !counts_host || !load_host) return DYNMO_EINVAL;
  int32_t seg[kMaxExperts + 1];
  hipStream_t st = (hipStream_t)stream;
  DYNMO_HIP_TRY(hipMemcpyAsync(seg, seg_offsets, sizeof(int32_t) * (d->E + 1), hipMemcpyDeviceToHost, st));
  DYNMO_HIP_TRY(hipStreamSynchronize(st));
  double rows = 0.0;
  for (int e = 0; e < d->E; ++e) {
    counts_host[e] = seg[e + 1] - seg[e];
    rows += (double)counts_host[e];
  }
  *load_host = rows * cost_per_row;
  return DYNMO_OK;
}

extern "C" int32_t dynmo_layer_load_begin(const dynmo_desc* d, const int32_t* seg_offsets, int32_t* seg_host,
                                          void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!seg_offsets || !seg_host) return DYNMO_EINVAL;
  DYNMO_HIP_TRY(hipMemcpyAsync(seg_host, seg_offsets, sizeof(int32_t) * (d->E + 1), hipMemcpyDeviceToHost,
                               (hipStream_t)stream));
  return DYNMO_OK;
}

extern "C" int32_t dynmo_layer_load_end(const dynmo_desc* d, const int32_t* seg_host, double cost_per_row,
                                        int32_t* counts_host, double* load_host) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!seg_host || !counts_host || !load_host) return DYNMO_EINVAL;
  double rows = 0.0;
  for (int e = 0; e < d->E; ++e) {
    counts_host[e] = seg_host[e + 1] - seg_host[e];
    rows += (double)counts_host[e];
  }
  *load_host = rows * cost_per_row;
  return DYNMO_OK;
}

namespace {

// Stage sums are differences of one running prefix sum, so that every candidate
// bottleneck is a value of the form prefix[j] - prefix[i].
struct Prefix {
  std::vector<double> p;
  Prefix(const double* loads, int L) : p((size_t)L + 1, 0.0) {
    for (int i = 0; i < L; ++i) p[i + 1] = p[i] + loads[i];
  }
  double sum(int i, int j) const { return p[j] - p[i]; }
};

// Linear probe: can the layers be covered by at most S contiguous stages whose
// sums do not exceed `cap` and that hold at most `max_layers` layers each?  Greedy left to right.
bool feasible(const Prefix& pre, int L, int S, double cap, int max_layers = 1 << 30) {
  int start = 0, used = 0;
  while (start < L) {
    if (used == S) return false;
    int end = start;
    while (end < L && end - start < max_layers && pre.sum(start, end + 1) <= cap) ++end;
    if (end == start) return false;  // a single layer exceeds cap
    start = end;
    ++used;
  }
  return true;
}

// Binary search on the bottleneck value.  Feasibility is monotone in the cap,
// and the optimum is itself a double (some prefix difference), so bisecting
// down to adjacent doubles lands exactly on it.
double optimal_bottleneck(const Prefix& pre, const double* loads, int L, int S) {
  double lo = 0.0;  // lo is infeasible unless it is the answer
  for (int i = 0; i < L; ++i) lo = fmax(lo, loads[i]);
  double hi = pre.sum(0, L);
  if (hi < lo) hi = lo;
  if (L == 0 || feasible(pre, L, S, lo)) return lo;
  while (true) {
    const double mid = lo + (hi - lo) * 0.5;
    if (!(mid > lo) || !(mid < hi)) break;
    if (feasible(pre, L, S, mid))
      hi = mid;
    else
      lo = mid;
  }
  return hi;
}

// The split: each stage takes as many layers as fit under both limits, but leaves one layer
// for every later stage (when there are at least as many layers as stages).  Returns the
// largest stage sum of the split.
double greedy_bounds(const Prefix& pre, int L, int S, double cap, int max_layers, int32_t* bounds) {
  int start = 0;
  bounds[0] = 0;
  double realised = 0.0;
  for (int s = 0; s < S; ++s) {
    int end;
    if (s == S - 1) {
      end = L;
    } else {
      const int limit = L >= S ? L - (S - s - 1) : L;
      end = start;
      while (end < limit && end - start < max_layers && pre.sum(start, end + 1) <= cap) ++end;
      if (L >= S && end == start) end = start + 1;
    }
    realised = fmax(realised, pre.sum(start, end));
    bounds[s + 1] = end;
    start = end;
  }
  return realised;
}

}  // namespace

extern "C" int32_t dynmo_partition(const double* loads_host, int32_t L, int32_t S, int32_t* bounds_host,
                                   double* bottleneck_host) {
  if (!loads_host || !bounds_host || !bottleneck_host || L < 0 || S <= 0) return DYNMO_EINVAL;
  for (int i = 0; i < L; ++i)
    if (!(loads_host[i] >= 0.0) || !isfinite(loads_host[i])) return DYNMO_EINVAL;
  Prefix pre(loads_host, L);
  const double best = optimal_bottleneck(pre, loads_host, L, S);
  *bottleneck_host = greedy_bounds(pre, L, S, best, 1 << 30, bounds_host);
  return DYNMO_OK;
}

extern "C" int32_t dynmo_partition_shadow(const double* loads_host, const int32_t* shadow_host, int32_t L, int32_t S,
                                          int32_t* bounds_host, double* bottleneck_host, int32_t* max_layers_host) {
  if (!loads_host || !bounds_host || !bottleneck_host || !max_layers_host || L < 0 || S <= 0) return DYNMO_EINVAL;
  for (int i = 0; i < L; ++i)
    if (!(loads_host[i] >= 0.0) || !isfinite(loads_host[i])) return DYNMO_EINVAL;
  // a shadow layer keeps its place and its memory but adds no load
  std::vector<double> eff(loads_host, loads_host + L);
  if (shadow_host)
    for (int i = 0; i < L; ++i)
      if (shadow_host[i]) eff[i] = 0.0;
  Prefix pre(eff.data(), L);
  const double best = optimal_bottleneck(pre, eff.data(), L, S);
  // Second criterion: the fewest layers on the fullest stage among the splits that keep the
  // optimal bottleneck.  Feasibility is monotone in that count too.
  int lo = L == 0 ? 0 : (L + S - 1) / S, hi = L;  // lo may be infeasible, hi is feasible
  while (lo < hi) {
    const int mid = lo + (hi - lo) / 2;
    if (feasible(pre, L, S, best, mid))
      hi = mid;
    else
      lo = mid + 1;
  }
  *bottleneck_host = greedy_bounds(pre, L, S, best, hi, bounds_host);
  int most = 0;
  for (int s = 0; s < S; ++s) most = bounds_host[s + 1] - bounds_host[s] > most ? bounds_host[s + 1] - bounds_host[s] : most;
  *max_layers_host = most;
  return DYNMO_OK;
}

extern "C" int32_t dynmo_uniform_bounds(int32_t L, int32_t S, int32_t* bounds_host) {
  if (!bounds_host || L < 0 || S <= 0) return DYNMO_EINVAL;
  const int base = L / S, rem = L % S;
  bounds_host[0] = 0;
  for (int s = 0; s < S; ++s) bounds_host[s + 1] = bounds_host[s] + base + (s < rem ? 1 : 0);
  return DYNMO_OK;
}

extern "C" int32_t dynmo_stage_loads(const double* loads_host, int32_t L, const int32_t* bounds_host, int32_t S,
                                     double* stage_loads_host) {
  if (!loads_host || !bounds_host || !stage_loads_host || L < 0 || S <= 0) return DYNMO_EINVAL;
  if (bounds_host[0] != 0 || bounds_host[S] != L) return DYNMO_EINVAL;
  for (int s = 0; s < S; ++s)
    if (bounds_host[s] > bounds_host[s + 1]) return DYNMO_EINVAL;
  for (int s = 0; s < S; ++s) {
    double acc = 0.0;
    for (int i = bounds_host[s]; i < bounds_host[s + 1]; ++i) acc += loads_host[i];
    stage_loads_host[s] = acc;
  }
  return DYNMO_OK;
}

extern "C" int32_t dynmo_imbalance(const double* stage_loads_host, int32_t S, double* imbalance_host) {
  if (!stage_loads_host || !imbalance_host || S <= 0) return DYNMO_EINVAL;
  double mx = stage_loads_host[0], mn = stage_loads_host[0], sum = 0.0;
  for (int s = 0; s < S; ++s) {
    mx = fmax(mx, stage_loads_host[s]);
    mn = fmin(mn, stage_loads_host[s]);
    sum += stage_loads_host[s];
  }
  if (!(sum > 0.0)) return DYNMO_EINVAL;
  *imbalance_host = (mx - mn) / (sum / S);
  return DYNMO_OK;
}

// ---- diffusion balancer -------------------------------------------------------
namespace {
double potential_of(const double* x, int S) {
  double phi = 0.0;
  for (int u = 0; u < S; ++u)
    for (int v = u + 1; v < S; ++v) phi += fabs(x[u] - x[v]);
  return phi;
}

double range_sum(const double* a, int begin, int end) {
  double acc = 0.0;
  for (int i = begin; i < end; ++i) acc += a[i];
  return acc;
}
}  // namespace

extern "C" int32_t dynmo_potential(const double* stage_loads_host, int32_t S, double* phi_host) {
  if (!stage_loads_host || !phi_host || S <= 0) return DYNMO_EINVAL;
  *phi_host = potential_of(stage_loads_host, S);
  return DYNMO_OK;
}

extern "C" int32_t dynmo_diffusion(const double* loads_host, int32_t L, int32_t S, int32_t* bounds_host,
                                   const double* layer_mem_host, double max_mem, double gamma, int32_t max_rounds,
                                   int32_t* rounds_host, double* phi_host) {
  if (!loads_host || !bounds_host || !rounds_host || !phi_host || L < 0 || S <= 0 || max_rounds < 0)
    return DYNMO_EINVAL;
  if (bounds_host[0] != 0 || bounds_host[S] != L) return DYNMO_EINVAL;
  for (int s = 0; s < S; ++s)
    if (bounds_host[s] > bounds_host[s + 1]) return DYNMO_EINVAL;
  for (int i = 0; i < L; ++i)
    if (!(loads_host[i] >= 0.0) || !isfinite(loads_host[i])) return DYNMO_EINVAL;
  std::vector<double> x(S), trial(S);
  for (int s = 0; s < S; ++s) x[s] = range_sum(loads_host, bounds_host[s], bounds_host[s + 1]);
  double phi = potential_of(x.data(), S);
  phi_host[0] = phi;
  int rounds = 0;
  while (rounds < max_rounds && !(phi <= gamma)) {
    // every single-layer transfer across a stage boundary; keep the one that lowers phi most
    double best_gain = 0.0, best_phi = phi;
    int best_boundary = -1, best_step = 0;
    for (int i = 1; i < S; ++i) {
      for (int dir = 0; dir < 2; ++dir) {
        const bool to_right = dir == 0;  // last layer of stage i-1 goes to stage i, else the reverse
        const int src = to_right ? i - 1 : i, dst = to_right ? i : i - 1;
        const int layer = to_right ? bounds_host[i] - 1 : bounds_host[i];
        if (bounds_host[src + 1] - bounds_host[src] <= 1) continue;
        if (layer_mem_host &&
            range_sum(layer_mem_host, bounds_host[dst], bounds_host[dst + 1]) + layer_mem_host[layer] > max_mem)
          continue;
        // stage sums of the trial assignment, each summed over its layers in order
        trial = x;
        const int nb = bounds_host[i] + (to_right ? -1 : 1);
        trial[i - 1] = range_sum(loads_host, bounds_host[i - 1], nb);
        trial[i] = range_sum(loads_host, nb, bounds_host[i + 1]);
        const double t_phi = potential_of(trial.data(), S);
        const double gain = phi - t_phi;
        if (gain > 0.0 && (best_boundary < 0 || gain > best_gain)) {
          best_gain = gain;
          best_phi = t_phi;
          best_boundary = i;
          best_step = to_right ? -1 : 1;
        }
      }
    }
    if (best_boundary < 0) break;
    bounds_host[best_boundary] += best_step;
    x[best_boundary - 1] = range_sum(loads_host, bounds_host[best_boundary - 1], bounds_host[best_boundary]);
    x[best_boundary] = range_sum(loads_host, bounds_host[best_boundary], bounds_host[best_boundary + 1]);
    phi = best_phi;
    ++rounds;
  }
  *rounds_host = rounds;
  phi_host[1] = phi;
  return DYNMO_OK;
}

// ---- re-pack ----------------------------------------------------------------------
// Consolidation onto fewer workers (Sec. 3.4).  Workers are visited in order; a worker that
// is still in use is folded, whole, into the first later worker in use that has room for
// everything it holds, as long as more workers are in use than wanted.  A worker that has
// been emptied neither gives nor takes again.  The walk records one merge per emptied
// worker and stops as soon as the wanted count is reached; the per-layer transfer list the
// caller asked for is written from those records at the end.
namespace {
struct Merge {
  int32_t from, into, layers;
};
}  // namespace

extern "C" int32_t dynmo_repack(int32_t n_workers, int32_t* active_host, double* mem_usage_host,
                                int32_t* num_layers_host, int32_t target_num_workers, double max_mem,
                                int32_t* transfers_host, int32_t capacity, int32_t* n_transfers_host) {
  if (!active_host || !mem_usage_host || !num_layers_host || !n_transfers_host || n_workers < 0 || capacity < 0 ||
      (capacity > 0 && !transfers_host))
    return DYNMO_EINVAL;
  for (int w = 0; w < n_workers; ++w)
    if (num_layers_host[w] < 0) return DYNMO_EINVAL;
  // Works on copies, so that a transfer list that does not fit leaves the caller's arrays untouched.
  std::vector<char> in_use(n_workers);
  std::vector<double> held(mem_usage_host, mem_usage_host + n_workers);
  std::vector<int32_t> layers(num_layers_host, num_layers_host + n_workers);
  int n_in_use = 0;
  for (int w = 0; w < n_workers; ++w) n_in_use += (in_use[w] = active_host[w] != 0) ? 1 : 0;
  std::vector<Merge> merges;
  int64_t n_moves = 0;
  for (int w = 0; w < n_workers && n_in_use > target_num_workers; ++w) {
    if (!in_use[w]) continue;
    int host = -1;  // first fit among the later workers
    for (int c = w + 1; c < n_workers && host < 0; ++c)
      if (in_use[c] && held[w] + held[c] < max_mem) host = c;
    if (host < 0) continue;
    merges.push_back({w, host, layers[w]});
    n_moves += layers[w];
    in_use[w] = 0;
    --n_in_use;
    held[host] += held[w];
    layers[host] += layers[w];
  }
  *n_transfers_host = (int32_t)n_moves;
  if (n_moves > capacity) return DYNMO_EWORKSPACE;
  int32_t* out = transfers_host;
  for (const Merge& m : merges)
    for (int32_t l = 0; l < m.layers; ++l) {
      *out++ = m.from;
      *out++ = m.into;
      *out++ = l;
    }
  for (int w = 0; w < n_workers; ++w) {
    if (!in_use[w]) active_host[w] = 0;
    mem_usage_host[w] = held[w];
    num_layers_host[w] = layers[w];
  }
  return DYNMO_OK;
}
