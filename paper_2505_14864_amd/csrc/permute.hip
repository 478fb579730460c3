// Permutation of routed token rows into contiguous per-expert segments, and its
// backward.  The index part is a stable counting sort done without ordered
// atomics: per-chunk histograms, a scan over chunks, then an in-chunk stable rank
// from wavefront ballots.  The row movement is a token-centric copy: each source
// row is read once and written to its (up to k) destinations with 16-byte
// accesses.
#include <mutex>

#include "common.h"
#include "profile.h"

namespace dynmo {

constexpr int kChunkThreads = 256;
constexpr int kChunkPasses = 4;
constexpr int kChunk = kChunkThreads * kChunkPasses;  // slots per workgroup

// chunk_counts[c*E + e] = number of slots of expert e in chunk c
__global__ __launch_bounds__(kChunkThreads) void permute_count_kernel(const int32_t* __restrict__ expert_idx, int n_slots,
                                                                      int E, int32_t* __restrict__ chunk_counts) {
  __shared__ int cnt[kMaxExperts];
  if (threadIdx.x < E) cnt[threadIdx.x] = 0;
  __syncthreads();
  const int base = blockIdx.x * kChunk;
#pragma unroll
  for (int p = 0; p < kChunkPasses; ++p) {
    const int i = base + p * kChunkThreads + threadIdx.x;
    if (i < n_slots) {
      const int e = expert_idx[i];
      if (e >= 0 && e < E) atomicAdd(&cnt[e], 1);  // integer sum: order-independent
    }
  }
  __syncthreads();
  if (threadIdx.x < E) chunk_counts[blockIdx.x * E + threadIdx.x] = cnt[threadIdx.x];
}

// One workgroup of sixteen wavefronts.  Turns chunk_counts into chunk bases (in place) and
// writes seg_offsets[E+1].  A wavefront takes one expert at a time and walks that expert's
// chunks 64 at a time with a wavefront-wide prefix sum, so the serial depth is
// n_chunks / 64 steps per expert instead of n_chunks.
constexpr int kScanThreads = 1024;

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

__global__ __launch_bounds__(kScanThreads) void permute_scan_kernel(int32_t* __restrict__ chunk_counts, int n_chunks, int E,
                                                                    int32_t* __restrict__ seg_offsets) {
  constexpr int kWaves = kScanThreads / 64;
  __shared__ int total[kMaxExperts];
  __shared__ int seg[kMaxExperts + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int e = wave; e < E; e += kWaves) {
    int s = 0;
    for (int c = lane; c < n_chunks; c += 64) s += chunk_counts[c * E + e];
    s = wave_inclusive_scan(s, lane);
    if (lane == 63) total[e] = s;
  }
  __syncthreads();
  if (wave == 0) {  // exclusive prefix sum over the experts (E <= 64 = one wavefront)
    const int v = lane < E ? total[lane] : 0;
    const int inc = wave_inclusive_scan(v, lane);
    if (lane < E) seg[lane] = inc - v;
    if (lane == E - 1) seg[E] = inc;
  }
  __syncthreads();
  if (threadIdx.x <= E) seg_offsets[threadIdx.x] = seg[threadIdx.x];
  for (int e = wave; e < E; e += kWaves) {
    int run = seg[e];
    for (int c0 = 0; c0 < n_chunks; c0 += 64) {
      const int c = c0 + lane;
      const int v = c < n_chunks ? chunk_counts[c * E + e] : 0;
      const int inc = wave_inclusive_scan(v, lane);
      if (c < n_chunks) chunk_counts[c * E + e] = run + inc - v;
      run += __shfl(inc, 63, 64);
    }
  }
}

// Stable rank of every slot inside its chunk, added to the chunk base.
__global__ __launch_bounds__(kChunkThreads) void permute_scatter_kernel(const int32_t* __restrict__ expert_idx,
                                                                        int n_slots, int E,
                                                                        const int32_t* __restrict__ chunk_base,
                                                                        int32_t* __restrict__ src_slot,
                                                                        int32_t* __restrict__ dst_pos) {
  constexpr int kWaves = kChunkThreads / 64;
  __shared__ int run[kMaxExperts];             // rows of expert e already placed by earlier passes
  __shared__ int wave_cnt[kWaves][kMaxExperts];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  if (threadIdx.x < E) run[threadIdx.x] = chunk_base[blockIdx.x * E + threadIdx.x];
  __syncthreads();
  const int base = blockIdx.x * kChunk;
  for (int p = 0; p < kChunkPasses; ++p) {
    const int i = base + p * kChunkThreads + threadIdx.x;
    int e = -1;
    if (i < n_slots) {
      e = expert_idx[i];
      if (e >= E) e = -1;
    }
    // rank among lower lanes of this wavefront with the same expert
    int rank = 0;
    for (int q = 0; q < E; ++q) {
      const unsigned long long m = __ballot(e == q);
      if (e == q) rank = __popcll(m & ((1ull << lane) - 1ull));
      if (lane == q) wave_cnt[wv][q] = __popcll(m);
    }
    __syncthreads();
    if (e >= 0) {
      int pos = run[e] + rank;
      for (int w = 0; w < wv; ++w) pos += wave_cnt[w][e];
      dst_pos[i] = pos;
      src_slot[pos] = i;
    } else if (i < n_slots) {
      dst_pos[i] = -1;
    }
    __syncthreads();
    if (threadIdx.x < E) {
      int s = 0;
      for (int w = 0; w < kWaves; ++w) s += wave_cnt[w][threadIdx.x];
      run[threadIdx.x] += s;
    }
    __syncthreads();
  }
}

// One wavefront per token: read the row once, write it to each routed slot.
template <int MAXK>
__global__ __launch_bounds__(256) void permute_rows_kernel(const u32x4* __restrict__ x, const int32_t* __restrict__ dst_pos,
                                                           u32x4* __restrict__ x_p, int T, int k, int row_vecs) {
  const int lane = threadIdx.x & 63;
  const long t = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (t >= T) return;
  long dst[MAXK];
  bool any = false;
#pragma unroll
  for (int s = 0; s < MAXK; ++s) {
    dst[s] = -1;
    if (s < k) {
      const int p = dst_pos[t * k + s];
      if (p >= 0) {
        dst[s] = (long)p * row_vecs;
        any = true;
      }
    }
  }
  if (!any) return;
  const u32x4* src = x + t * row_vecs;
  for (int c = lane; c < row_vecs; c += 64 * 4) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (c + u * 64 < row_vecs) v[u] = src[c + u * 64];
#pragma unroll
    for (int s = 0; s < MAXK; ++s) {
      if (dst[s] >= 0) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (c + u * 64 < row_vecs) x_p[dst[s] + c + u * 64] = v[u];
      }
    }
  }
}

// dx[t] = dbase[t] + sum_s dx_p[dst_pos[t,s]]  (fp32 sum in ascending s).  One wavefront
// per token; the row is walked in groups of 4 x 64 pieces with all loads of a group
// issued before any is used.
template <typename T, int MAXK>
__global__ __launch_bounds__(256) void permute_bwd_kernel(const u32x4* __restrict__ dx_p, const int32_t* __restrict__ dst_pos,
                                                          const u32x4* __restrict__ dbase, u32x4* __restrict__ dx, int Tn,
                                                          int k, int row_vecs) {
  constexpr int V = Elem<T>::kVec;
  constexpr int U = 4;
  const int lane = threadIdx.x & 63;
  const long t = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (t >= Tn) return;
  long src[MAXK];
#pragma unroll
  for (int s = 0; s < MAXK; ++s) {
    src[s] = -1;
    if (s < k) {
      const int p = dst_pos[t * k + s];
      if (p >= 0) src[s] = (long)p * row_vecs;
    }
  }
  const u32x4* brow = dbase ? dbase + t * row_vecs : nullptr;
  u32x4* orow = dx + t * row_vecs;
  for (int c0 = lane; c0 < row_vecs; c0 += 64 * U) {
    u32x4 bv[U], xv[MAXK][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      bv[u] = u32x4{0, 0, 0, 0};
      if (brow && c0 + 64 * u < row_vecs) bv[u] = brow[c0 + 64 * u];
    }
#pragma unroll
    for (int s = 0; s < MAXK; ++s)
      if (src[s] >= 0) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (c0 + 64 * u < row_vecs) xv[s][u] = dx_p[src[s] + c0 + 64 * u];
      }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (c0 + 64 * u >= row_vecs) continue;
      float acc[V];
      if (brow) {
        unpack16<T>(bv[u], acc);
      } else {
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] = 0.f;
      }
#pragma unroll
      for (int s = 0; s < MAXK; ++s)
        if (src[s] >= 0) {
          float f[V];
          unpack16<T>(xv[s][u], f);
#pragma unroll
          for (int j = 0; j < V; ++j) acc[j] += f[j];
        }
      orow[c0 + 64 * u] = pack16<T>(acc);
    }
  }
}

static inline int n_chunks_of(const dynmo_desc* d) { return (int)(((int64_t)d->T * d->k + kChunk - 1) / kChunk); }

template <int MAXK>
static int32_t launch_rows(const dynmo_desc* d, const void* x, const int32_t* dst_pos, void* x_p, hipStream_t st) {
  const int row_vecs = (int)((size_t)d->H * elem_bytes(d->dtype) / 16);
  const unsigned blocks = (unsigned)(((int64_t)d->T * 64 + 255) / 256);
  DYNMO_TIMED_LAUNCH(K_PERMUTE_ROWS, st,
                     permute_rows_kernel<MAXK><<<dim3(blocks), dim3(256), 0, st>>>((const u32x4*)x, dst_pos, (u32x4*)x_p,
                                                                                   d->T, d->k, row_vecs));
  return DYNMO_OK;
}

template <typename T>
static int32_t launch_permute_bwd(const dynmo_desc* d, const void* dx_p, const int32_t* dst_pos, const void* dbase,
                                  void* dx, hipStream_t st) {
  const int row_vecs = (int)((size_t)d->H * sizeof(T) / 16);
  const unsigned blocks = (unsigned)(((int64_t)d->T * 64 + 255) / 256);
#define DYNMO_PERMUTE_BWD_LAUNCH(MAXK)                                                                          \
  DYNMO_TIMED_LAUNCH(K_PERMUTE_BWD, st,                                                                         \
                     permute_bwd_kernel<T, MAXK><<<dim3(blocks), dim3(256), 0, st>>>(                           \
                         (const u32x4*)dx_p, dst_pos, (const u32x4*)dbase, (u32x4*)dx, d->T, d->k, row_vecs))
  if (d->k == 1) {
    DYNMO_PERMUTE_BWD_LAUNCH(1);
  } else if (d->k == 2) {
    DYNMO_PERMUTE_BWD_LAUNCH(2);
  } else if (d->k <= 4) {
    DYNMO_PERMUTE_BWD_LAUNCH(4);
  } else if (d->k <= 8) {
    DYNMO_PERMUTE_BWD_LAUNCH(8);
  } else {
    DYNMO_PERMUTE_BWD_LAUNCH(kMaxExperts);
  }
#undef DYNMO_PERMUTE_BWD_LAUNCH
  return DYNMO_OK;
}

}  // namespace dynmo

using namespace dynmo;

extern "C" size_t dynmo_permute_workspace_bytes(const dynmo_desc* d) {
  if (check_desc(d)) return 0;
  // the chunk histograms, plus slack to align whatever address the caller hands over
  return align_up((size_t)(n_chunks_of(d) > 0 ? n_chunks_of(d) : 1) * d->E * sizeof(int32_t), 256) + 256;
}

namespace dynmo {
// The permutation proper; chunk_counts holds n_chunks * E ints of scratch (fully rewritten).
static int32_t permute_run(const dynmo_desc* d, const void* x, const int32_t* expert_idx, void* x_p, int32_t* seg_offsets,
                           int32_t* src_slot, int32_t* dst_pos, int32_t* chunk_counts, hipStream_t st) {
  const int n_slots = d->T * d->k;
  const int nc = n_chunks_of(d);
  if (nc > 0) {
    DYNMO_TIMED_LAUNCH(K_PERMUTE_COUNT, st,
                       permute_count_kernel<<<dim3(nc), dim3(kChunkThreads), 0, st>>>(expert_idx, n_slots, d->E,
                                                                                      chunk_counts));
  }
  DYNMO_TIMED_LAUNCH(K_PERMUTE_SCAN, st,
                     permute_scan_kernel<<<dim3(1), dim3(kScanThreads), 0, st>>>(chunk_counts, nc, d->E, seg_offsets));
  if (nc == 0) return DYNMO_OK;
  DYNMO_TIMED_LAUNCH(K_PERMUTE_SCATTER, st,
                     permute_scatter_kernel<<<dim3(nc), dim3(kChunkThreads), 0, st>>>(expert_idx, n_slots, d->E,
                                                                                      chunk_counts, src_slot, dst_pos));
  if (!x_p) return DYNMO_OK;  // indices only: the caller gathers the rows itself
  if (d->k <= 2) return launch_rows<2>(d, x, dst_pos, x_p, st);
  if (d->k <= 8) return launch_rows<8>(d, x, dst_pos, x_p, st);
  return launch_rows<kMaxExperts>(d, x, dst_pos, x_p, st);
}

static int32_t permute_check(const dynmo_desc* d, const void* x, const int32_t* expert_idx, void* x_p, int32_t* seg_offsets,
                             int32_t* src_slot, int32_t* dst_pos) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!expert_idx || !seg_offsets || !src_slot || !dst_pos || (x_p && !x)) return DYNMO_EINVAL;
  if (misaligned16(x, x_p)) return DYNMO_EINVAL;
  return DYNMO_OK;
}
}  // namespace dynmo

extern "C" int32_t dynmo_permute(const dynmo_desc* d, const void* x, const int32_t* expert_idx, void* x_p,
                                 int32_t* seg_offsets, int32_t* src_slot, int32_t* dst_pos, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  int32_t rc = permute_check(d, x, expert_idx, x_p, seg_offsets, src_slot, dst_pos);
  if (rc) return rc;
  if (!workspace) return DYNMO_EINVAL;
  if (workspace_bytes < dynmo_permute_workspace_bytes(d)) return DYNMO_EWORKSPACE;
  int32_t* chunk_counts = (int32_t*)align_up((size_t)workspace, 256);
  return permute_run(d, x, expert_idx, x_p, seg_offsets, src_slot, dst_pos, chunk_counts, (hipStream_t)stream);
}

// ---- the permutation for callers that cannot allocate ------------------------------
// The chunk histograms live in a file-scope device array instead of a caller workspace.
// Every device the library runs on holds its own copy at its own address, which is looked
// up once per device (with that device current) and used from then on; the array's name
// itself is only a host-side handle and is never passed to a kernel.
namespace dynmo {
constexpr size_t kStaticScratchInts = (size_t)1 << 18;  // 1 MiB: 4096 chunks of 1024 slots x 64 experts
static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

constexpr int kMaxScratchDevices = 64;
static std::mutex g_scratch_mutex;
static int32_t* g_scratch_ptr[kMaxScratchDevices] = {};

// the calling thread's current device's copy of `scratch`, or nullptr with *rc set
static int32_t* static_scratch(int32_t* rc) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    *rc = hip_fail(e);
    return nullptr;
  }
  if (dev < 0 || dev >= kMaxScratchDevices) {
    *rc = DYNMO_EUNSUPPORTED;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      *rc = hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol);
      return nullptr;
    }
    g_scratch_ptr[dev] = (int32_t*)ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace dynmo

extern "C" size_t dynmo_permute_static_max_slots(int32_t E) {
  if (E <= 0 || E > kMaxExperts) return 0;
  return kStaticScratchInts / (size_t)E * kChunk;
}

extern "C" int32_t dynmo_permute_static(const dynmo_desc* d, const void* x, const int32_t* expert_idx, void* x_p,
                                        int32_t* seg_offsets, int32_t* src_slot, int32_t* dst_pos, void* stream) {
  int32_t rc = permute_check(d, x, expert_idx, x_p, seg_offsets, src_slot, dst_pos);
  if (rc) return rc;
  if ((size_t)n_chunks_of(d) * d->E > kStaticScratchInts) return DYNMO_EWORKSPACE;  // beyond the fixed scratch
  int32_t* chunk_counts = static_scratch(&rc);
  if (!chunk_counts) return rc;
  // nothing to clear: the count kernel rewrites every histogram entry the later kernels read
  return permute_run(d, x, expert_idx, x_p, seg_offsets, src_slot, dst_pos, chunk_counts, (hipStream_t)stream);
}

namespace dynmo {
// kept[i] = expert_idx[i] if fewer than `capacity` earlier slots chose the same expert
// (the slot's rank inside its expert segment is its row minus the segment's first row)
__global__ void route_drop_kernel(const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ seg,
                                  const int32_t* __restrict__ dst_pos, int32_t* __restrict__ kept, int n_slots, int E,
                                  int capacity) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_slots) return;
  const int e = expert_idx[i];
  int out = -1;
  if (e >= 0 && e < E && dst_pos[i] - seg[e] < capacity) out = e;
  kept[i] = out;
}

static size_t drop_index_bytes(const dynmo_desc* d) {  // seg_offsets, src_slot, dst_pos of the ranking pass
  return align_up(((size_t)d->E + 1 + 2 * (size_t)d->T * d->k) * sizeof(int32_t), 256);
}
}  // namespace dynmo

extern "C" size_t dynmo_route_drop_workspace_bytes(const dynmo_desc* d) {
  if (check_desc(d)) return 0;
  return dynmo_permute_workspace_bytes(d) + drop_index_bytes(d) + 256;
}

extern "C" int32_t dynmo_route_drop(const dynmo_desc* d, const int32_t* expert_idx, int32_t capacity,
                                    int32_t* expert_idx_kept, void* workspace, size_t workspace_bytes, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!expert_idx || !expert_idx_kept || !workspace || capacity < 0) return DYNMO_EINVAL;
  if (workspace_bytes < dynmo_route_drop_workspace_bytes(d)) return DYNMO_EWORKSPACE;
  const int n_slots = d->T * d->k;
  if (n_slots == 0) return DYNMO_OK;
  // The stable ranking the permutation uses gives every slot its rank among the slots
  // of its expert in ascending slot order; a slot is kept while that rank is below the capacity.
  char* base = (char*)align_up((size_t)workspace, 256);
  int32_t* seg = (int32_t*)base;
  int32_t* src_slot = seg + d->E + 1;
  int32_t* dst_pos = src_slot + n_slots;
  void* ws = base + drop_index_bytes(d);
  rc = dynmo_permute(d, nullptr, expert_idx, nullptr, seg, src_slot, dst_pos, ws, dynmo_permute_workspace_bytes(d),
                     stream);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  DYNMO_TIMED_LAUNCH(K_ROUTE_DROP, st,
                     route_drop_kernel<<<dim3((n_slots + 255) / 256), dim3(256), 0, st>>>(
                         expert_idx, seg, dst_pos, expert_idx_kept, n_slots, d->E, capacity));
  return DYNMO_OK;
}

extern "C" int32_t dynmo_permute_bwd(const dynmo_desc* d, const void* dx_p, const int32_t* dst_pos, const void* dbase,
                                     void* dx, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!dx_p || !dst_pos || !dx) return DYNMO_EINVAL;
  if (misaligned16(dx_p, dbase, dx)) return DYNMO_EINVAL;
  if (d->T == 0) return DYNMO_OK;
  hipStream_t st = (hipStream_t)stream;
  return d->dtype == DYNMO_BF16 ? launch_permute_bwd<bf16_t>(d, dx_p, dst_pos, dbase, dx, st)
                                : launch_permute_bwd<float>(d, dx_p, dst_pos, dbase, dx, st);
}
