// Weighted scatter-combine of expert outputs back to token order, and its
// backward.  Both are HBM-bound row kernels: one wavefront per token, 16-byte
// accesses, fp32 arithmetic, slots summed in ascending order.
#include "common.h"
#include "profile.h"

namespace dynmo {

// Both kernels give one wavefront to a token and walk its row in groups of
// kUnroll x 64 sixteen-byte pieces: all loads of a group are issued before any of
// them is used, so each lane keeps (slots + 1) x kUnroll loads in flight.
constexpr int kUnroll = 4;

template <typename T, int MAXK>
__global__ __launch_bounds__(256) void combine_kernel(const u32x4* __restrict__ y_p, const int32_t* __restrict__ dst_pos,
                                                      const float* __restrict__ gate_w, const u32x4* __restrict__ base,
                                                      u32x4* __restrict__ out, int Tn, int k, int row_vecs) {
  constexpr int V = Elem<T>::kVec;
  const int lane = threadIdx.x & 63;
  const long t = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (t >= Tn) return;
  long src[MAXK];
  float w[MAXK];
  bool any = false;
#pragma unroll
  for (int s = 0; s < MAXK; ++s) {
    src[s] = -1;
    w[s] = 0.f;
    if (s < k) {
      const int p = dst_pos[t * k + s];
      if (p >= 0) {
        src[s] = (long)p * row_vecs;
        w[s] = gate_w[t * k + s];
        any = true;
      }
    }
  }
  const u32x4* brow = base ? base + t * row_vecs : nullptr;
  u32x4* orow = out + t * row_vecs;
  if (!any) {  // unrouted token: pass the base through (or zeros)
    for (int c = lane; c < row_vecs; c += 64) {
      u32x4 v = {0, 0, 0, 0};
      if (brow) v = brow[c];
      orow[c] = v;
    }
    return;
  }
  for (int c0 = lane; c0 < row_vecs; c0 += 64 * kUnroll) {
    u32x4 yv[MAXK][kUnroll], bv[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      bv[u] = u32x4{0, 0, 0, 0};
      if (brow && c0 + 64 * u < row_vecs) bv[u] = brow[c0 + 64 * u];
    }
#pragma unroll
    for (int s = 0; s < MAXK; ++s)
      if (src[s] >= 0) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
          if (c0 + 64 * u < row_vecs) yv[s][u] = y_p[src[s] + c0 + 64 * u];
      }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
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
          unpack16<T>(yv[s][u], f);
#pragma unroll
          for (int j = 0; j < V; ++j) acc[j] += w[s] * f[j];
        }
      orow[c0 + 64 * u] = pack16<T>(acc);
    }
  }
}

template <typename T, int MAXK>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const u32x4* __restrict__ dout, const u32x4* __restrict__ y_p,
                                                          const int32_t* __restrict__ dst_pos,
                                                          const float* __restrict__ gate_w, u32x4* __restrict__ dy_p,
                                                          float* __restrict__ dgate, int Tn, int k, int row_vecs) {
  constexpr int V = Elem<T>::kVec;
  const int lane = threadIdx.x & 63;
  const long t = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (t >= Tn) return;
  long row[MAXK];
  float w[MAXK];
  float dot[MAXK];
  bool any = false;
#pragma unroll
  for (int s = 0; s < MAXK; ++s) {
    row[s] = -1;
    w[s] = 0.f;
    dot[s] = 0.f;
    if (s < k) {
      const int p = dst_pos[t * k + s];
      if (p >= 0) {
        row[s] = (long)p * row_vecs;
        w[s] = gate_w[t * k + s];
        any = true;
      }
    }
  }
  if (any) {
    const u32x4* drow = dout + t * row_vecs;
    for (int c0 = lane; c0 < row_vecs; c0 += 64 * kUnroll) {
      u32x4 dv[kUnroll], yv[MAXK][kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        if (c0 + 64 * u < row_vecs) dv[u] = drow[c0 + 64 * u];
#pragma unroll
      for (int s = 0; s < MAXK; ++s)
        if (row[s] >= 0) {
#pragma unroll
          for (int u = 0; u < kUnroll; ++u)
            if (c0 + 64 * u < row_vecs) yv[s][u] = y_p[row[s] + c0 + 64 * u];
        }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        if (c0 + 64 * u >= row_vecs) continue;
        float d[V];
        unpack16<T>(dv[u], d);
#pragma unroll
        for (int s = 0; s < MAXK; ++s)
          if (row[s] >= 0) {
            float y[V], o[V];
            unpack16<T>(yv[s][u], y);
#pragma unroll
            for (int j = 0; j < V; ++j) {
              dot[s] += d[j] * y[j];
              o[j] = w[s] * d[j];
            }
            dy_p[row[s] + c0 + 64 * u] = pack16<T>(o);
          }
      }
    }
  }
#pragma unroll
  for (int s = 0; s < MAXK; ++s) {
    if (s < k) {
      float v = dot[s];
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
      if (lane == 0) dgate[t * k + s] = row[s] >= 0 ? v : 0.f;
    }
  }
}

template <typename T>
static int32_t launch_combine(const dynmo_desc* d, const void* y_p, const int32_t* dst_pos, const float* gate_w,
                              const void* base, void* out, hipStream_t st) {
  const int row_vecs = (int)((size_t)d->H * sizeof(T) / 16);
  const unsigned blocks = (unsigned)(((int64_t)d->T * 64 + 255) / 256);
#define DYNMO_COMBINE_LAUNCH(MAXK)                                                                              \
  DYNMO_TIMED_LAUNCH(K_COMBINE, st,                                                                             \
                     combine_kernel<T, MAXK><<<dim3(blocks), dim3(256), 0, st>>>(                               \
                         (const u32x4*)y_p, dst_pos, gate_w, (const u32x4*)base, (u32x4*)out, d->T, d->k, row_vecs))
  if (d->k == 1) {
    DYNMO_COMBINE_LAUNCH(1);
  } else if (d->k == 2) {
    DYNMO_COMBINE_LAUNCH(2);
  } else if (d->k <= 4) {
    DYNMO_COMBINE_LAUNCH(4);
  } else {
    DYNMO_COMBINE_LAUNCH(kMaxCombineSlots);
  }
#undef DYNMO_COMBINE_LAUNCH
  return DYNMO_OK;
}

template <typename T>
static int32_t launch_combine_bwd(const dynmo_desc* d, const void* dout, const void* y_p, const int32_t* dst_pos,
                                  const float* gate_w, void* dy_p, float* dgate, hipStream_t st) {
  const int row_vecs = (int)((size_t)d->H * sizeof(T) / 16);
  const unsigned blocks = (unsigned)(((int64_t)d->T * 64 + 255) / 256);
#define DYNMO_COMBINE_BWD_LAUNCH(MAXK)                                                                          \
  DYNMO_TIMED_LAUNCH(K_COMBINE_BWD, st,                                                                         \
                     combine_bwd_kernel<T, MAXK><<<dim3(blocks), dim3(256), 0, st>>>(                           \
                         (const u32x4*)dout, (const u32x4*)y_p, dst_pos, gate_w, (u32x4*)dy_p, dgate, d->T, d->k, row_vecs))
  if (d->k == 1) {
    DYNMO_COMBINE_BWD_LAUNCH(1);
  } else if (d->k == 2) {
    DYNMO_COMBINE_BWD_LAUNCH(2);
  } else if (d->k <= 4) {
    DYNMO_COMBINE_BWD_LAUNCH(4);
  } else {
    DYNMO_COMBINE_BWD_LAUNCH(kMaxCombineSlots);
  }
#undef DYNMO_COMBINE_BWD_LAUNCH
  return DYNMO_OK;
}

}  // namespace dynmo

using namespace dynmo;

extern "C" int32_t dynmo_combine(const dynmo_desc* d, const void* y_p, const int32_t* dst_pos, const float* gate_w,
                                 const void* base, void* out, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!y_p || !dst_pos || !gate_w || !out) return DYNMO_EINVAL;
  if (base == out) return DYNMO_EINVAL;
  if (misaligned16(y_p, base, out)) return DYNMO_EINVAL;
  if (d->k > kMaxCombineSlots) return DYNMO_EUNSUPPORTED;
  if (d->T == 0) return DYNMO_OK;
  hipStream_t st = (hipStream_t)stream;
  return d->dtype == DYNMO_BF16 ? launch_combine<bf16_t>(d, y_p, dst_pos, gate_w, base, out, st)
                                : launch_combine<float>(d, y_p, dst_pos, gate_w, base, out, st);
}

extern "C" int32_t dynmo_combine_bwd(const dynmo_desc* d, const void* dout, const void* y_p, const int32_t* dst_pos,
                                     const float* gate_w, void* dy_p, float* dgate, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!dout || !y_p || !dst_pos || !gate_w || !dy_p || !dgate) return DYNMO_EINVAL;
  if (misaligned16(dout, y_p, dy_p)) return DYNMO_EINVAL;
  if (d->k > kMaxCombineSlots) return DYNMO_EUNSUPPORTED;
  if (d->T == 0) return DYNMO_OK;
  hipStream_t st = (hipStream_t)stream;
  return d->dtype == DYNMO_BF16 ? launch_combine_bwd<bf16_t>(d, dout, y_p, dst_pos, gate_w, dy_p, dgate, st)
                                : launch_combine_bwd<float>(d, dout, y_p, dst_pos, gate_w, dy_p, dgate, st);
}
