// Weighted scatter-combine of expert outputs back to token order, and its
// backward.  Both are HBM-bound row kernels: one wavefront per token, 16-byte
// accesses, fp32 arithmetic, slots summed in ascending order.
#include "common.h"
#include "profile.h"

namespace dynmo {

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const u32x4* __restrict__ y_p, const int32_t* __restrict__ dst_pos,
                                                      const float* __restrict__ gate_w, const u32x4* __restrict__ base,
                                                      u32x4* __restrict__ out, int Tn, int k, int row_vecs) {
  constexpr int V = Elem<T>::kVec;
  const int lane = threadIdx.x & 63;
  const long t = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (t >= Tn) return;
  long src[kMaxCombineSlots];
  float w[kMaxCombineSlots];
  bool any = false;
#pragma unroll
  for (int s = 0; s < kMaxCombineSlots; ++s) {
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
  if (!any) {  // unrouted token: pass the base through (or zeros)
    for (int c = lane; c < row_vecs; c += 64) {
      u32x4 v = {0, 0, 0, 0};
      if (base) v = base[t * row_vecs + c];
      out[t * row_vecs + c] = v;
    }
    return;
  }
  for (int c = lane; c < row_vecs; c += 64) {
    float acc[V];
    if (base) {
      unpack16<T>(base[t * row_vecs + c], acc);
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) acc[j] = 0.f;
    }
#pragma unroll
    for (int s = 0; s < kMaxCombineSlots; ++s) {
      if (src[s] >= 0) {
        float f[V];
        unpack16<T>(y_p[src[s] + c], f);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] += w[s] * f[j];
      }
    }
    out[t * row_vecs + c] = pack16<T>(acc);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const u32x4* __restrict__ dout, const u32x4* __restrict__ y_p,
                                                          const int32_t* __restrict__ dst_pos,
                                                          const float* __restrict__ gate_w, u32x4* __restrict__ dy_p,
                                                          float* __restrict__ dgate, int Tn, int k, int row_vecs) {
  constexpr int V = Elem<T>::kVec;
  const int lane = threadIdx.x & 63;
  const long t = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (t >= Tn) return;
  long row[kMaxCombineSlots];
  float w[kMaxCombineSlots];
  float dot[kMaxCombineSlots];
  bool any = false;
#pragma unroll
  for (int s = 0; s < kMaxCombineSlots; ++s) {
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
    for (int c = lane; c < row_vecs; c += 64) {
      float d[V];
      unpack16<T>(dout[t * row_vecs + c], d);
#pragma unroll
      for (int s = 0; s < kMaxCombineSlots; ++s) {
        if (row[s] >= 0) {
          float y[V], o[V];
          unpack16<T>(y_p[row[s] + c], y);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            dot[s] += d[j] * y[j];
            o[j] = w[s] * d[j];
          }
          dy_p[row[s] + c] = pack16<T>(o);
        }
      }
    }
  }
#pragma unroll
  for (int s = 0; s < kMaxCombineSlots; ++s) {
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
  DYNMO_TIMED_LAUNCH(K_COMBINE, st,
                     combine_kernel<T><<<dim3(blocks), dim3(256), 0, st>>>((const u32x4*)y_p, dst_pos, gate_w,
                                                                           (const u32x4*)base, (u32x4*)out, d->T, d->k,
                                                                           row_vecs));
  return DYNMO_OK;
}

template <typename T>
static int32_t launch_combine_bwd(const dynmo_desc* d, const void* dout, const void* y_p, const int32_t* dst_pos,
                                  const float* gate_w, void* dy_p, float* dgate, hipStream_t st) {
  const int row_vecs = (int)((size_t)d->H * sizeof(T) / 16);
  const unsigned blocks = (unsigned)(((int64_t)d->T * 64 + 255) / 256);
  DYNMO_TIMED_LAUNCH(K_COMBINE_BWD, st,
                     combine_bwd_kernel<T><<<dim3(blocks), dim3(256), 0, st>>>((const u32x4*)dout, (const u32x4*)y_p,
                                                                               dst_pos, gate_w, (u32x4*)dy_p, dgate, d->T,
                                                                               d->k, row_vecs));
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
  if (d->k > kMaxCombineSlots) return DYNMO_EUNSUPPORTED;
  if (d->T == 0) return DYNMO_OK;
  hipStream_t st = (hipStream_t)stream;
  return d->dtype == DYNMO_BF16 ? launch_combine_bwd<bf16_t>(d, dout, y_p, dst_pos, gate_w, dy_p, dgate, st)
                                : launch_combine_bwd<float>(d, dout, y_p, dst_pos, gate_w, dy_p, dgate, st);
}
