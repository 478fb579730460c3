// Shared host/device helpers for the gfx950 kernels: status handling, descriptor
// checks, bf16 conversion and 16-byte vector access.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dynmo.h"

namespace dynmo {

extern thread_local int32_t g_last_hip_error;

inline int32_t hip_fail(hipError_t e) {
  g_last_hip_error = (int32_t)e;
  return DYNMO_EHIP;
}

#define DYNMO_HIP_TRY(expr)                                \
  do {                                                     \
    hipError_t _e = (expr);                                \
    if (_e != hipSuccess) return ::dynmo::hip_fail(_e);    \
  } while (0)

// Launch check: hipGetLastError after a <<<>>> launch.
#define DYNMO_LAUNCH_CHECK() DYNMO_HIP_TRY(hipGetLastError())

constexpr int kMaxExperts = 64;
constexpr int kMaxCombineSlots = 8;

inline int32_t check_desc(const dynmo_desc* d) {
  if (!d) return DYNMO_EINVAL;
  if (d->T < 0 || d->H <= 0 || d->F <= 0 || d->E <= 0 || d->k <= 0) return DYNMO_EINVAL;
  if (d->k > d->E) return DYNMO_EINVAL;
  if (d->dtype != DYNMO_F32 && d->dtype != DYNMO_BF16) return DYNMO_EINVAL;
  if (d->E > kMaxExperts) return DYNMO_EUNSUPPORTED;
  if ((int64_t)d->T * d->k >= (int64_t)1 << 30) return DYNMO_EUNSUPPORTED;
  if (d->dtype == DYNMO_BF16 && ((d->H % 8) || (d->F % 8))) return DYNMO_EUNSUPPORTED;
  if (d->dtype == DYNMO_F32 && (d->H % 4)) return DYNMO_EUNSUPPORTED;  // rows move in 16-byte pieces
  return DYNMO_OK;
}

// Row data moves in 16-byte pieces: true if any of the pointers (null ones aside) is not
// 16-byte aligned.
template <typename... P>
inline bool misaligned16(P... ptrs) {
  return (((uintptr_t)(const void*)ptrs | ...) & 15) != 0;
}

inline size_t elem_bytes(int32_t dtype) { return dtype == DYNMO_BF16 ? 2 : 4; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

typedef uint16_t bf16_t;  // raw bfloat16 bits
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte access

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// fp32 -> bf16, round to nearest even, with the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kVec = 4;  // elements per 16 bytes
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <>
struct Elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 16-byte chunk <-> float lanes
template <typename T>
__device__ __forceinline__ void unpack16(const u32x4& v, float* f);
template <>
__device__ __forceinline__ void unpack16<float>(const u32x4& v, float* f) {
  f[0] = __uint_as_float(v.x);
  f[1] = __uint_as_float(v.y);
  f[2] = __uint_as_float(v.z);
  f[3] = __uint_as_float(v.w);
}
template <>
__device__ __forceinline__ void unpack16<bf16_t>(const u32x4& v, float* f) {
  f[0] = __uint_as_float(v.x << 16);
  f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16);
  f[3] = __uint_as_float(v.y & 0xffff0000u);
  f[4] = __uint_as_float(v.z << 16);
  f[5] = __uint_as_float(v.z & 0xffff0000u);
  f[6] = __uint_as_float(v.w << 16);
  f[7] = __uint_as_float(v.w & 0xffff0000u);
}
template <typename T>
__device__ __forceinline__ u32x4 pack16(const float* f);
template <>
__device__ __forceinline__ u32x4 pack16<float>(const float* f) {
  u32x4 v;
  v.x = __float_as_uint(f[0]);
  v.y = __float_as_uint(f[1]);
  v.z = __float_as_uint(f[2]);
  v.w = __float_as_uint(f[3]);
  return v;
}
template <>
__device__ __forceinline__ u32x4 pack16<bf16_t>(const float* f) {
  u32x4 v;
  v.x = pack_bf16x2(f[0], f[1]);
  v.y = pack_bf16x2(f[2], f[3]);
  v.z = pack_bf16x2(f[4], f[5]);
  v.w = pack_bf16x2(f[6], f[7]);
  return v;
}

__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + __expf(-z)); }

}  // namespace dynmo
