// Two reference kernels that measure what the device can reach, for judging the
// library's kernels against the machine rather than against data-sheet numbers:
// a register-resident bf16 MFMA loop (no memory traffic at all) and a plain
// streaming copy (16 bytes per lane, four independent loads in flight).
#include "common.h"

namespace dynmo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kPeakBlocks = 256, kPeakThreads = 512, kPeakAcc = 16;

// Eight wavefronts per workgroup (two per SIMD), sixteen independent 16 x 16 accumulator
// blocks per wavefront (two A fragments x eight B fragments, the instruction and the
// operand reuse of the grouped GEMM's k loop): every MFMA has its operands in registers and
// depends only on the MFMA issued sixteen instructions earlier.  The operands are either
// fixed small numbers (few bits change between MFMAs: the least power the loop can draw) or
// fragments taken from the caller's buffer (random data makes the loop draw what a real
// product draws, and the clock follows).
__global__ __launch_bounds__(kPeakThreads, 1) void peak_mfma_kernel(const u32x4* __restrict__ operands,
                                                                    float* __restrict__ sink, int iters) {
  bf16x8_t a[2], b[8];
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    if (operands) {
      // eight 1 KiB fragments in the buffer: 0, 1 feed A; 4..7, then 2, 3 and 4, 5 with the lanes rotated, feed B
      if (q < 2) a[q] = __builtin_bit_cast(bf16x8_t, operands[q * 64 + lane]);
      const int slot = q < 4 ? 4 + q : q - 2;
      b[q] = __builtin_bit_cast(bf16x8_t, operands[slot * 64 + ((lane + (q >= 6 ? 32 : 0)) & 63)]);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (q < 2) a[q][j] = (__bf16)(0.001f * lane + j);
        b[q][j] = (__bf16)(0.5f * j);
      }
    }
  }
  f32x4_t acc[kPeakAcc];
#pragma unroll
  for (int i = 0; i < kPeakAcc; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kPeakAcc; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i >> 3], b[i & 7], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kPeakAcc; ++i) s += acc[i][0];
  sink[(size_t)blockIdx.x * kPeakThreads + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void peak_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  u32x4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i + u * 256 < n) v[u] = src[i + u * 256];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i + u * 256 < n) dst[i + u * 256] = v[u];
}

}  // namespace dynmo

using namespace dynmo;

extern "C" int32_t dynmo_peak_mfma_bf16(int32_t iters, const void* operands, float* sink, double* flops_host,
                                        void* stream) {
  if (iters <= 0 || !sink || !flops_host) return DYNMO_EINVAL;
  peak_mfma_kernel<<<dim3(kPeakBlocks), dim3(kPeakThreads), 0, (hipStream_t)stream>>>((const u32x4*)operands, sink,
                                                                                      iters);
  DYNMO_LAUNCH_CHECK();
  // one 16x16x32 MFMA = 2 * 16 * 16 * 32 flop per wavefront
  *flops_host = (double)kPeakBlocks * (kPeakThreads / 64) * (double)iters * kPeakAcc * 16384.0;
  return DYNMO_OK;
}

extern "C" int32_t dynmo_peak_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes % 16) return DYNMO_EINVAL;
  const size_t n = bytes / 16;
  if (n == 0) return DYNMO_OK;
  if ((n + 1023) / 1024 > 0x7fffffffu) return DYNMO_EUNSUPPORTED;
  peak_copy_kernel<<<dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, (hipStream_t)stream>>>((const u32x4*)src,
                                                                                              (u32x4*)dst, n);
  DYNMO_LAUNCH_CHECK();
  return DYNMO_OK;
}
