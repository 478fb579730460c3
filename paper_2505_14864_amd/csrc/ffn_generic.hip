// Grouped SwiGLU FFN, shape-generic kernels: fp32 everywhere, and bf16 for shapes
// the MFMA kernels do not take.  A 64x64 output tile per workgroup, K staged
// through LDS in steps of 16, a 4x4 register block per thread, fp32 accumulate.
// Operands are addressed with explicit (row, k) element strides so the same tile
// loop serves X W^T, dY W, and the token-contracted dY^T A products.
#include "common.h"
#include "ffn.h"
#include "profile.h"

namespace dynmo {

constexpr int GT = 64;  // tile rows and columns
constexpr int GK = 16;  // k step

// S[kk][r] = base[row(row0+r)*rs + (k0+kk)*ks], zero outside [.., row_end) x [.., k_end).
// row(i) = i, or rowmap[i] / rowdiv when the rows are gathered through an index
// (K-contiguous operands only).  The thread mapping follows whichever stride is 1
// so that loads coalesce.
template <typename T>
__device__ __forceinline__ void stage_tile(float (*S)[GT + 1], const T* __restrict__ base, long rs, long ks, int row0,
                                           int row_end, int k0, int k_end, const int32_t* __restrict__ rowmap = nullptr,
                                           int rowdiv = 1) {
  const int tid = threadIdx.x;
  if (ks == 1) {
    const int kk = tid % GK;
#pragma unroll
    for (int j = 0; j < GT / (256 / GK); ++j) {
      const int r = tid / GK + j * (256 / GK);
      float v = 0.f;
      if (row0 + r < row_end && k0 + kk < k_end) {
        const long row = rowmap ? rowmap[row0 + r] / rowdiv : row0 + r;
        v = Elem<T>::load(base + row * rs + (long)(k0 + kk));
      }
      S[kk][r] = v;
    }
  } else {
    const int r = tid % GT;
#pragma unroll
    for (int j = 0; j < GK / (256 / GT); ++j) {
      const int kk = tid / GT + j * (256 / GT);
      float v = 0.f;
      if (row0 + r < row_end && k0 + kk < k_end) v = Elem<T>::load(base + (long)(row0 + r) * rs + (long)(k0 + kk) * ks);
      S[kk][r] = v;
    }
  }
}

// acc[i][j] += sum_k A(m0+ty*4+i, k) * B(n0+tx*4+j, k) over k in [k_begin, k_end)
template <typename T>
__device__ __forceinline__ void mac_phase(float (&acc)[4][4], const T* A, long a_rs, long a_ks, int m0, int m_end,
                                          const T* B, long b_rs, long b_ks, int n0, int n_end, int k_begin, int k_end,
                                          float (*As)[GT + 1], float (*Bs)[GT + 1],
                                          const int32_t* __restrict__ a_rowmap = nullptr, int a_rowdiv = 1) {
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  for (int k0 = k_begin; k0 < k_end; k0 += GK) {
    stage_tile<T>(As, A, a_rs, a_ks, m0, m_end, k0, k_end, a_rowmap, a_rowdiv);
    stage_tile<T>(Bs, B, b_rs, b_ks, n0, n_end, k0, k_end);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
}

// G = X Wg^T, U = X Wu^T, A = silu(G) U for one 64x64 tile of one expert segment.
// With `gather`, row p of X is x_p[gather[p] / gather_div] (rows fetched from the
// token-ordered input through the slot index).
template <typename T>
__global__ __launch_bounds__(256) void gateup_generic_kernel(const T* __restrict__ x_p, const int32_t* __restrict__ seg,
                                                             const T* __restrict__ Wg, const T* __restrict__ Wu,
                                                             T* __restrict__ G, T* __restrict__ U, T* __restrict__ A, int E,
                                                             int H, int F, const int32_t* __restrict__ gather,
                                                             int gather_div) {
  __shared__ float As[GK][GT + 1], Bs[GK][GT + 1];
  int e, m0, m_end;
  if (!find_m_tile(seg, E, blockIdx.y, GT, &e, &m0, &m_end)) return;
  const int n0 = blockIdx.x * GT;
  float accG[4][4] = {}, accU[4][4] = {};
  mac_phase<T>(accG, x_p, H, 1, m0, m_end, Wg + (long)e * F * H, H, 1, n0, F, 0, H, As, Bs, gather, gather_div);
  mac_phase<T>(accU, x_p, H, 1, m0, m_end, Wu + (long)e * F * H, H, 1, n0, F, 0, H, As, Bs, gather, gather_div);
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= m_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= F) continue;
      const float g = accG[i][j], u = accU[i][j];
      Elem<T>::store(G + (long)m * F + n, g);
      Elem<T>::store(U + (long)m * F + n, u);
      Elem<T>::store(A + (long)m * F + n, g * sigmoidf_(g) * u);
    }
  }
}

enum { EPI_STORE = 0, EPI_SWIGLU_BWD = 1 };

// Segmented-M GEMM: C[m, n] = sum_k A1(m,k) B1_e(n,k) (+ sum_k A2(m,k) B2_e(n,k)).
// B operands are per expert: element (n, k) of expert e at B + e*b_es + n*b_rs + k*b_ks.
template <typename T, int EPI>
__global__ __launch_bounds__(256) void seg_gemm_generic_kernel(const int32_t* __restrict__ seg, int E, int N, int K,
                                                               const T* __restrict__ A1, const T* __restrict__ B1,
                                                               const T* __restrict__ A2, const T* __restrict__ B2, long a_rs,
                                                               long b_es, long b_rs, long b_ks, T* __restrict__ C,
                                                               const T* __restrict__ Gs, const T* __restrict__ Us,
                                                               T* __restrict__ dG, T* __restrict__ dU, T* __restrict__ Aout,
                                                               const int32_t* __restrict__ scatter,
                                                               const float* __restrict__ scale, const T* res, T* out) {
  __shared__ float As[GK][GT + 1], Bs[GK][GT + 1];
  int e, m0, m_end;
  if (!find_m_tile(seg, E, blockIdx.y, GT, &e, &m0, &m_end)) return;
  const int n0 = blockIdx.x * GT;
  float acc[4][4] = {};
  mac_phase<T>(acc, A1, a_rs, 1, m0, m_end, B1 + (long)e * b_es, b_rs, b_ks, n0, N, 0, K, As, Bs);
  if (A2) mac_phase<T>(acc, A2, a_rs, 1, m0, m_end, B2 + (long)e * b_es, b_rs, b_ks, n0, N, 0, K, As, Bs);
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= m_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      const long o = (long)m * N + n;
      if (EPI == EPI_STORE) {
        if (C) Elem<T>::store(C + o, acc[i][j]);
        if (scatter) {  // folded combine of a one-slot layer
          const int token = scatter[m];
          const long ot = (long)token * N + n;
          Elem<T>::store(out + ot, (res ? Elem<T>::load(res + ot) : 0.f) + (scale ? scale[token] : 1.f) * acc[i][j]);
        }
      } else {
        const float g = Elem<T>::load(Gs + o), u = Elem<T>::load(Us + o);
        float a, dg, du;
        swiglu_bwd(acc[i][j], g, u, &a, &dg, &du);
        Elem<T>::store(Aout + o, a);
        Elem<T>::store(dG + o, dg);
        Elem<T>::store(dU + o, du);
      }
    }
  }
}

// dW[e][m, n] = sum over rows p of expert e of A[p, m] * B[p, n]   (zeros if no rows)
template <typename T>
__global__ __launch_bounds__(256) void dw_generic_kernel(const int32_t* __restrict__ seg, int M, int N,
                                                         const T* __restrict__ A, const T* __restrict__ B,
                                                         T* __restrict__ dW) {
  __shared__ float As[GK][GT + 1], Bs[GK][GT + 1];
  const int e = blockIdx.z;
  const int k_begin = seg[e], k_end = seg[e + 1];
  const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
  float acc[4][4] = {};
  mac_phase<T>(acc, A, 1, M, m0, M, B, 1, N, n0, N, k_begin, k_end, As, Bs);
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  T* out = dW + (long)e * M * N;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < N) Elem<T>::store(out + (long)m * N + n, acc[i][j]);
    }
  }
}

template <typename T>
static int32_t fwd_generic_t(const dynmo_desc* d, const void* x_p, const int32_t* gather, const int32_t* seg,
                             const void* Wg, const void* Wu, const void* Wd, void* y_p, void* G, void* U, void* A,
                             const FoldedCombine* fc, hipStream_t st) {
  const int m_tiles = max_m_tiles(d, GT);
  if (m_tiles == 0) return DYNMO_OK;
  const long FH = (long)d->F * d->H;
  DYNMO_TIMED_LAUNCH(K_FFN_GATEUP, st, gateup_generic_kernel<T><<<dim3((d->F + GT - 1) / GT, m_tiles), dim3(256), 0, st>>>(
      (const T*)x_p, seg, (const T*)Wg, (const T*)Wu, (T*)G, (T*)U, (T*)A, d->E, d->H, d->F, gather, d->k));
  // Y = A Wd^T : B(n=h, k=f) = Wd[e][h*F + f]
  DYNMO_TIMED_LAUNCH(K_FFN_DOWN, st, seg_gemm_generic_kernel<T, EPI_STORE><<<dim3((d->H + GT - 1) / GT, m_tiles), dim3(256), 0, st>>>(
      seg, d->E, d->H, d->F, (const T*)A, (const T*)Wd, nullptr, nullptr, d->F, FH, d->F, 1, (T*)y_p, nullptr, nullptr,
      nullptr, nullptr, nullptr, fc ? fc->scatter : nullptr, fc ? fc->scale : nullptr, fc ? (const T*)fc->res : nullptr,
      fc ? (T*)fc->out : nullptr));
  return DYNMO_OK;
}

template <typename T>
static int32_t bwd_generic_t(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G, const void* U,
                             const int32_t* seg, const void* Wg, const void* Wu, const void* Wd, void* dx_p, void* dWg,
                             void* dWu, void* dWd, void* dG, void* dU, void* A, const FoldedCombine* fc, hipStream_t st) {
  const int m_tiles = max_m_tiles(d, GT);
  const long FH = (long)d->F * d->H;
  const unsigned tf = (d->F + GT - 1) / GT, th = (d->H + GT - 1) / GT;
  if (m_tiles > 0) {
    // dA = dY Wd : B(n=f, k=h) = Wd[e][h*F + f]; epilogue gives A, dG, dU
    DYNMO_TIMED_LAUNCH(K_FFN_DA, st, seg_gemm_generic_kernel<T, EPI_SWIGLU_BWD><<<dim3(tf, m_tiles), dim3(256), 0, st>>>(
        seg, d->E, d->F, d->H, (const T*)dy_p, (const T*)Wd, nullptr, nullptr, d->H, FH, 1, d->F, nullptr, (const T*)G,
        (const T*)U, (T*)dG, (T*)dU, (T*)A, nullptr, nullptr, nullptr, nullptr));
    // dX = dG Wg + dU Wu : B(n=h, k=f) = W[e][f*H + h]
    DYNMO_TIMED_LAUNCH(K_FFN_DX, st, seg_gemm_generic_kernel<T, EPI_STORE><<<dim3(th, m_tiles), dim3(256), 0, st>>>(
        seg, d->E, d->H, d->F, (const T*)dG, (const T*)Wg, (const T*)dU, (const T*)Wu, d->F, FH, 1, d->H, (T*)dx_p, nullptr,
        nullptr, nullptr, nullptr, nullptr, fc ? fc->scatter : nullptr, fc ? fc->scale : nullptr,
        fc ? (const T*)fc->res : nullptr, fc ? (T*)fc->out : nullptr));
  }
  // The weight gradients are written for every expert, rows or not.
  DYNMO_TIMED_LAUNCH(K_FFN_DWD, st,
                     dw_generic_kernel<T><<<dim3(tf, th, d->E), dim3(256), 0, st>>>(seg, d->H, d->F, (const T*)dy_p,
                                                                                    (const T*)A, (T*)dWd));
  DYNMO_TIMED_LAUNCH(K_FFN_DWG, st,
                     dw_generic_kernel<T><<<dim3(th, tf, d->E), dim3(256), 0, st>>>(seg, d->F, d->H, (const T*)dG,
                                                                                    (const T*)x_p, (T*)dWg));
  DYNMO_TIMED_LAUNCH(K_FFN_DWU, st,
                     dw_generic_kernel<T><<<dim3(th, tf, d->E), dim3(256), 0, st>>>(seg, d->F, d->H, (const T*)dU,
                                                                                    (const T*)x_p, (T*)dWu));
  return DYNMO_OK;
}

int32_t ffn_fwd_generic(const dynmo_desc* d, const void* x_p, const int32_t* gather, const int32_t* seg, const void* Wg,
                        const void* Wu, const void* Wd, void* y_p, void* G, void* U, void* A, const FoldedCombine* fc,
                        hipStream_t st) {
  return d->dtype == DYNMO_BF16 ? fwd_generic_t<bf16_t>(d, x_p, gather, seg, Wg, Wu, Wd, y_p, G, U, A, fc, st)
                                : fwd_generic_t<float>(d, x_p, gather, seg, Wg, Wu, Wd, y_p, G, U, A, fc, st);
}

int32_t ffn_bwd_generic(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G, const void* U,
                        const int32_t* seg, const void* Wg, const void* Wu, const void* Wd, void* dx_p, void* dWg,
                        void* dWu, void* dWd, void* dG, void* dU, void* A, const FoldedCombine* fc, hipStream_t st) {
  return d->dtype == DYNMO_BF16
             ? bwd_generic_t<bf16_t>(d, dy_p, x_p, G, U, seg, Wg, Wu, Wd, dx_p, dWg, dWu, dWd, dG, dU, A, fc, st)
             : bwd_generic_t<float>(d, dy_p, x_p, G, U, seg, Wg, Wu, Wd, dx_p, dWg, dWu, dWd, dG, dU, A, fc, st);
}

}  // namespace dynmo
