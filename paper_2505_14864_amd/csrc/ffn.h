// Pieces shared by the grouped-FFN kernels: the ragged row-tile lookup, the
// SwiGLU backward formula, and the entry points of the two kernel families.
#pragma once

#include "common.h"

namespace dynmo {

// Upper bound on the number of BM-row tiles over all expert segments: every
// segment can add one partial tile.  The true count is only known on the device.
inline int max_m_tiles(const dynmo_desc* d, int BM) {
  const int64_t rows = (int64_t)d->T * d->k;
  if (rows == 0) return 0;
  const int64_t full = rows / BM;
  const int64_t partial = d->E < rows ? d->E : rows;
  return (int)(full + partial);
}

// Maps a flat row-tile index to (expert, first row, end row) by walking the
// segment offsets.  Returns false for an index past the last tile.
__device__ __forceinline__ bool find_m_tile(const int32_t* __restrict__ seg, int E, int tile, int BM, int* e_out,
                                            int* m0, int* m_end) {
  int first = 0;
  int begin = seg[0];
  for (int e = 0; e < E; ++e) {
    const int end = seg[e + 1];
    const int nt = (end - begin + BM - 1) / BM;
    if (tile < first + nt) {
      *e_out = e;
      *m0 = begin + (tile - first) * BM;
      *m_end = end;
      return true;
    }
    first += nt;
    begin = end;
  }
  return false;
}

// Given dA and the saved pre-activations: A = silu(g) u, dG = dA u silu'(g), dU = dA silu(g).
__device__ __forceinline__ void swiglu_bwd(float dA, float g, float u, float* a, float* dg, float* du) {
  const float s = sigmoidf_(g);
  const float gs = g * s;
  *a = gs * u;
  *dg = dA * u * (s * (1.f + g * (1.f - s)));
  *du = dA * gs;
}

// The combine of a one-slot layer (k = 1) folded into the stores of Y = A Wd^T: row p also
// goes to out[t] = res[t] + scale[t] * Y[p], t = scatter[p].  res may be nullptr (zero) or out.
// The same record folds the scatter back to token order into the stores of dX (backward):
// scale is then nullptr (weight 1), res the upstream gradient of the residual, out = dx.
struct FoldedCombine {
  const int32_t* scatter;
  const float* scale;
  const void* res;
  void* out;
};

// In both forward families `gather` is NULL (x_p holds the expert-sorted rows) or the
// slot index: row p is then x_p[gather[p] / k], x_p being the token-ordered input.
// `fc` is NULL or the folded combine; y_p (forward) / dx_p (backward) may be NULL only with it.
int32_t ffn_fwd_generic(const dynmo_desc* d, const void* x_p, const int32_t* gather, const int32_t* seg, const void* Wg,
                        const void* Wu, const void* Wd, void* y_p, void* G, void* U, void* A, const FoldedCombine* fc,
                        hipStream_t st);
int32_t ffn_bwd_generic(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G, const void* U,
                        const int32_t* seg, const void* Wg, const void* Wu, const void* Wd, void* dx_p, void* dWg,
                        void* dWu, void* dWd, void* dG, void* dU, void* A, const FoldedCombine* fc, hipStream_t st);


// bf16 matrix-core kernels
bool ffn_mfma_supported(const dynmo_desc* d);
size_t ffn_mfma_scratch_bytes();  // 256-byte aligned device scratch both calls below need
int32_t ffn_fwd_mfma(const dynmo_desc* d, const void* x_p, const int32_t* gather, const int32_t* seg, const void* Wg,
                     const void* Wu, const void* Wd, void* y_p, void* G, void* U, void* A, void* scratch,
                     const FoldedCombine* fc, hipStream_t st);
int32_t ffn_bwd_mfma(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G, const void* U,
                     const int32_t* seg, const void* Wg, const void* Wu, const void* Wd, void* dx_p, void* dWg,
                     void* dWu, void* dWd, void* dG, void* dU, void* A, void* scratch, const FoldedCombine* fc,
                     hipStream_t st);

}  // namespace dynmo
