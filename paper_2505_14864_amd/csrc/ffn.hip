// C-ABI entry points of the grouped SwiGLU FFN: argument checks, workspace
// carving and the choice of kernel family.
#include "ffn.h"

using namespace dynmo;

namespace dynmo {
thread_local int32_t g_last_hip_error = 0;

static size_t act_bytes(const dynmo_desc* d) {  // one [T*k, F] activation buffer
  return align_up((size_t)d->T * d->k * d->F * elem_bytes(d->dtype), 256);
}
static size_t mfma_scratch(const dynmo_desc* d) { return ffn_mfma_supported(d) ? ffn_mfma_scratch_bytes() : 0; }
}  // namespace dynmo

extern "C" int32_t dynmo_version(void) { return 1; }
extern "C" int32_t dynmo_last_hip_error(void) { return g_last_hip_error; }

extern "C" size_t dynmo_grouped_ffn_fwd_workspace_bytes(const dynmo_desc* d) {
  if (check_desc(d)) return 0;
  return act_bytes(d) + mfma_scratch(d) + 256;  // A = silu(G) U
}

extern "C" size_t dynmo_grouped_ffn_bwd_workspace_bytes(const dynmo_desc* d) {
  if (check_desc(d)) return 0;
  return 3 * act_bytes(d) + mfma_scratch(d) + 256;  // dG, dU, A
}

namespace dynmo {
static int32_t ffn_fwd_entry(const dynmo_desc* d, const void* rows, const int32_t* gather, const int32_t* seg_offsets,
                             const void* Wg, const void* Wu, const void* Wd, void* y_p, void* G_save, void* U_save,
                             void* workspace, size_t workspace_bytes, const FoldedCombine* fc, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!rows || !seg_offsets || !Wg || !Wu || !Wd || !G_save || !U_save || !workspace) return DYNMO_EINVAL;
  if (!y_p && !fc) return DYNMO_EINVAL;
  if (misaligned16(rows, Wg, Wu, Wd, y_p, G_save, U_save) || (fc && misaligned16(fc->res, fc->out)))
    return DYNMO_EINVAL;
  if (workspace_bytes < dynmo_grouped_ffn_fwd_workspace_bytes(d)) return DYNMO_EWORKSPACE;
  void* A = (void*)align_up((size_t)workspace, 256);
  if (ffn_mfma_supported(d))
    return ffn_fwd_mfma(d, rows, gather, seg_offsets, Wg, Wu, Wd, y_p, G_save, U_save, A, (char*)A + act_bytes(d),
                        fc, (hipStream_t)stream);
  if (max_m_tiles(d, 64) > 65535) return DYNMO_EUNSUPPORTED;  // the generic kernels put row tiles on grid y
  return ffn_fwd_generic(d, rows, gather, seg_offsets, Wg, Wu, Wd, y_p, G_save, U_save, A, fc, (hipStream_t)stream);
}
}  // namespace dynmo

extern "C" int32_t dynmo_grouped_ffn_fwd(const dynmo_desc* d, const void* x_p, const int32_t* seg_offsets,
                                         const void* Wg, const void* Wu, const void* Wd, void* y_p, void* G_save,
                                         void* U_save, void* workspace, size_t workspace_bytes, void* stream) {
  return ffn_fwd_entry(d, x_p, nullptr, seg_offsets, Wg, Wu, Wd, y_p, G_save, U_save, workspace, workspace_bytes,
                       nullptr, stream);
}

extern "C" int32_t dynmo_grouped_ffn_fwd_gather(const dynmo_desc* d, const void* x, const int32_t* src_slot,
                                                const int32_t* seg_offsets, const void* Wg, const void* Wu,
                                                const void* Wd, void* y_p, void* G_save, void* U_save,
                                                void* workspace, size_t workspace_bytes, void* stream) {
  if (!src_slot) return DYNMO_EINVAL;
  // gathered rows are addressed with 32-bit byte offsets from the first row of x, whose top
  // bit marks "outside": the whole input must stay below 2 GiB
  if (d && (int64_t)d->T * d->H * (int64_t)elem_bytes(d->dtype) >= ((int64_t)1 << 31)) return DYNMO_EUNSUPPORTED;
  return ffn_fwd_entry(d, x, src_slot, seg_offsets, Wg, Wu, Wd, y_p, G_save, U_save, workspace, workspace_bytes,
                       nullptr, stream);
}

extern "C" int32_t dynmo_grouped_ffn_fwd_combine(const dynmo_desc* d, const void* x_p, const void* x,
                                                 const int32_t* src_slot, const int32_t* seg_offsets, const void* Wg,
                                                 const void* Wu, const void* Wd, const float* gate_w, const void* res,
                                                 void* out, void* y_p, void* G_save, void* U_save, void* workspace,
                                                 size_t workspace_bytes, void* stream) {
  if (!d || !src_slot || !gate_w || !out || (x_p == nullptr) == (x == nullptr)) return DYNMO_EINVAL;
  if (d->k != 1) return DYNMO_EINVAL;  // with two slots per token two rows would meet in one output row
  if (x && (int64_t)d->T * d->H * (int64_t)elem_bytes(d->dtype) >= ((int64_t)1 << 31)) return DYNMO_EUNSUPPORTED;
  const FoldedCombine fc = {src_slot, gate_w, res, out};
  return ffn_fwd_entry(d, x_p ? x_p : x, x_p ? nullptr : src_slot, seg_offsets, Wg, Wu, Wd, y_p, G_save, U_save,
                       workspace, workspace_bytes, &fc, stream);
}

namespace dynmo {
static int32_t ffn_bwd_entry(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G_save,
                             const void* U_save, const int32_t* seg_offsets, const void* Wg, const void* Wu,
                             const void* Wd, void* dx_p, void* dWg, void* dWu, void* dWd, void* workspace,
                             size_t workspace_bytes, const FoldedCombine* fc, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!dy_p || !x_p || !G_save || !U_save || !seg_offsets || !Wg || !Wu || !Wd || !dWg || !dWu || !dWd || !workspace)
    return DYNMO_EINVAL;
  if (!dx_p && !fc) return DYNMO_EINVAL;
  if (misaligned16(dy_p, x_p, G_save, U_save, Wg, Wu, Wd, dx_p, dWg, dWu, dWd) || (fc && misaligned16(fc->res, fc->out)))
    return DYNMO_EINVAL;
  if (workspace_bytes < dynmo_grouped_ffn_bwd_workspace_bytes(d)) return DYNMO_EWORKSPACE;
  char* base = (char*)align_up((size_t)workspace, 256);
  void* dG = base;
  void* dU = base + act_bytes(d);
  void* A = base + 2 * act_bytes(d);
  if (ffn_mfma_supported(d))
    return ffn_bwd_mfma(d, dy_p, x_p, G_save, U_save, seg_offsets, Wg, Wu, Wd, dx_p, dWg, dWu, dWd, dG, dU, A,
                        base + 3 * act_bytes(d), fc, (hipStream_t)stream);
  if (max_m_tiles(d, 64) > 65535) return DYNMO_EUNSUPPORTED;  // the generic kernels put row tiles on grid y
  return ffn_bwd_generic(d, dy_p, x_p, G_save, U_save, seg_offsets, Wg, Wu, Wd, dx_p, dWg, dWu, dWd, dG, dU, A, fc,
                         (hipStream_t)stream);
}
}  // namespace dynmo

extern "C" int32_t dynmo_grouped_ffn_bwd(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G_save,
                                         const void* U_save, const int32_t* seg_offsets, const void* Wg,
                                         const void* Wu, const void* Wd, void* dx_p, void* dWg, void* dWu, void* dWd,
                                         void* workspace, size_t workspace_bytes, void* stream) {
  return ffn_bwd_entry(d, dy_p, x_p, G_save, U_save, seg_offsets, Wg, Wu, Wd, dx_p, dWg, dWu, dWd, workspace,
                       workspace_bytes, nullptr, stream);
}

extern "C" int32_t dynmo_grouped_ffn_bwd_scatter(const dynmo_desc* d, const void* dy_p, const void* x_p,
                                                 const void* G_save, const void* U_save, const int32_t* seg_offsets,
                                                 const int32_t* src_slot, const void* Wg, const void* Wu,
                                                 const void* Wd, const void* dbase, void* dx, void* dx_p, void* dWg,
                                                 void* dWu, void* dWd, void* workspace, size_t workspace_bytes,
                                                 void* stream) {
  if (!d || !src_slot || !dx) return DYNMO_EINVAL;
  if (d->k != 1) return DYNMO_EINVAL;  // with two slots per token two rows would meet in one row of dx
  const FoldedCombine fc = {src_slot, nullptr, dbase, dx};
  return ffn_bwd_entry(d, dy_p, x_p, G_save, U_save, seg_offsets, Wg, Wu, Wd, dx_p, dWg, dWu, dWd, workspace,
                       workspace_bytes, &fc, stream);
}
