/*
 * dynmo.h -- C ABI of the MI355X (gfx950) token-routed sparse FFN layer.
 *
 * The layer is the unit of work whose cost DynMo (arXiv 2505.14864) profiles and
 * rebalances: tokens are routed to experts (Sec. 2.1), or bypass the layer
 * (Mixture-of-Depths, Sec. 2.6), or have left the network early (Sec. 2.5), and
 * the work of the layer is the per-token FFN cost times the routed-token count.
 *
 * Conventions for every call
 *   - returns DYNMO_OK (0) or a negative DYNMO_E* code; never throws or aborts.
 *   - every tensor pointer is a DEVICE pointer owned by the caller unless the
 *     parameter name ends in _host.  The library keeps no device memory: scratch
 *     comes from the caller's workspace (size from dynmo_*_workspace_bytes).
 *   - outputs are overwritten, never accumulated into.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work
 *     and return; only dynmo_layer_load synchronises the stream (dynmo_layer_load_begin /
 *     _end are the same export without that).
 *   - activation, weight and gradient tensors must be 16-byte aligned (rows move in
 *     16-byte pieces); a misaligned one gives DYNMO_EINVAL.  Workspaces need no alignment
 *     (the *_workspace_bytes values include the slack the library needs to align them).
 *   - tensors are row-major and contiguous.  T tokens, H hidden size, F FFN size,
 *     E experts, k slots per token; flat slot i = t*k + s.  Index type int32,
 *     -1 = "slot not routed".  R = number of routed slots = seg_offsets[E].
 *     Buffers with a leading R dimension are sized for the worst case T*k; rows
 *     at or beyond R are left unspecified.
 *   - dtype DYNMO_F32: activations/weights float.  DYNMO_BF16: bfloat16 storage,
 *     fp32 accumulation, results rounded to nearest-even once.
 *     Logits, scores, gate weights and their gradients are always float.
 *   - weights: Wg, Wu are [E, F, H]; Wd is [E, H, F].
 *   - limits: 1 <= k <= E <= 64 (k <= 8 for the combine calls); for DYNMO_BF16
 *     H and F must be multiples of 8, for DYNMO_F32 H a multiple of 4.  Violations return DYNMO_EINVAL /
 *     DYNMO_EUNSUPPORTED before anything is launched.
 *     The fp32 path (and bf16 shapes the matrix-core kernels do not take) is limited to
 *     floor(T*k / 64) + min(E, T*k) <= 65535 (DYNMO_EUNSUPPORTED beyond).
 *   - NaN in logits or scores is undefined input, and so is a token whose logits are all
 *     -inf (its gate weights would be 0/0).
 */
#ifndef DYNMO_H
#define DYNMO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DYNMO_OK = 0,
  DYNMO_EINVAL = -1,       /* null pointer, bad shape, k > E, cap > S ... */
  DYNMO_EUNSUPPORTED = -2, /* shape or dtype outside the limits above */
  DYNMO_EWORKSPACE = -3,   /* workspace smaller than the *_workspace_bytes value */
  DYNMO_EHIP = -4          /* a HIP call failed; see dynmo_last_hip_error() */
};

enum { DYNMO_F32 = 0, DYNMO_BF16 = 1 };

typedef struct dynmo_desc {
  int32_t T;     /* tokens */
  int32_t H;     /* hidden size */
  int32_t F;     /* FFN intermediate size */
  int32_t E;     /* experts (1 for Mixture-of-Depths / early exit) */
  int32_t k;     /* slots per token (1 for Mixture-of-Depths / early exit) */
  int32_t dtype; /* DYNMO_F32 or DYNMO_BF16 */
} dynmo_desc;

int32_t dynmo_version(void);
/* The hipError_t of the last failed HIP call made by this library on the calling thread. */
int32_t dynmo_last_hip_error(void);

/* ---- route ------------------------------------------------------------- */

/* Token-choice top-k routing, the routing function R of Sec. 2.1.  Per token the
 * experts are ordered by (logit descending, expert index ascending); slot s gets
 * the s-th of them; gate_w is the softmax over the k selected logits.
 * logits [T,E] -> expert_idx [T,k], gate_w [T,k]. */
int32_t dynmo_route_topk(const dynmo_desc* d, const float* logits, int32_t* expert_idx, float* gate_w,
                         void* stream);

/* Mixture-of-Depths capacity routing (Sec. 2.6): per sequence of S scores the
 * `cap` largest (ties: lower position) are processed, the rest bypass the layer.
 * Needs T == B*S, E == 1, k == 1, 0 <= cap <= S.
 * scores [B,S] -> expert_idx [T,1] (0 selected / -1 not), gate_w [T,1]
 * (sigmoid(score) if selected, else 0). */
int32_t dynmo_route_capacity(const dynmo_desc* d, const float* scores, int32_t B, int32_t S, int32_t cap,
                             int32_t* expert_idx, float* gate_w, void* stream);

/* Early-exit activity (Sec. 2.5): a token is processed by stage-local layer
 * `layer` (1-based) iff exit_layer[t] >= layer.  Needs E == 1, k == 1.
 * exit_layer [T] -> expert_idx [T,1] (0 / -1), gate_w [T,1] (1 / 0). */
int32_t dynmo_route_active(const dynmo_desc* d, const int32_t* exit_layer, int32_t layer, int32_t* expert_idx,
                           float* gate_w, void* stream);

/* Backward of dynmo_route_topk through the gate softmax (the selection carries no
 * gradient): dlogits[t,e_s] = w_s (dgate_s - sum_j w_j dgate_j), zero elsewhere.
 * dgate [T,k], gate_w [T,k], expert_idx [T,k] -> dlogits [T,E]. */
int32_t dynmo_route_topk_bwd(const dynmo_desc* d, const float* dgate, const float* gate_w,
                             const int32_t* expert_idx, float* dlogits, void* stream);

/* Backward of dynmo_route_capacity: dscores[t] = sigmoid'(score) dgate[t] for
 * selected tokens, zero otherwise.  All arrays [T]. */
int32_t dynmo_route_capacity_bwd(const dynmo_desc* d, const float* dgate, const float* scores,
                                 const int32_t* expert_idx, float* dscores, void* stream);

/* Variants of the token-choice routing that the paper's discussion of MoE balancing
 * names (Sec. 2.1: bias terms added to the token-to-expert affinity scores; Sec. 6:
 * expert capacity in the GShard / Switch family).
 *
 * dynmo_route_topk_ex: like dynmo_route_topk, but the experts are ordered by
 * logits[t,e] + bias[e] (one fp32 add; bias [E] or NULL) and the gate weights are taken
 * from the raw logits: DYNMO_NORM_SELECTED = softmax over the k selected logits,
 * DYNMO_NORM_ALL = softmax over all E logits read at the selected experts.
 * Backward: dynmo_route_topk_bwd for DYNMO_NORM_SELECTED, dynmo_route_topk_all_bwd
 * (dlogit[e] = sum_s dgate_s w_s ([e == e_s] - p[e]), p the softmax over all E) for
 * DYNMO_NORM_ALL.  The selection and the bias carry no gradient. */
enum { DYNMO_NORM_SELECTED = 0, DYNMO_NORM_ALL = 1 };
int32_t dynmo_route_topk_ex(const dynmo_desc* d, const float* logits, const float* bias, int32_t gate_norm,
                            int32_t* expert_idx, float* gate_w, void* stream);
int32_t dynmo_route_topk_all_bwd(const dynmo_desc* d, const float* dgate, const float* logits,
                                 const int32_t* expert_idx, float* dlogits, void* stream);

/* Expert capacity with token dropping: slots are served in ascending flat order
 * t*k + s and a slot whose expert already holds `capacity` slots is dropped:
 * expert_idx_kept [T,k] = expert_idx, or -1 for a dropped (or already unrouted) slot.
 * Feed expert_idx_kept to dynmo_permute; keep expert_idx and gate_w for the routing
 * backward (a dropped slot gets dgate = 0 from dynmo_combine_bwd). */
size_t dynmo_route_drop_workspace_bytes(const dynmo_desc* d);
int32_t dynmo_route_drop(const dynmo_desc* d, const int32_t* expert_idx, int32_t capacity,
                         int32_t* expert_idx_kept, void* workspace, size_t workspace_bytes, void* stream);

/* ---- permute ----------------------------------------------------------- */

size_t dynmo_permute_workspace_bytes(const dynmo_desc* d);

/* Groups the routed slots into one contiguous row segment per expert -- the
 * token sets R^-1(e) of Sec. 2.1 -- by a stable counting sort of the flat slots
 * keyed by expert: row p = seg_offsets[e] + (number of earlier slots of expert e).
 * x [T,H], expert_idx [T,k] -> x_p [T*k,H] (x_p[p] = x[src_slot[p] / k]),
 * seg_offsets [E+1], src_slot [T*k], dst_pos [T,k] (-1 if unrouted).
 * With x_p = NULL only the indices are produced (x may then be NULL too).
 * The result is deterministic (no dependence on atomic ordering). */
int32_t dynmo_permute(const dynmo_desc* d, const void* x, const int32_t* expert_idx, void* x_p,
                      int32_t* seg_offsets, int32_t* src_slot, int32_t* dst_pos, void* workspace,
                      size_t workspace_bytes, void* stream);

/* dynmo_permute for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same arguments, results and kernels as dynmo_permute, but the scratch (the per-chunk
 * expert histograms) lives in a fixed 1 MiB device array inside the library, one copy per
 * GPU, held until the process ends.  The call allocates and frees nothing.  Limit:
 * ceil(T*k / 1024) * E <= 262144, i.e. T*k <= dynmo_permute_static_max_slots(E) slots
 * (4 194 304 slots at E = 64, 33 554 432 at E = 8); beyond it DYNMO_EWORKSPACE is returned
 * and nothing is launched.  Nothing in the array has to start at zero (every entry that
 * is read is rewritten first), but all calls on one GPU share it: two calls that overlap
 * in time on the same GPU (different streams or threads) race.  Calls on one stream, or
 * otherwise ordered, are fine. */
size_t dynmo_permute_static_max_slots(int32_t E);
int32_t dynmo_permute_static(const dynmo_desc* d, const void* x, const int32_t* expert_idx, void* x_p,
                             int32_t* seg_offsets, int32_t* src_slot, int32_t* dst_pos, void* stream);

/* Backward of permute (and of the pass-through residual when dbase != NULL):
 * dx[t] = dbase[t] + sum over routed slots s of dx_p[dst_pos[t,s]].
 * dx_p [T*k,H], dst_pos [T,k], dbase [T,H] or NULL -> dx [T,H]. */
int32_t dynmo_permute_bwd(const dynmo_desc* d, const void* dx_p, const int32_t* dst_pos, const void* dbase,
                          void* dx, void* stream);

/* ---- grouped FFN ------------------------------------------------------- */

size_t dynmo_grouped_ffn_fwd_workspace_bytes(const dynmo_desc* d);

/* The per-token workload c_e of Sec. 2.1 (c_i of Sec. 2.5 / 2.6): for the rows of
 * each expert segment, G = X Wg[e]^T, U = X Wu[e]^T, A = silu(G) * U, Y = A Wd[e]^T.
 * x_p [T*k,H], seg_offsets [E+1], weights -> y_p [T*k,H]; G_save, U_save [T*k,F]
 * are kept for the backward pass.  The workspace holds A and, for bf16, 64 MiB of
 * fp32 partial tiles (a last, sparsely filled round of output tiles is split along
 * the contraction and summed in a fixed order, so results are reproducible); its
 * contents are scratch: two calls that overlap in time need separate workspaces. */
int32_t dynmo_grouped_ffn_fwd(const dynmo_desc* d, const void* x_p, const int32_t* seg_offsets, const void* Wg,
                              const void* Wu, const void* Wd, void* y_p, void* G_save, void* U_save,
                              void* workspace, size_t workspace_bytes, void* stream);

/* The same layer with the row gather fused into the first product: the rows are read
 * straight from the token-ordered input, row p of the expert-sorted order being
 * x[src_slot[p] / k] (R^-1(e) of Sec. 2.1 applied inside the kernel's loads), so a
 * forward-only caller can skip the row copy of dynmo_permute (x_p = NULL there).
 * x [T,H], src_slot [T*k] as written by dynmo_permute; everything else, and the
 * workspace size, as for dynmo_grouped_ffn_fwd.  x must be smaller than 2 GiB
 * (DYNMO_EUNSUPPORTED otherwise). */
int32_t dynmo_grouped_ffn_fwd_gather(const dynmo_desc* d, const void* x, const int32_t* src_slot,
                                     const int32_t* seg_offsets, const void* Wg, const void* Wu, const void* Wd,
                                     void* y_p, void* G_save, void* U_save, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* The same layer for k = 1 (at most one routed row per token: the Mixture-of-Depths
 * block of Sec. 2.6, the shrinking layers of Sec. 2.5, top-1 MoE) with the weighted
 * combine folded into the stores of the last product: for every routed row p, with
 * t = src_slot[p],  out[t] = res[t] + gate_w[t] * Y[p]  (fp32 sum, rounded once).
 * Rows of out whose token has no routed row are NOT written: with res == out the
 * residual stream is updated in place and unrouted tokens pass through at no traffic;
 * with res == NULL (zero) or a separate res the caller owns those rows.
 * Exactly one of x_p [T,H] (expert-sorted rows) and x [T,H] (token order, rows fetched
 * through src_slot as in dynmo_grouped_ffn_fwd_gather, same 2 GiB limit) is non-NULL;
 * x may be out (the first product has finished reading before the last one stores).
 * gate_w [T] fp32; res, out [T,H]; y_p [T,H] or NULL (the unweighted rows, which
 * dynmo_combine_bwd needs for the gate gradient); G_save, U_save, workspace as for
 * dynmo_grouped_ffn_fwd.  d->k != 1 gives DYNMO_EINVAL. */
int32_t dynmo_grouped_ffn_fwd_combine(const dynmo_desc* d, const void* x_p, const void* x, const int32_t* src_slot,
                                      const int32_t* seg_offsets, const void* Wg, const void* Wu, const void* Wd,
                                      const float* gate_w, const void* res, void* out, void* y_p, void* G_save,
                                      void* U_save, void* workspace, size_t workspace_bytes, void* stream);

size_t dynmo_grouped_ffn_bwd_workspace_bytes(const dynmo_desc* d);

/* Backward of dynmo_grouped_ffn_fwd: dA = dY Wd; dG = dA U silu'(G); dU = dA silu(G);
 * dWd[e] = dY_e^T A_e; dX = dG Wg + dU Wu; dWg[e] = dG_e^T X_e; dWu[e] = dU_e^T X_e.
 * dWg, dWu [E,F,H] and dWd [E,H,F] are fully overwritten (zeros for an expert
 * with no rows); dx_p [T*k,H]. */
int32_t dynmo_grouped_ffn_bwd(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G_save,
                              const void* U_save, const int32_t* seg_offsets, const void* Wg, const void* Wu,
                              const void* Wd, void* dx_p, void* dWg, void* dWu, void* dWd, void* workspace,
                              size_t workspace_bytes, void* stream);

/* The backward pass for k = 1 (Mixture-of-Depths, Sec. 2.6; the shrinking layers of Sec. 2.5;
 * top-1 MoE) with the scatter back to token order (dynmo_permute_bwd) folded into the stores of
 * the dX product: for every routed row p, with t = src_slot[p],  dx[t] = dbase[t] + dX[p]
 * (fp32 sum, rounded once).  Rows of dx whose token has no routed row are NOT written: with
 * dbase == dx the upstream gradient of the residual stream is updated in place and unrouted
 * tokens pass through at no traffic; with dbase == NULL (zero) or a separate dbase the caller
 * owns those rows.  dx_p [T,H] or NULL (the rows in expert order, if the caller wants them);
 * everything else, and the workspace size, as for dynmo_grouped_ffn_bwd.  d->k != 1 gives
 * DYNMO_EINVAL. */
int32_t dynmo_grouped_ffn_bwd_scatter(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G_save,
                                      const void* U_save, const int32_t* seg_offsets, const int32_t* src_slot,
                                      const void* Wg, const void* Wu, const void* Wd, const void* dbase, void* dx,
                                      void* dx_p, void* dWg, void* dWu, void* dWd, void* workspace,
                                      size_t workspace_bytes, void* stream);

/* ---- combine ----------------------------------------------------------- */

/* out[t] = base[t] + sum over routed slots s (ascending) of gate_w[t,s] y_p[dst_pos[t,s]].
 * base is NULL (zero) for MoE and the layer input for Mixture-of-Depths / early
 * exit, whose unrouted tokens pass through unchanged (Sec. 2.5, 2.6).  out must
 * not alias base.  y_p [T*k,H], dst_pos [T,k], gate_w [T,k] -> out [T,H]. */
int32_t dynmo_combine(const dynmo_desc* d, const void* y_p, const int32_t* dst_pos, const float* gate_w,
                      const void* base, void* out, void* stream);

/* Backward of combine: dy_p[p] = gate_w[t,s] dout[t]; dgate[t,s] = <dout[t], y_p[p]>
 * with p = dst_pos[t,s] (dgate = 0 for unrouted slots). */
int32_t dynmo_combine_bwd(const dynmo_desc* d, const void* dout, const void* y_p, const int32_t* dst_pos,
                          const float* gate_w, void* dy_p, float* dgate, void* stream);

/* ---- load export and the host-side balancer ---------------------------- */

/* Exports the load the balancer consumes (Sec. 2.1: tokens per expert times the
 * per-token cost; Sec. 2.5 / 2.6 with one expert).  Copies seg_offsets to the
 * host, synchronises `stream`, and writes counts_host[e] = rows of expert e and
 * *load_host = sum_e counts[e] * cost_per_row.  counts_host [E] and load_host
 * are HOST pointers. */
int32_t dynmo_layer_load(const dynmo_desc* d, const int32_t* seg_offsets, double cost_per_row,
                         int32_t* counts_host, double* load_host, void* stream);

/* The same export in two halves, for a caller that must not stall the stream: the segment
 * offsets are final once dynmo_permute has run, long before the layer's backward pass ends.
 * dynmo_layer_load_begin enqueues the copy of seg_offsets [E+1] into seg_host and returns
 * without waiting; seg_host is a HOST pointer to E+1 ints of PINNED memory (hipHostMalloc, a
 * pinned tensor) that the caller owns and keeps alive and unread until it knows the copy has
 * completed (an event it recorded behind this call, or any later synchronisation of `stream`).
 * dynmo_layer_load_end then turns seg_host into counts_host [E] and *load_host exactly as
 * dynmo_layer_load does; it is host arithmetic only and makes no GPU call. */
int32_t dynmo_layer_load_begin(const dynmo_desc* d, const int32_t* seg_offsets, int32_t* seg_host, void* stream);
int32_t dynmo_layer_load_end(const dynmo_desc* d, const int32_t* seg_host, double cost_per_row,
                             int32_t* counts_host, double* load_host);

/* Partition balancer (Sec. 3.3, Sec. 5): the contiguous split of loads[L] into S
 * stages that minimises the largest stage load (the min-max objective of Sec. 2),
 * found by bisecting on the bottleneck value with a greedy left-to-right feasibility
 * scan.
 * Writes bounds_host[S+1] (stage i owns layers bounds[i] .. bounds[i+1]-1): the
 * split where each stage takes as many layers as fit under the optimal
 * bottleneck while leaving one layer for each later stage; *bottleneck_host gets
 * the optimum.  Host pointers only; loads must be finite and >= 0. */
int32_t dynmo_partition(const double* loads_host, int32_t L, int32_t S, int32_t* bounds_host,
                        double* bottleneck_host);

/* Partition with shadow layers (Sec. 4, Mixture of Depths: a block that is skipped is treated
 * as a shadow layer when the layers are redistributed).  shadow_host [L] (NULL = none): a
 * non-zero entry marks a layer that keeps its place in the order and its memory but adds no
 * load.  The split minimises first the largest stage load, with the shadow layers counted as
 * zero, and then, among the splits that reach that optimum, the largest number of layers on
 * one stage (free layers are spread instead of piling up on one worker).  bounds_host [S+1]:
 * from the left, each stage takes as many layers as both limits allow while leaving one layer
 * for every later stage; *bottleneck_host and *max_layers_host get the two optima.  Host
 * pointers only; loads must be finite and >= 0. */
int32_t dynmo_partition_shadow(const double* loads_host, const int32_t* shadow_host, int32_t L, int32_t S,
                               int32_t* bounds_host, double* bottleneck_host, int32_t* max_layers_host);

/* Equal layer counts per stage (the static split the paper compares against). */
int32_t dynmo_uniform_bounds(int32_t L, int32_t S, int32_t* bounds_host);

/* Stage loads L_i of Sec. 2 for a contiguous assignment. */
int32_t dynmo_stage_loads(const double* loads_host, int32_t L, const int32_t* bounds_host, int32_t S,
                          double* stage_loads_host);

/* Imbalance (L_max - L_min) / mean(L) of Sec. 2, Eq. 1-2. */
int32_t dynmo_imbalance(const double* stage_loads_host, int32_t S, double* imbalance_host);

/* Potential of Sec. 3.3 (proof of Lemma 2): phi = sum over unordered pairs of stages of |x_u - x_v|. */
int32_t dynmo_potential(const double* stage_loads_host, int32_t S, double* phi_host);

/* Diffusion balancer (Sec. 3.3: iterative, layers move from overloaded workers to
 * underloaded neighbours; phi never increases; stop once phi <= gamma).  The stages are
 * the workers, in pipeline order, and stay contiguous: a round moves one layer across
 * one stage boundary -- of all such transfers that keep the giving stage non-empty, fit
 * the receiving stage's memory (sum of layer_mem_host over its layers plus the layer
 * <= max_mem; no limit when layer_mem_host is NULL) and strictly lower phi, the one that
 * lowers it most (ties: lower boundary, then the transfer towards the later stage).  Ends
 * when phi <= gamma, when no transfer lowers phi, or after max_rounds rounds.
 * bounds_host [S+1]: the starting split on entry, the result on exit.  *rounds_host gets
 * the number of transfers made, phi_host[0] / phi_host[1] the potential before / after.
 * Host pointers only; loads must be finite and >= 0. */
int32_t dynmo_diffusion(const double* loads_host, int32_t L, int32_t S, int32_t* bounds_host,
                        const double* layer_mem_host, double max_mem, double gamma, int32_t max_rounds,
                        int32_t* rounds_host, double* phi_host);

/* Re-pack (Sec. 3.4, Algorithm 2): first-fit consolidation onto fewer workers.  Workers
 * are visited in order; while more than target_num_workers are active, an active worker
 * whose memory fits, together with that of a later active worker, strictly under max_mem
 * is freed (active = 0) into the first such worker, which takes over its memory and its
 * layers; every moved layer is listed as a transfer (freed worker, receiving worker, layer
 * index on the freed worker).  A freed worker neither gives nor takes again.
 * active_host, mem_usage_host, num_layers_host [n_workers]: in and out (a freed worker's
 * memory and layer count are left as they were).  transfers_host: 3 * capacity ints;
 * *n_transfers_host gets the number of transfers.  If they do not fit, returns
 * DYNMO_EWORKSPACE with the needed count in *n_transfers_host and every array unchanged.
 * Host pointers only. */
int32_t dynmo_repack(int32_t n_workers, int32_t* active_host, double* mem_usage_host, int32_t* num_layers_host,
                     int32_t target_num_workers, double max_mem, int32_t* transfers_host, int32_t capacity,
                     int32_t* n_transfers_host);

/* ---- profiling step ------------------------------------------------------ */

/* The paper's profiling step (Sec. 3.1, Sec. 4: the iteration after a change is
 * timed per layer and the times feed the "by Time" balancers).  While enabled,
 * every kernel the library launches is bracketed by a hipEvent pair on its
 * stream; totals are kept per kernel role (dynmo_profile_kernel_name) and are
 * process-wide.  dynmo_profile_read waits for the recorded launches of that role
 * to finish, then returns their summed duration in milliseconds and their count
 * (HOST pointers).  dynmo_profile_reset waits likewise and zeroes all totals. */
int32_t dynmo_profile_enable(int32_t on);
int32_t dynmo_profile_reset(void);
int32_t dynmo_profile_kernel_count(void);
const char* dynmo_profile_kernel_name(int32_t id);
int32_t dynmo_profile_read(int32_t id, double* total_ms_host, int64_t* launches_host);

/* ---- what the device can reach ---------------------------------------------- */

/* Measurement aids, not part of the method: reference kernels whose duration the
 * caller times on `stream` to get the box's own ceilings next to the data-sheet ones.
 *
 * dynmo_peak_mfma_bf16: 256 workgroups of eight wavefronts issue `iters` x 16
 * v_mfma_f32_16x16x32_bf16 each on register operands; *flops_host (HOST) gets the
 * flop count of the launch.  operands: DEVICE, 8 KiB of bf16 data the operand
 * registers are filled from (random data draws the power of a real product), or
 * NULL for fixed small numbers.  sink: DEVICE, 256 * 512 floats, overwritten.
 *
 * dynmo_peak_copy: plain streaming copy of `bytes` (a multiple of 16; DEVICE
 * pointers, 16-byte aligned, not overlapping): reads `bytes`, writes `bytes`. */
int32_t dynmo_peak_mfma_bf16(int32_t iters, const void* operands, float* sink, double* flops_host, void* stream);
int32_t dynmo_peak_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DYNMO_H */
