// Routing kernels: token-choice top-k (MoE), per-sequence capacity top-k
// (Mixture-of-Depths), early-exit activity, and the gate backward passes.
#include "common.h"
#include "profile.h"

namespace dynmo {

// ---------------------------------------------------------------------------
// Top-k over E <= 64 logits.  A token owns LPT = pow2ceil(E) adjacent lanes of a
// wavefront, one logit per lane, so a 64-lane wavefront routes 64/LPT tokens and
// the logit loads are contiguous across the wavefront.  Each of the k rounds is
// a butterfly arg-max over the token's lanes with the order
// (value descending, expert index ascending); the winner is then retired.
// ---------------------------------------------------------------------------
struct Cand {
  float v;
  int idx;  // INT_MAX when the lane holds no live candidate
};

__device__ __forceinline__ bool better(const Cand& a, const Cand& b) {
  const bool av = a.idx != 0x7fffffff, bv = b.idx != 0x7fffffff;
  if (av != bv) return av;
  if (!av) return false;
  return a.v > b.v || (a.v == b.v && a.idx < b.idx);
}

template <int LPT>
__global__ __launch_bounds__(256) void route_topk_kernel(const float* __restrict__ logits, int32_t* __restrict__ expert_idx,
                                                         float* __restrict__ gate_w, int T, int E, int k) {
  constexpr int TOK_PER_WAVE = 64 / LPT;
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int j = lane % LPT;
  const long t = (long)wave * TOK_PER_WAVE + lane / LPT;
  const bool live = t < T && j < E;
  Cand mine;
  mine.v = live ? logits[t * E + j] : 0.f;
  mine.idx = live ? j : 0x7fffffff;
  float my_val = 0.f, top = 0.f, denom = 0.f;
  int my_idx = 0;
  for (int s = 0; s < k; ++s) {
    Cand best = mine;
#pragma unroll
    for (int m = 1; m < LPT; m <<= 1) {
      Cand o;
      o.v = __shfl_xor(best.v, m, 64);
      o.idx = __shfl_xor(best.idx, m, 64);
      if (better(o, best)) best = o;
    }
    if (s == 0) top = best.v;
    denom += __expf(best.v - top);
    if (j == s) {
      my_val = best.v;
      my_idx = best.idx;
    }
    if (mine.idx == best.idx) mine.idx = 0x7fffffff;  // retire the winner
  }
  if (t < T && j < k) {
    expert_idx[t * k + j] = my_idx;
    gate_w[t * k + j] = __expf(my_val - top) / denom;
  }
}

// The same selection with its two variants: the order is taken on logit + bias (one
// fp32 add; the bias steers the selection only), and the gate weights come from the raw
// logits as the softmax over the selected ones or over all E.  Same lane layout.
struct CandRaw {
  float v;    // logit + bias: what the order is taken on
  float raw;  // the logit itself
  int idx;
};

template <int LPT>
__global__ __launch_bounds__(256) void route_topk_ex_kernel(const float* __restrict__ logits, const float* __restrict__ bias,
                                                            int norm_all, int32_t* __restrict__ expert_idx,
                                                            float* __restrict__ gate_w, int T, int E, int k) {
  constexpr int TOK_PER_WAVE = 64 / LPT;
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int j = lane % LPT;
  const long t = (long)wave * TOK_PER_WAVE + lane / LPT;
  const bool live = t < T && j < E;
  const float raw = live ? logits[t * E + j] : 0.f;
  CandRaw mine;
  mine.raw = raw;
  mine.v = live ? (bias ? raw + bias[j] : raw) : 0.f;
  mine.idx = live ? j : 0x7fffffff;
  float my_raw = 0.f;
  int my_idx = 0;
  for (int s = 0; s < k; ++s) {
    CandRaw best = mine;
#pragma unroll
    for (int m = 1; m < LPT; m <<= 1) {
      CandRaw o;
      o.v = __shfl_xor(best.v, m, 64);
      o.raw = __shfl_xor(best.raw, m, 64);
      o.idx = __shfl_xor(best.idx, m, 64);
      const Cand a = {o.v, o.idx}, b = {best.v, best.idx};
      if (better(a, b)) best = o;
    }
    if (j == s) {
      my_raw = best.raw;
      my_idx = best.idx;
    }
    if (mine.idx == best.idx) mine.idx = 0x7fffffff;  // retire the winner
  }
  // softmax statistics over the token's lanes: lane j < k holds slot j's logit; for the
  // all-expert normalisation lane j < E contributes its own logit instead
  const bool in_sum = norm_all ? live : (t < T && j < k);
  const float z = norm_all ? raw : my_raw;
  float mx = in_sum ? z : -INFINITY;
#pragma unroll
  for (int m = 1; m < LPT; m <<= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
  float sum = in_sum ? __expf(z - mx) : 0.f;
#pragma unroll
  for (int m = 1; m < LPT; m <<= 1) sum += __shfl_xor(sum, m, 64);
  if (t < T && j < k) {
    expert_idx[t * k + j] = my_idx;
    gate_w[t * k + j] = __expf(my_raw - mx) / sum;
  }
}

// ---------------------------------------------------------------------------
// Capacity top-k: one workgroup per sequence.  This kernel takes sequences of any
// length (the launcher uses it beyond 4096 scores; shorter ones go to the register
// kernel below).  A 4-pass, 8-bit-per-pass radix select on order-preserving integer
// keys finds the cap-th largest score; ties at that value are resolved by ascending
// position with an ordered block scan.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0;  // -0.0 equals +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kCapThreads = 1024;

__global__ __launch_bounds__(kCapThreads) void route_capacity_kernel(const float* __restrict__ scores,
                                                                     int32_t* __restrict__ expert_idx,
                                                                     float* __restrict__ gate_w, int S, int cap) {
  __shared__ int hist[256];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_remaining;
  __shared__ int wave_cnt[kCapThreads / 64];
  __shared__ int sh_running;
  const float* sc = scores + (long)blockIdx.x * S;
  int32_t* ei = expert_idx + (long)blockIdx.x * S;
  float* gw = gate_w + (long)blockIdx.x * S;
  const int tid = threadIdx.x;

  if (cap <= 0 || cap >= S) {
    const bool all = cap >= S;
    for (int i = tid; i < S; i += kCapThreads) {
      ei[i] = all ? 0 : -1;
      gw[i] = all ? sigmoidf_(sc[i]) : 0.f;
    }
    return;
  }

  // radix select: after the passes, sh_prefix is the key of the cap-th largest
  // score and sh_remaining how many keys equal to it are still to be taken.
  if (tid == 0) {
    sh_prefix = 0;
    sh_remaining = cap;
  }
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const uint32_t himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int i = tid; i < S; i += kCapThreads) {
      const uint32_t key = score_key(sc[i]);
      if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 0xff], 1);
    }
    __syncthreads();
    if (tid == 0) {
      int remaining = sh_remaining;
      int b = 255;
      for (; b > 0; --b) {
        if (hist[b] >= remaining) break;
        remaining -= hist[b];
      }
      sh_prefix = prefix | ((uint32_t)b << shift);
      sh_remaining = remaining;
    }
    __syncthreads();
  }
  const uint32_t thr = sh_prefix;
  const int need_equal = sh_remaining;
  if (tid == 0) sh_running = 0;
  __syncthreads();

  const int lane = tid & 63, wv = tid >> 6;
  for (int base = 0; base < S; base += kCapThreads) {
    const int i = base + tid;
    float s = 0.f;
    uint32_t key = 0;
    if (i < S) {
      s = sc[i];
      key = score_key(s);
    }
    const bool eq = i < S && key == thr;
    const unsigned long long m = __ballot(eq);
    if (lane == 0) wave_cnt[wv] = __popcll(m);
    __syncthreads();
    int before = sh_running + __popcll(m & ((1ull << lane) - 1ull));
    int total = 0;
    for (int w = 0; w < kCapThreads / 64; ++w) {
      const int c = wave_cnt[w];
      if (w < wv) before += c;
      total += c;
    }
    if (i < S) {
      const bool sel = key > thr || (eq && before < need_equal);
      ei[i] = sel ? 0 : -1;
      gw[i] = sel ? sigmoidf_(s) : 0.f;
    }
    __syncthreads();
    if (tid == 0) sh_running += total;
    __syncthreads();
  }
}

// The same selection for sequences of at most kRegThreads * KPT scores, whose keys fit in
// registers (KPT per thread, score i of the sequence in thread i % kRegThreads): the cap-th
// largest key is found one bit at a time, most significant first -- bit b stays set if at
// least cap keys are >= the candidate -- with one workgroup-wide count per bit (ballots,
// four wavefront sums through LDS, one barrier).  No atomics and no serial histogram walk:
// a few microseconds instead of tens for the 2048-token sequences of the Mixture-of-Depths
// block.
constexpr int kRegThreads = 256;

template <int KPT>
__global__ __launch_bounds__(kRegThreads) void route_capacity_reg_kernel(const float* __restrict__ scores,
                                                                         int32_t* __restrict__ expert_idx,
                                                                         float* __restrict__ gate_w, int S, int cap) {
  constexpr int kWaves = kRegThreads / 64;
  static_assert(kWaves == 4, "the per-step counts are read back as one int4");
  static_assert(KPT * kWaves <= 64, "the tie scan below covers one wavefront's worth of partial counts");
  __shared__ int4 cnt[2];  // per-wavefront counts of one step, double-buffered by step parity
  __shared__ int eq_cnt[KPT * kWaves];
  const float* sc = scores + (long)blockIdx.x * S;
  int32_t* ei = expert_idx + (long)blockIdx.x * S;
  float* gw = gate_w + (long)blockIdx.x * S;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;

  float s[KPT];
  uint32_t key[KPT];
  bool valid[KPT];
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int i = j * kRegThreads + tid;
    valid[j] = i < S;
    s[j] = valid[j] ? sc[i] : 0.f;
    key[j] = valid[j] ? score_key(s[j]) : 0u;  // candidates below are never 0: padding is not counted
  }
  if (cap <= 0 || cap >= S) {
    const bool all = cap >= S;
#pragma unroll
    for (int j = 0; j < KPT; ++j)
      if (valid[j]) {
        ei[j * kRegThreads + tid] = all ? 0 : -1;
        gw[j * kRegThreads + tid] = all ? sigmoidf_(s[j]) : 0.f;
      }
    return;
  }

  // number of keys in the workgroup for which pred holds; `buf` alternates between calls so
  // that a wavefront one barrier ahead never overwrites counts still being read
  auto count = [&](auto pred, int buf) {
    int n = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) n += __popcll(__ballot(pred(j)));
    if (lane == 0) ((int*)&cnt[buf])[wv] = n;
    __syncthreads();
    const int4 c = cnt[buf];
    return __builtin_amdgcn_readfirstlane(c.x + c.y + c.z + c.w);
  };

  uint32_t thr = 0;  // becomes the cap-th largest key
  for (int b = 31; b >= 0; --b) {
    const uint32_t cand = thr | (1u << b);
    if (count([&](int j) { return key[j] >= cand; }, b & 1) >= cap) thr = cand;
  }
  const int greater = count([&](int j) { return valid[j] && key[j] > thr; }, 1);
  const int need_equal = cap - greater;  // ties at the threshold: the first need_equal by position

  unsigned long long eq[KPT];
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    eq[j] = __ballot(valid[j] && key[j] == thr);
    if (lane == 0) eq_cnt[j * kWaves + wv] = __popcll(eq[j]);
  }
  __syncthreads();
  // positions ascend with (j, wavefront, lane): exclusive scan of the partial counts in that order
  const int c = lane < KPT * kWaves ? eq_cnt[lane] : 0;
  int incl = c;
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const int up = __shfl_up(incl, m, 64);
    if (lane >= m) incl += up;
  }
  const int excl = incl - c;
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int before = __shfl(excl, j * kWaves + wv, 64) + __popcll(eq[j] & ((1ull << lane) - 1ull));
    if (valid[j]) {
      const bool sel = key[j] > thr || (key[j] == thr && before < need_equal);
      ei[j * kRegThreads + tid] = sel ? 0 : -1;
      gw[j * kRegThreads + tid] = sel ? sigmoidf_(s[j]) : 0.f;
    }
  }
}

__global__ void route_active_kernel(const int32_t* __restrict__ exit_layer, int layer, int32_t* __restrict__ expert_idx,
                                    float* __restrict__ gate_w, int T) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < T) {
    const bool act = exit_layer[t] >= layer;
    expert_idx[t] = act ? 0 : -1;
    gate_w[t] = act ? 1.f : 0.f;
  }
}

__global__ void route_topk_bwd_kernel(const float* __restrict__ dgate, const float* __restrict__ gate_w,
                                      const int32_t* __restrict__ expert_idx, float* __restrict__ dlogits, int T, int E,
                                      int k) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  float inner = 0.f;
  for (int s = 0; s < k; ++s) inner += gate_w[(long)t * k + s] * dgate[(long)t * k + s];
  for (int e = 0; e < E; ++e) dlogits[(long)t * E + e] = 0.f;
  for (int s = 0; s < k; ++s) {
    const int e = expert_idx[(long)t * k + s];
    if (e >= 0 && e < E) dlogits[(long)t * E + e] = gate_w[(long)t * k + s] * (dgate[(long)t * k + s] - inner);
  }
}

// Backward of the all-expert normalisation: with p = softmax(logits) over all E and
// w_s = p[e_s], dlogit[e] = sum_s dgate_s w_s ([e == e_s] - p[e]).  One thread per token.
__global__ void route_topk_all_bwd_kernel(const float* __restrict__ dgate, const float* __restrict__ logits,
                                          const int32_t* __restrict__ expert_idx, float* __restrict__ dlogits, int T,
                                          int E, int k) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float* lg = logits + (long)t * E;
  float mx = lg[0];
  for (int e = 1; e < E; ++e) mx = fmaxf(mx, lg[e]);
  float sum = 0.f;
  for (int e = 0; e < E; ++e) sum += __expf(lg[e] - mx);
  const float inv = 1.f / sum;
  float inner = 0.f;
  for (int s = 0; s < k; ++s) {
    const int e = expert_idx[(long)t * k + s];
    if (e >= 0 && e < E) inner += dgate[(long)t * k + s] * __expf(lg[e] - mx) * inv;
  }
  for (int e = 0; e < E; ++e) dlogits[(long)t * E + e] = -__expf(lg[e] - mx) * inv * inner;
  for (int s = 0; s < k; ++s) {
    const int e = expert_idx[(long)t * k + s];
    if (e >= 0 && e < E) dlogits[(long)t * E + e] += dgate[(long)t * k + s] * __expf(lg[e] - mx) * inv;
  }
}

__global__ void route_capacity_bwd_kernel(const float* __restrict__ dgate, const float* __restrict__ scores,
                                          const int32_t* __restrict__ expert_idx, float* __restrict__ dscores, int T) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  float r = 0.f;
  if (expert_idx[t] >= 0) {
    const float s = sigmoidf_(scores[t]);
    r = s * (1.f - s) * dgate[t];
  }
  dscores[t] = r;
}

template <int LPT>
static int32_t launch_topk(const dynmo_desc* d, const float* logits, int32_t* ei, float* gw, hipStream_t st) {
  const long tok_per_block = (256 / 64) * (64 / LPT);
  const long blocks = (d->T + tok_per_block - 1) / tok_per_block;
  if (blocks > 0) {
    DYNMO_TIMED_LAUNCH(K_ROUTE_TOPK, st,
                       route_topk_kernel<LPT><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(logits, ei, gw, d->T, d->E,
                                                                                            d->k));
  }
  return DYNMO_OK;
}

template <int LPT>
static int32_t launch_topk_ex(const dynmo_desc* d, const float* logits, const float* bias, int norm_all, int32_t* ei,
                              float* gw, hipStream_t st) {
  const long tok_per_block = (256 / 64) * (64 / LPT);
  const long blocks = (d->T + tok_per_block - 1) / tok_per_block;
  if (blocks > 0) {
    DYNMO_TIMED_LAUNCH(K_ROUTE_TOPK, st, route_topk_ex_kernel<LPT><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(
        logits, bias, norm_all, ei, gw, d->T, d->E, d->k));
  }
  return DYNMO_OK;
}

}  // namespace dynmo

using namespace dynmo;

extern "C" int32_t dynmo_route_topk_ex(const dynmo_desc* d, const float* logits, const float* bias, int32_t gate_norm,
                                       int32_t* expert_idx, float* gate_w, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!logits || !expert_idx || !gate_w || (gate_norm != DYNMO_NORM_SELECTED && gate_norm != DYNMO_NORM_ALL))
    return DYNMO_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const int E = d->E, all = gate_norm == DYNMO_NORM_ALL;
  if (E <= 1) return launch_topk_ex<1>(d, logits, bias, all, expert_idx, gate_w, st);
  if (E <= 2) return launch_topk_ex<2>(d, logits, bias, all, expert_idx, gate_w, st);
  if (E <= 4) return launch_topk_ex<4>(d, logits, bias, all, expert_idx, gate_w, st);
  if (E <= 8) return launch_topk_ex<8>(d, logits, bias, all, expert_idx, gate_w, st);
  if (E <= 16) return launch_topk_ex<16>(d, logits, bias, all, expert_idx, gate_w, st);
  if (E <= 32) return launch_topk_ex<32>(d, logits, bias, all, expert_idx, gate_w, st);
  return launch_topk_ex<64>(d, logits, bias, all, expert_idx, gate_w, st);
}

extern "C" int32_t dynmo_route_topk_all_bwd(const dynmo_desc* d, const float* dgate, const float* logits,
                                            const int32_t* expert_idx, float* dlogits, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!dgate || !logits || !expert_idx || !dlogits) return DYNMO_EINVAL;
  if (d->T > 0) {
    DYNMO_TIMED_LAUNCH(K_ROUTE_TOPK_BWD, (hipStream_t)stream,
                       route_topk_all_bwd_kernel<<<dim3((d->T + 255) / 256), dim3(256), 0, (hipStream_t)stream>>>(
                           dgate, logits, expert_idx, dlogits, d->T, d->E, d->k));
  }
  return DYNMO_OK;
}

extern "C" int32_t dynmo_route_topk(const dynmo_desc* d, const float* logits, int32_t* expert_idx, float* gate_w,
                                    void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!logits || !expert_idx || !gate_w) return DYNMO_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const int E = d->E;
  if (E <= 1) return launch_topk<1>(d, logits, expert_idx, gate_w, st);
  if (E <= 2) return launch_topk<2>(d, logits, expert_idx, gate_w, st);
  if (E <= 4) return launch_topk<4>(d, logits, expert_idx, gate_w, st);
  if (E <= 8) return launch_topk<8>(d, logits, expert_idx, gate_w, st);
  if (E <= 16) return launch_topk<16>(d, logits, expert_idx, gate_w, st);
  if (E <= 32) return launch_topk<32>(d, logits, expert_idx, gate_w, st);
  return launch_topk<64>(d, logits, expert_idx, gate_w, st);
}

extern "C" int32_t dynmo_route_capacity(const dynmo_desc* d, const float* scores, int32_t B, int32_t S, int32_t cap,
                                        int32_t* expert_idx, float* gate_w, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!scores || !expert_idx || !gate_w) return DYNMO_EINVAL;
  if (d->E != 1 || d->k != 1 || B < 0 || S <= 0 || (int64_t)B * S != d->T || cap < 0 || cap > S) return DYNMO_EINVAL;
  if (B > 0) {
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)B);
    if (S <= 4 * kRegThreads) {
      DYNMO_TIMED_LAUNCH(K_ROUTE_CAPACITY, st,
                         route_capacity_reg_kernel<4><<<grid, dim3(kRegThreads), 0, st>>>(scores, expert_idx, gate_w, S, cap));
    } else if (S <= 8 * kRegThreads) {
      DYNMO_TIMED_LAUNCH(K_ROUTE_CAPACITY, st,
                         route_capacity_reg_kernel<8><<<grid, dim3(kRegThreads), 0, st>>>(scores, expert_idx, gate_w, S, cap));
    } else if (S <= 16 * kRegThreads) {
      DYNMO_TIMED_LAUNCH(K_ROUTE_CAPACITY, st,
                         route_capacity_reg_kernel<16><<<grid, dim3(kRegThreads), 0, st>>>(scores, expert_idx, gate_w, S, cap));
    } else {
      DYNMO_TIMED_LAUNCH(K_ROUTE_CAPACITY, st,
                         route_capacity_kernel<<<grid, dim3(kCapThreads), 0, st>>>(scores, expert_idx, gate_w, S, cap));
    }
  }
  return DYNMO_OK;
}

extern "C" int32_t dynmo_route_active(const dynmo_desc* d, const int32_t* exit_layer, int32_t layer,
                                      int32_t* expert_idx, float* gate_w, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!exit_layer || !expert_idx || !gate_w) return DYNMO_EINVAL;
  if (d->E != 1 || d->k != 1) return DYNMO_EINVAL;
  if (d->T > 0) {
    hipStream_t st = (hipStream_t)stream;
    DYNMO_TIMED_LAUNCH(K_ROUTE_ACTIVE, st,
                       route_active_kernel<<<dim3((d->T + 255) / 256), dim3(256), 0, st>>>(exit_layer, layer, expert_idx,
                                                                                           gate_w, d->T));
  }
  return DYNMO_OK;
}

extern "C" int32_t dynmo_route_topk_bwd(const dynmo_desc* d, const float* dgate, const float* gate_w,
                                        const int32_t* expert_idx, float* dlogits, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!dgate || !gate_w || !expert_idx || !dlogits) return DYNMO_EINVAL;
  if (d->T > 0) {
    hipStream_t st = (hipStream_t)stream;
    DYNMO_TIMED_LAUNCH(K_ROUTE_TOPK_BWD, st,
                       route_topk_bwd_kernel<<<dim3((d->T + 255) / 256), dim3(256), 0, st>>>(dgate, gate_w, expert_idx,
                                                                                             dlogits, d->T, d->E, d->k));
  }
  return DYNMO_OK;
}

extern "C" int32_t dynmo_route_capacity_bwd(const dynmo_desc* d, const float* dgate, const float* scores,
                                            const int32_t* expert_idx, float* dscores, void* stream) {
  int32_t rc = check_desc(d);
  if (rc) return rc;
  if (!dgate || !scores || !expert_idx || !dscores) return DYNMO_EINVAL;
  if (d->E != 1 || d->k != 1) return DYNMO_EINVAL;
  if (d->T > 0) {
    hipStream_t st = (hipStream_t)stream;
    DYNMO_TIMED_LAUNCH(K_ROUTE_CAPACITY_BWD, st,
                       route_capacity_bwd_kernel<<<dim3((d->T + 255) / 256), dim3(256), 0, st>>>(dgate, scores, expert_idx,
                                                                                                 dscores, d->T));
  }
  return DYNMO_OK;
}
