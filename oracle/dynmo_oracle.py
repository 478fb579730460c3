"""Plain CPU oracle of the token-routed sparse FFN layer, forward and backward.

THIS IS TEST INFRASTRUCTURE. It defines what the GPU library must compute and
is deliberately slow and literal. It shares no code with the HIP path, and the
product package never imports it.

Arithmetic: every floating-point input (fp32, or bf16 widened exactly to fp32)
is converted to float64 and all intermediate and output values stay float64.
Integer outputs are int32. Top-k decisions compare the input values exactly
(widening fp32 to fp64 preserves order), so they are the fp32 decisions.

What follows the paper and what is a reading of it:
  * The paper (DynMo, arXiv 2505.14864) treats the routed layers as black
    boxes.  It fixes the *problem statement*: workers, tasks, loads and the
    min-max objective (Sec. 2), the imbalance metric (Sec. 2, Eq. 1-2), the
    MoE load (Sec. 2.1), early-exit load (Sec. 2.5), MoD load (Sec. 2.6), the
    Partition balancer (Sec. 3.3 and Sec. 5) and the re-pack pseudo-code
    (Sec. 3.4, Algorithm 2).
  * Routing, permutation, SwiGLU FFN and combine are the textbook definitions
    of those layers (token-choice top-k with softmax over the selected logits,
    stable counting sort by expert, down(silu(gate(x)) * up(x)), weighted
    scatter-add).  Each function's docstring states the reading it takes.

Pins (tests/test_oracle_*.py): brute-force top-k by full sort in pure Python,
closed forms for the gates, an independent permutation checker, the dense
masked FFN equivalent evaluated and differentiated by torch (fp64 autograd),
central finite differences, special cases (E=1,k=1 dense MLP; Wd=0; nobody
exits / everybody exits), brute-force enumeration of contiguous splits for the
partitioner, hand-worked imbalance vectors, partitions, diffusion runs and a
re-pack trace under tests/golden/ and in the tests, the closed form of the
diffusion potential over order statistics, scipy's softmax and torch autograd
for the routing variants, and a planted-mistake test that the pins catch.

Every function here has at least one such pin; none is unpinned.  The layer's
component functions (permute, grouped FFN, combine and their backward passes)
are pinned through the whole-layer chains, and the planted-mistake test shows
that a mistake in any single one of them fails those pins.  The paper
prints no tensor values for this path, so no pin is a number taken from the
paper: they are all mathematical checks of the kinds listed above.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64
I32 = np.int32


def _f64(a):
    return np.asarray(a).astype(F64)


# --------------------------------------------------------------------------
# Routing
# --------------------------------------------------------------------------

def route_topk(logits, k):
    """Token-choice top-k routing (Sec. 2.1: routing function R maps tokens to
    experts; Sec. 4 names Mixtral-style routing).

    Per token the experts are ordered by (logit descending, index ascending);
    slot s takes the s-th expert of that order.  Gate weights are the softmax
    over the k selected logits.  +0.0 and -0.0 are equal.  NaN is undefined.

    logits: [T, E] float.  Returns expert_idx int32 [T, k], gate_w f64 [T, k].
    """
    lg = _f64(logits)
    T, E = lg.shape
    if not (1 <= k <= E):
        raise ValueError("k must be in [1, E]")
    # stable sort of the negated values: equal values keep ascending index
    order = np.argsort(-lg, axis=1, kind="stable")
    idx = order[:, :k]
    sel = np.take_along_axis(lg, idx, axis=1)
    ex = np.exp(sel - sel[:, :1])
    gate = ex / ex.sum(axis=1, keepdims=True)
    return idx.astype(I32), gate


def route_topk_biased(logits, k, bias=None, norm="selected"):
    """Token-choice top-k with the two variants the paper's survey of MoE routing
    names (Sec. 2.1: bias terms added to the token-to-expert affinity scores, as
    in auxiliary-loss-free balancing; Sec. 6: the GShard / Switch family).

    Selection orders the experts by (logit + bias) -- that sum is taken in
    float32, the precision the scores arrive in, because it decides an integer
    -- descending, index ascending on ties.  The bias steers the selection only:
    gate weights come from the raw logits, either as the softmax over the k
    selected ones (norm="selected", the same as route_topk) or as the softmax
    over all E experts read at the selected ones (norm="all").

    Returns expert_idx int32 [T, k], gate_w f64 [T, k].
    """
    lg32 = np.asarray(logits, dtype=np.float32)
    T, E = lg32.shape
    if not (1 <= k <= E):
        raise ValueError("k must be in [1, E]")
    score = lg32 if bias is None else (lg32 + np.asarray(bias, dtype=np.float32)[None, :]).astype(np.float32)
    order = np.argsort(-score.astype(F64), axis=1, kind="stable")
    idx = order[:, :k]
    lg = lg32.astype(F64)
    sel = np.take_along_axis(lg, idx, axis=1)
    if norm == "selected":
        ex = np.exp(sel - sel.max(axis=1, keepdims=True))
        gate = ex / ex.sum(axis=1, keepdims=True)
    elif norm == "all":
        m = lg.max(axis=1, keepdims=True)
        gate = np.exp(sel - m) / np.exp(lg - m).sum(axis=1, keepdims=True)
    else:
        raise ValueError(norm)
    return idx.astype(I32), gate


def route_topk_biased_bwd(dgate, logits, expert_idx, norm="selected"):
    """Gradient of the gate weights of route_topk_biased with respect to the raw
    logits (selection and bias carry none).  With p the softmax the weights are
    read from (over the selected logits, or over all E):
    dlogit[e] = sum_s dgate_s * w_s * ([e == e_s] - p[e])."""
    dg = _f64(dgate)
    lg = _f64(logits)
    ei = np.asarray(expert_idx).astype(np.int64)
    T, E = lg.shape
    out = np.zeros((T, E), F64)
    for t in range(T):
        if norm == "selected":
            z = lg[t, ei[t]]
            p_sel = np.exp(z - z.max())
            p_sel /= p_sel.sum()
            p = np.zeros(E, F64)
            p[ei[t]] = p_sel
        else:
            p = np.exp(lg[t] - lg[t].max())
            p /= p.sum()
        w = p[ei[t]]
        inner = float((dg[t] * w).sum())
        out[t] = -p * inner
        for s in range(ei.shape[1]):
            out[t, ei[t, s]] += dg[t, s] * w[s]
    return out


def capacity_drop(expert_idx, E, capacity):
    """Expert capacity with token dropping (Sec. 6: an expert processes at most
    `capacity` tokens).  Slots are served in ascending flat order i = t*k + s:
    a slot whose expert already holds `capacity` slots is dropped (-1), it is
    not re-routed.  Returns the kept assignment, same shape."""
    ei = np.asarray(expert_idx)
    flat = ei.reshape(-1).astype(np.int64)
    kept = flat.copy()
    held = [0] * E
    for i, e in enumerate(flat):
        if e < 0:
            continue
        if held[e] >= capacity:
            kept[i] = -1
        else:
            held[e] += 1
    return kept.reshape(ei.shape).astype(I32)


def route_capacity(scores, cap):
    """Mixture-of-Depths capacity routing (Sec. 2.6: tokens bypass a layer
    unless they are among the top-k of their sequence).

    Per sequence the tokens are ordered by (score descending, position
    ascending) and the first `cap` are selected.  Selected tokens go to the
    single expert 0 with gate sigmoid(score); the others get -1 and gate 0.

    scores: [B, S] float.  Returns expert_idx int32 [B*S, 1], gate f64 [B*S, 1].
    """
    sc = _f64(scores)
    B, S = sc.shape
    if not (0 <= cap <= S):
        raise ValueError("cap must be in [0, S]")
    order = np.argsort(-sc, axis=1, kind="stable")
    sel = np.zeros((B, S), dtype=bool)
    np.put_along_axis(sel, order[:, :cap], True, axis=1)
    idx = np.where(sel, 0, -1).astype(I32)
    gate = np.where(sel, 1.0 / (1.0 + np.exp(-sc)), 0.0)
    return idx.reshape(B * S, 1), gate.reshape(B * S, 1)


def route_active(exit_layer, layer):
    """Early-exit activity (Sec. 2.5: t_i tokens are processed by layer i and
    t_i decreases with depth).  A token is processed by stage-local layer
    `layer` (1-based) iff exit_layer[t] >= layer.  Gate is 1 for active tokens.
    """
    ex = np.asarray(exit_layer)
    act = ex >= layer
    idx = np.where(act, 0, -1).astype(I32).reshape(-1, 1)
    gate = np.where(act, 1.0, 0.0).astype(F64).reshape(-1, 1)
    return idx, gate


# --------------------------------------------------------------------------
# Permutation into contiguous expert segments
# --------------------------------------------------------------------------

def permute(x, expert_idx, E):
    """Group routed slots by expert (Sec. 2.1: R^{-1}(e) is the token set of
    expert e).  A stable counting sort of the flat slots i = t*k + s keyed by
    expert: row p = seg_offsets[e] + (number of earlier slots with expert e).

    x: [T, H]; expert_idx: [T, k] with -1 for an unrouted slot.
    Returns x_p [R, H] (same dtype as x, rows are copies), seg_offsets int32
    [E+1], src_slot int32 [R], dst_pos int32 [T, k] (-1 if unrouted).
    """
    x = np.asarray(x)
    ei = np.asarray(expert_idx)
    T, k = ei.shape
    flat = ei.reshape(-1)
    counts = [0] * E
    for e in flat:
        if e >= 0:
            counts[int(e)] += 1
    seg = [0] * (E + 1)
    for e in range(E):
        seg[e + 1] = seg[e] + counts[e]
    R = seg[E]
    running = [0] * E
    src_slot = np.full(R, -1, dtype=I32)
    dst_pos = np.full(T * k, -1, dtype=I32)
    for i in range(T * k):
        e = int(flat[i])
        if e < 0:
            continue
        p = seg[e] + running[e]
        running[e] += 1
        src_slot[p] = i
        dst_pos[i] = p
    x_p = x[src_slot // k] if R > 0 else x[:0]
    return x_p.copy(), np.asarray(seg, dtype=I32), src_slot, dst_pos.reshape(T, k)


# --------------------------------------------------------------------------
# Grouped SwiGLU FFN
# --------------------------------------------------------------------------

def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def grouped_ffn_fwd(x_p, seg_offsets, Wg, Wu, Wd):
    """Per-expert SwiGLU FFN on contiguous row segments.  This is the per-token
    workload c_e of Sec. 2.1 (and c_i of Sec. 2.5 / 2.6 with one expert).

    For rows p of expert e:  G = X Wg[e]^T,  U = X Wu[e]^T,
    A = G * sigmoid(G) * U,  Y = A Wd[e]^T.  No biases.

    x_p [R, H]; Wg, Wu [E, F, H]; Wd [E, H, F].  Returns y_p, G, U (f64).
    """
    seg = np.asarray(seg_offsets)
    E, F, H = Wg.shape
    R = x_p.shape[0]
    y = np.zeros((R, H), F64)
    G = np.zeros((R, F), F64)
    U = np.zeros((R, F), F64)
    for e in range(E):
        a, b = int(seg[e]), int(seg[e + 1])
        if b <= a:
            continue
        X = _f64(x_p[a:b])
        G[a:b] = X @ _f64(Wg[e]).T
        U[a:b] = X @ _f64(Wu[e]).T
        A = G[a:b] * _sigmoid(G[a:b]) * U[a:b]
        y[a:b] = A @ _f64(Wd[e]).T
    return y, G, U


def grouped_ffn_bwd(dy_p, x_p, G, U, seg_offsets, Wg, Wu, Wd):
    """Backward of grouped_ffn_fwd.

    dA = dY Wd;  s = sigmoid(G);  dG = dA * U * s*(1 + G*(1-s));
    dU = dA * G*s;  dWd[e] = dY_e^T A_e;  dX = dG Wg + dU Wu;
    dWg[e] = dG_e^T X_e;  dWu[e] = dU_e^T X_e.  Empty experts get zero dW.
    """
    seg = np.asarray(seg_offsets)
    E, F, H = Wg.shape
    R = x_p.shape[0]
    dx = np.zeros((R, H), F64)
    dWg = np.zeros((E, F, H), F64)
    dWu = np.zeros((E, F, H), F64)
    dWd = np.zeros((E, H, F), F64)
    for e in range(E):
        a, b = int(seg[e]), int(seg[e + 1])
        if b <= a:
            continue
        X = _f64(x_p[a:b])
        dY = _f64(dy_p[a:b])
        g = _f64(G[a:b])
        u = _f64(U[a:b])
        s = _sigmoid(g)
        A = g * s * u
        dA = dY @ _f64(Wd[e])
        dG = dA * u * (s * (1.0 + g * (1.0 - s)))
        dU = dA * (g * s)
        dWd[e] = dY.T @ A
        dx[a:b] = dG @ _f64(Wg[e]) + dU @ _f64(Wu[e])
        dWg[e] = dG.T @ X
        dWu[e] = dU.T @ X
    return dx, dWg, dWu, dWd


# --------------------------------------------------------------------------
# Combine and the backward of combine / permute / route
# --------------------------------------------------------------------------

def combine(y_p, dst_pos, gate_w, base, T):
    """out[t] = base[t] + sum over routed slots s (ascending) of
    gate_w[t,s] * y_p[dst_pos[t,s]].  base is None (zero) for MoE and the
    layer input for MoD / early exit, where unselected tokens pass through
    unchanged (Sec. 2.5, 2.6)."""
    dp = np.asarray(dst_pos)
    k = dp.shape[1]
    y = _f64(y_p)
    H = y.shape[1]
    out = np.zeros((T, H), F64) if base is None else _f64(base).copy()
    gw = _f64(gate_w)
    for s in range(k):
        routed = dp[:, s] >= 0
        rows = dp[routed, s]
        out[routed] += gw[routed, s][:, None] * y[rows]
    return out


def combine_bwd(dout, y_p, dst_pos, gate_w):
    """dy_p[p] = gate_w[t,s] * dout[t];  dgate[t,s] = <dout[t], y_p[p]>,
    with p = dst_pos[t,s]; zero dgate for unrouted slots."""
    dp = np.asarray(dst_pos)
    T, k = dp.shape
    y = _f64(y_p)
    do = _f64(dout)
    gw = _f64(gate_w)
    dy = np.zeros_like(y)
    dgate = np.zeros((T, k), F64)
    for s in range(k):
        routed = dp[:, s] >= 0
        rows = dp[routed, s]
        dy[rows] = gw[routed, s][:, None] * do[routed]
        dgate[routed, s] = np.einsum("th,th->t", do[routed], y[rows])
    return dy, dgate


def permute_bwd(dx_p, dst_pos, dbase):
    """dx[t] = dbase[t] + sum over routed slots of dx_p[dst_pos[t,s]].
    dbase is the upstream gradient when the layer has a pass-through residual
    (MoD, early exit) and None for MoE."""
    dp = np.asarray(dst_pos)
    T, k = dp.shape
    dxp = _f64(dx_p)
    H = dxp.shape[1]
    dx = np.zeros((T, H), F64) if dbase is None else _f64(dbase).copy()
    for s in range(k):
        routed = dp[:, s] >= 0
        dx[routed] += dxp[dp[routed, s]]
    return dx


def route_topk_bwd(dgate, gate_w, expert_idx, E):
    """Jacobian of the softmax over the k selected logits, scattered to the
    selected experts: dlogit[t,e_s] = w_s * (dgate_s - sum_j w_j dgate_j).
    The selection itself carries no gradient."""
    dg = _f64(dgate)
    w = _f64(gate_w)
    ei = np.asarray(expert_idx)
    T, k = ei.shape
    inner = (w * dg).sum(axis=1, keepdims=True)
    dsel = w * (dg - inner)
    dlogits = np.zeros((T, E), F64)
    np.put_along_axis(dlogits, ei.astype(np.int64), dsel, axis=1)
    return dlogits


def route_capacity_bwd(dgate, scores, expert_idx):
    """dscore[t] = sigmoid'(score[t]) * dgate[t] for selected tokens, else 0."""
    sc = _f64(scores).reshape(-1)
    s = _sigmoid(sc)
    sel = np.asarray(expert_idx).reshape(-1) >= 0
    return np.where(sel, s * (1.0 - s) * _f64(dgate).reshape(-1), 0.0)


# --------------------------------------------------------------------------
# Loads, imbalance, partitioning (Sec. 2, 2.1, 2.5, 2.6, 3.3, 5)
# --------------------------------------------------------------------------

def expert_counts(expert_idx, E):
    """Direct count of tokens per expert, |R^{-1}(e)| of Sec. 2.1."""
    flat = np.asarray(expert_idx).reshape(-1)
    return np.asarray([int(np.sum(flat == e)) for e in range(E)], dtype=I32)


def layer_load(seg_offsets, c_row):
    """Per-expert row counts from the segment offsets and the layer load
    sum_e counts[e] * c_row (Sec. 2.1; with one expert this is the
    (t_i/t)*c_i*t of Sec. 2.5 and r_i*t_i*c_i of Sec. 2.6)."""
    seg = np.asarray(seg_offsets, dtype=np.int64)
    counts = (seg[1:] - seg[:-1]).astype(I32)
    return counts, float(counts.astype(F64).sum() * c_row)


def worker_loads_moe(counts, expert_to_worker, n_workers, c_row):
    """Sec. 2.1: L_j = sum over experts e placed on worker j of
    sum over tokens routed to e of c_e."""
    L = np.zeros(n_workers, F64)
    for e, w in enumerate(expert_to_worker):
        L[w] += float(counts[e]) * c_row
    return L


def imbalance(L):
    """Sec. 2, Eq. 1-2: (L_max - L_min) / mean(L)."""
    L = _f64(L)
    return float((L.max() - L.min()) / (L.sum() / L.size))


def stage_loads(loads, bounds):
    """Sec. 2: L_i = sum of the costs of the layers assigned to stage i, for a
    contiguous assignment bounds[i] <= layer < bounds[i+1]."""
    loads = _f64(loads)
    return np.asarray([loads[bounds[i]:bounds[i + 1]].sum() for i in range(len(bounds) - 1)], F64)


def partition_dp(loads, S):
    """Optimal contiguous layer-to-stage split (Sec. 2 objective min_A max_i
    L_i restricted to contiguous stages, which is what the Partition balancer
    of Sec. 3.3 / Sec. 5 solves).  Exact dynamic program over prefix sums:
    best[s][j] = min over i of max(best[s-1][i], prefix[j] - prefix[i]).
    Stages may be empty only when L < S.  Returns the optimal bottleneck.
    """
    loads = _f64(loads)
    L = loads.size
    prefix = np.zeros(L + 1, F64)
    for i in range(L):
        prefix[i + 1] = prefix[i] + loads[i]
    INF = float("inf")
    best = [[INF] * (L + 1) for _ in range(S + 1)]
    best[0][0] = 0.0
    for s in range(1, S + 1):
        for j in range(0, L + 1):
            b = INF
            for i in range(0, j + 1):
                if best[s - 1][i] == INF:
                    continue
                v = max(best[s - 1][i], prefix[j] - prefix[i])
                if v < b:
                    b = v
            best[s][j] = b
    return float(best[S][L])


def partition_canonical_bounds(loads, S, bottleneck):
    """The canonical split at a given feasible bottleneck: walking left to
    right, each stage takes as many layers as fit under the bottleneck while
    leaving at least one layer for every later stage (when L >= S).
    Stage sums are prefix differences, as in partition_dp."""
    loads = _f64(loads)
    L = loads.size
    prefix = np.zeros(L + 1, F64)
    for i in range(L):
        prefix[i + 1] = prefix[i] + loads[i]
    bounds = [0]
    start = 0
    for s in range(S):
        remaining_stages = S - s - 1
        if s == S - 1:
            end = L
        else:
            end = start
            limit = L - remaining_stages if L >= S else L
            while end < limit and prefix[end + 1] - prefix[start] <= bottleneck:
                end += 1
            if L >= S and end == start:
                end = start + 1
        bounds.append(end)
        start = end
    return np.asarray(bounds, dtype=I32)


def partition_shadow(loads, shadow, S):
    """Partition with shadow layers (Sec. 4, Mixture of Depths: a block that is skipped is
    treated as a shadow layer when the layers are redistributed over the workers).

    Reading taken (the paper names the idea only): a shadow layer keeps its place in the
    layer order and its memory but adds no load.  A contiguous split is therefore judged
    first by its bottleneck max_i L_i, computed with the shadow layers' loads set to zero
    (the objective of Sec. 2), and among the splits that reach the optimal bottleneck by
    the largest number of layers any stage has to hold -- free layers can sit on either
    side of a boundary, so they are spread instead of piling up on one worker.  Stages are
    non-empty when L >= S.  Of the splits optimal in both, the canonical one lets each stage,
    from the left, take as many layers as both limits allow while leaving one layer for
    every later stage.

    Two exact dynamic programs over prefix sums, the second restricted to stages whose
    load stays under the first one's optimum:
      best[s][j]  = min_i max(best[s-1][i],  prefix[j] - prefix[i])
      count[s][j] = min_i max(count[s-1][i], j - i)   over i with prefix[j] - prefix[i] <= bottleneck
    Returns (bottleneck, max_layers, bounds int32 [S+1]).
    """
    loads = _f64(loads)
    L = loads.size
    eff = [0.0 if (shadow is not None and shadow[i]) else float(loads[i]) for i in range(L)]
    bottleneck = partition_dp(eff, S)
    prefix = [0.0] * (L + 1)
    for i in range(L):
        prefix[i + 1] = prefix[i] + eff[i]
    INF = float("inf")
    need_nonempty = L >= S
    count = [[INF] * (L + 1) for _ in range(S + 1)]
    count[0][0] = 0
    for s in range(1, S + 1):
        for j in range(0, L + 1):
            b = INF
            for i in range(0, j + 1):
                if count[s - 1][i] == INF or (need_nonempty and i == j):
                    continue
                if prefix[j] - prefix[i] <= bottleneck:
                    b = min(b, max(count[s - 1][i], j - i))
            count[s][j] = b
    max_layers = int(count[S][L])
    bounds = [0]
    start = 0
    for s in range(S):
        if s == S - 1:
            end = L
        else:
            limit = L - (S - s - 1) if need_nonempty else L
            end = start
            while end < limit and end - start < max_layers and prefix[end + 1] - prefix[start] <= bottleneck:
                end += 1
            if need_nonempty and end == start:
                end = start + 1
        bounds.append(end)
        start = end
    return bottleneck, max_layers, np.asarray(bounds, dtype=I32)


def uniform_bounds(L, S):
    """The static baseline the paper compares against: equal layer counts per
    stage (remainder to the first stages)."""
    base, rem = divmod(L, S)
    b = [0]
    for s in range(S):
        b.append(b[-1] + base + (1 if s < rem else 0))
    return np.asarray(b, dtype=I32)


def potential(stage_load):
    """Sec. 3.3 (proof of Lemma 2): phi = sum over unordered worker pairs of |x_u - x_v|."""
    x = _f64(stage_load)
    return float(sum(abs(x[u] - x[v]) for u in range(x.size) for v in range(u + 1, x.size)))


def diffusion_balance(loads, bounds, layer_mem=None, max_mem=float("inf"), gamma=0.0, max_rounds=10 ** 6):
    """Diffusion balancer (Sec. 3.3: iterative, decentralised; layers move from
    overloaded workers to underloaded neighbours; the potential phi of Lemma 2
    never increases and the run stops once phi <= gamma).

    The paper gives the idea, not a listing.  This reading is taken:
      * workers are the pipeline stages in order and a stage's neighbours are
        the stages next to it: a stage hands its last layer to the next stage
        or its first layer to the previous one, so stages stay contiguous;
      * one round = one transfer: among all single-layer transfers between
        neighbours that keep the source non-empty, fit the receiver's memory
        (sum of layer_mem on it + the layer <= max_mem) and strictly reduce
        phi, the one with the largest reduction is applied (ties: the lower
        boundary first, then the transfer towards the higher stage);
      * the run ends when phi <= gamma, when no transfer reduces phi, or after
        max_rounds rounds.
    loads[l] is the load of layer l (by Param or by Time), bounds the starting
    contiguous assignment.  Returns (bounds, history) with history[r] = phi
    after r rounds (history[0] = phi of the start).
    """
    loads = _f64(loads)
    b = [int(v) for v in bounds]
    S = len(b) - 1
    mem = np.zeros_like(loads) if layer_mem is None else _f64(layer_mem)

    def phi_of(bb):
        return potential(stage_loads(loads, bb))

    history = [phi_of(b)]
    for _ in range(max_rounds):
        if history[-1] <= gamma:
            break
        best = None
        for i in range(1, S):  # boundary between stage i-1 and stage i
            for to_right in (True, False):
                nb = list(b)
                if to_right:  # last layer of stage i-1 goes to stage i
                    layer, src, dst = b[i] - 1, i - 1, i
                    nb[i] -= 1
                else:         # first layer of stage i goes to stage i-1
                    layer, src, dst = b[i], i, i - 1
                    nb[i] += 1
                if b[src + 1] - b[src] <= 1:
                    continue
                if float(mem[b[dst]:b[dst + 1]].sum() + mem[layer]) > max_mem:
                    continue
                gain = history[-1] - phi_of(nb)
                if gain > 0 and (best is None or gain > best[0]):
                    best = (gain, nb)
        if best is None:
            break
        b = best[1]
        history.append(phi_of(b))
    return np.asarray(b, dtype=I32), history


def repack_first_fit(active_workers, mem_usage, num_layers, target_num_workers, max_mem):
    """First-fit consolidation onto fewer workers (Sec. 3.4, Algorithm 2).

    For every ordered pair src < dst: if the two memory footprints fit
    together under max_mem and more workers are active than the target, src is
    deactivated and each of its layers is listed as a transfer to dst, whose
    memory and layer count grow accordingly.

    The printed pseudo-code is silent on three points; this reading is taken:
      * a worker already emptied (inactive) is neither a source nor a target;
      * once src has been merged into a dst, it is not merged again;
      * src's own counters are left as they are (the listing never clears
        them) but are never read again because src is inactive.
    Returns (transfers, active_workers, mem_usage, num_layers) as new lists.
    """
    active = [int(a) for a in active_workers]
    mem = [float(m) for m in mem_usage]
    nl = [int(n) for n in num_layers]
    n = len(active)
    transfers = []
    for src in range(n):
        for dst in range(src + 1, n):
            if not active[src] or not active[dst]:
                continue
            if mem[src] + mem[dst] < max_mem and sum(active) > target_num_workers:
                active[src] = 0
                for lyr in range(nl[src]):
                    transfers.append((src, dst, lyr))
                mem[dst] += mem[src]
                nl[dst] += nl[src]
    return transfers, active, mem, nl


# --------------------------------------------------------------------------
# Whole-layer chains (the order the product calls its kernels in)
# --------------------------------------------------------------------------

def layer_fwd(x, expert_idx, gate_w, Wg, Wu, Wd, residual):
    """permute -> grouped FFN -> combine.  `residual` selects base = x
    (MoD / early exit) or base = 0 (MoE).  Returns a dict of every
    intermediate so tests can compare stage by stage."""
    E = Wg.shape[0]
    T = x.shape[0]
    x_p, seg, src_slot, dst_pos = permute(x, expert_idx, E)
    y_p, G, U = grouped_ffn_fwd(x_p, seg, Wg, Wu, Wd)
    out = combine(y_p, dst_pos, gate_w, x if residual else None, T)
    return dict(x_p=x_p, seg_offsets=seg, src_slot=src_slot, dst_pos=dst_pos,
                y_p=y_p, G=G, U=U, out=out)


def layer_bwd(dout, fwd, gate_w, Wg, Wu, Wd, residual):
    """combine_bwd -> grouped FFN bwd -> permute_bwd, given layer_fwd's dict."""
    dy_p, dgate = combine_bwd(dout, fwd["y_p"], fwd["dst_pos"], gate_w)
    dx_p, dWg, dWu, dWd = grouped_ffn_bwd(dy_p, fwd["x_p"], fwd["G"], fwd["U"],
                                          fwd["seg_offsets"], Wg, Wu, Wd)
    dx = permute_bwd(dx_p, fwd["dst_pos"], dout if residual else None)
    return dict(dy_p=dy_p, dgate=dgate, dx_p=dx_p, dWg=dWg, dWu=dWu, dWd=dWd, dx=dx)


def moe_layer(logits, x, Wg, Wu, Wd, k, dout):
    """Config-1/2/3 chain: top-k route, layer fwd, layer bwd, route bwd."""
    E = Wg.shape[0]
    idx, gate = route_topk(logits, k)
    fwd = layer_fwd(x, idx, gate, Wg, Wu, Wd, residual=False)
    bwd = layer_bwd(dout, fwd, gate, Wg, Wu, Wd, residual=False)
    dlogits = route_topk_bwd(bwd["dgate"], gate, idx, E)
    return dict(expert_idx=idx, gate_w=gate, dlogits=dlogits, **fwd, **bwd)


def mod_layer(scores, cap, x, Wg, Wu, Wd, dout):
    """Config-4 chain: selected tokens get x + sigmoid(score) * FFN(x), the
    others pass through (Sec. 2.6)."""
    idx, gate = route_capacity(scores, cap)
    fwd = layer_fwd(x, idx, gate, Wg, Wu, Wd, residual=True)
    bwd = layer_bwd(dout, fwd, gate, Wg, Wu, Wd, residual=True)
    dscores = route_capacity_bwd(bwd["dgate"], scores, idx)
    return dict(expert_idx=idx, gate_w=gate, dscores=dscores, **fwd, **bwd)


def early_exit_stack(exit_layer, x, weights, dout):
    """Config-5 chain: for l = 1..L, tokens with exit_layer >= l get
    x + FFN_l(x), exited tokens carry their state through (Sec. 2.5).
    Backward runs l = L..1.  `weights` is a list of (Wg, Wu, Wd), each with a
    leading expert dimension of 1.  Returns per-layer dicts plus out, dx and
    the per-layer active counts t_l."""
    L = len(weights)
    xs = [_f64(x)]
    fwds, gates = [], []
    for l in range(1, L + 1):
        idx, gate = route_active(exit_layer, l)
        Wg, Wu, Wd = weights[l - 1]
        f = layer_fwd(xs[-1], idx, gate, Wg, Wu, Wd, residual=True)
        f["expert_idx"] = idx
        fwds.append(f)
        gates.append(gate)
        xs.append(f["out"])
    d = _f64(dout)
    bwds = [None] * L
    for l in range(L, 0, -1):
        Wg, Wu, Wd = weights[l - 1]
        b = layer_bwd(d, fwds[l - 1], gates[l - 1], Wg, Wu, Wd, residual=True)
        bwds[l - 1] = b
        d = b["dx"]
    active = np.asarray([int(f["seg_offsets"][-1]) for f in fwds], dtype=I32)
    return dict(fwd=fwds, bwd=bwds, out=xs[-1], dx=d, active=active)
