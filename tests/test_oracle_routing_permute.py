"""Pins for the oracle's routing and permutation (CPU only).

None of these re-use the oracle's own formulation: top-k is checked against a
full sort written in pure Python, gates against closed forms, and permutation
against an independent checker of the properties that determine it uniquely.
"""
import math

import numpy as np
import pytest

from oracle import dynmo_oracle as orc


def brute_topk(row, k):
    order = sorted(range(len(row)), key=lambda e: (-float(row[e]), e))
    return order[:k]


def check_permutation(x, expert_idx, E, x_p, seg, src_slot, dst_pos):
    """Independent checker: the properties below fix the result uniquely."""
    T, k = expert_idx.shape
    flat = expert_idx.reshape(-1)
    routed = [i for i in range(T * k) if flat[i] >= 0]
    R = len(routed)
    assert seg[0] == 0 and seg[E] == R
    assert all(seg[e] <= seg[e + 1] for e in range(E))
    for e in range(E):
        assert seg[e + 1] - seg[e] == sum(1 for i in routed if flat[i] == e)
    dp = dst_pos.reshape(-1)
    assert sorted(int(dp[i]) for i in routed) == list(range(R))  # bijection onto [0,R)
    assert all(dp[i] == -1 for i in range(T * k) if flat[i] < 0)
    for e in range(E):
        seg_rows = src_slot[seg[e]:seg[e + 1]]
        assert all(flat[i] == e for i in seg_rows)
        assert all(seg_rows[j] < seg_rows[j + 1] for j in range(len(seg_rows) - 1))
    for i in routed:
        assert src_slot[dp[i]] == i
        assert np.array_equal(x_p[dp[i]], x[i // k])


@pytest.mark.parametrize("T,E,k,seed", [(37, 4, 2, 0), (16, 8, 8, 1), (50, 16, 4, 2), (9, 5, 1, 3), (20, 3, 3, 4)])
def test_topk_matches_full_sort(T, E, k, seed):
    rng = np.random.default_rng(seed)
    # few distinct values so that ties are common
    logits = rng.integers(-2, 3, size=(T, E)).astype(np.float32) * 0.5
    idx, gate = orc.route_topk(logits, k)
    for t in range(T):
        assert list(idx[t]) == brute_topk(logits[t], k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, gate = orc.route_topk(logits, k)
    for t in range(T):
        assert list(idx[t]) == brute_topk(logits[t], k)
        sel = [float(logits[t, e]) for e in idx[t]]
        den = sum(math.exp(v - sel[0]) for v in sel)
        for s in range(k):
            assert gate[t, s] == pytest.approx(math.exp(sel[s] - sel[0]) / den, rel=1e-14)


def test_topk_adversarial():
    E = 6
    eq = np.full((3, E), 0.25, np.float32)
    idx, gate = orc.route_topk(eq, 4)
    assert (idx == np.arange(4)).all()
    assert np.all(gate == 0.25)  # exactly 1/k
    z = np.array([[0.0, -0.0, 0.0, -0.0, -1.0, -1.0]], np.float32)
    idx, _ = orc.route_topk(z, 3)
    assert list(idx[0]) == [0, 1, 2]  # +0 and -0 are equal -> lower index
    d = np.array([[1.0, 3.0, 3.0, 2.0, 3.0, 0.0]], np.float32)
    idx, gate = orc.route_topk(d, 4)
    assert list(idx[0]) == [1, 2, 4, 3]
    idx, gate = orc.route_topk(d, 1)
    assert list(idx[0]) == [1] and gate[0, 0] == 1.0  # k=1 -> weight exactly 1
    idx, gate = orc.route_topk(d, 6)  # k = E
    assert list(idx[0]) == [1, 2, 4, 3, 0, 5]
    assert abs(gate.sum() - 1.0) < 1e-15
    assert np.all(np.diff(gate[0]) <= 0)  # weights follow the logit order


def test_capacity_matches_full_sort():
    rng = np.random.default_rng(5)
    B, S = 3, 41
    for cap in (0, 1, 7, 40, 41):
        scores = rng.integers(-3, 4, size=(B, S)).astype(np.float32)
        idx, gate = orc.route_capacity(scores, cap)
        idx = idx.reshape(B, S)
        gate = gate.reshape(B, S)
        for b in range(B):
            chosen = set(sorted(range(S), key=lambda t: (-float(scores[b, t]), t))[:cap])
            for t in range(S):
                if t in chosen:
                    assert idx[b, t] == 0
                    assert gate[b, t] == pytest.approx(1.0 / (1.0 + math.exp(-float(scores[b, t]))), rel=1e-15)
                else:
                    assert idx[b, t] == -1 and gate[b, t] == 0.0
    idx, gate = orc.route_capacity(np.zeros((1, 8), np.float32), 3)
    assert list(idx[:, 0]) == [0, 0, 0, -1, -1, -1, -1, -1]
    assert np.all(gate[:3, 0] == 0.5)  # sigmoid(0)


def test_route_active():
    ex = np.array([1, 5, 2, 3, 1, 4], np.int32)
    for l in range(1, 6):
        idx, gate = orc.route_active(ex, l)
        assert list(idx[:, 0]) == [0 if e >= l else -1 for e in ex]
        assert list(gate[:, 0]) == [1.0 if e >= l else 0.0 for e in ex]


@pytest.mark.parametrize("T,E,k,seed", [(64, 4, 2, 0), (33, 7, 3, 1), (10, 2, 2, 2)])
def test_permute_is_the_unique_stable_grouping(T, E, k, seed):
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, _ = orc.route_topk(logits, k)
    x = rng.standard_normal((T, 5)).astype(np.float32)
    x_p, seg, src, dst = orc.permute(x, idx, E)
    check_permutation(x, idx, E, x_p, seg, src, dst)
    assert seg[E] == T * k  # dropless: segment sizes sum to tokens x k


def test_permute_with_unrouted_and_empty():
    rng = np.random.default_rng(3)
    T = 40
    ei = np.where(rng.random((T, 1)) < 0.3, 0, -1).astype(np.int32)
    x = rng.standard_normal((T, 3)).astype(np.float32)
    x_p, seg, src, dst = orc.permute(x, ei, 1)
    check_permutation(x, ei, 1, x_p, seg, src, dst)
    # compaction keeps ascending token order
    assert list(src) == [t for t in range(T) if ei[t, 0] == 0]
    # an expert nobody picks gets an empty segment; nothing routed at all
    ei2 = np.full((T, 1), -1, np.int32)
    x_p, seg, src, dst = orc.permute(x, ei2, 3)
    assert list(seg) == [0, 0, 0, 0] and x_p.shape == (0, 3) and np.all(dst == -1)
    ei3 = np.array([[2], [0], [2], [2]], np.int32)
    x_p, seg, src, dst = orc.permute(x[:4], ei3, 3)
    assert list(seg) == [0, 1, 1, 4] and list(src) == [1, 0, 2, 3] and list(dst[:, 0]) == [1, 0, 2, 3]


def test_counts_and_loads():
    rng = np.random.default_rng(4)
    T, E, k, H, F = 100, 8, 2, 16, 24
    idx, _ = orc.route_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    _, seg, _, _ = orc.permute(np.zeros((T, 1), np.float32), idx, E)
    counts, load = orc.layer_load(seg, 18 * H * F)
    assert np.array_equal(counts, np.bincount(idx.reshape(-1), minlength=E))
    assert np.array_equal(counts, orc.expert_counts(idx, E))
    assert counts.sum() == T * k and load == T * k * 18 * H * F
    # Sec. 2.1: worker load = sum over its experts of tokens x cost
    L = orc.worker_loads_moe(counts, [0, 0, 1, 1, 2, 2, 3, 3], 4, 2.0)
    assert list(L) == [2.0 * (counts[2 * j] + counts[2 * j + 1]) for j in range(4)]
    # Sec. 2.6: MoD load = capacity fraction x dense cost
    idx, _ = orc.route_capacity(rng.standard_normal((4, 64)).astype(np.float32), 8)
    _, seg, _, _ = orc.permute(np.zeros((256, 1), np.float32), idx, 1)
    counts, load = orc.layer_load(seg, 10.0)
    assert load == pytest.approx((8 / 64) * 256 * 10.0)
    # Sec. 2.5: t_l decreases with depth and equals #{exit >= l}
    ex = rng.geometric(0.3, size=500)
    prev = None
    for l in range(1, 6):
        idx, _ = orc.route_active(ex, l)
        _, seg, _, _ = orc.permute(np.zeros((500, 1), np.float32), idx, 1)
        t_l = int(seg[1])
        assert t_l == int((ex >= l).sum())
        assert prev is None or t_l <= prev
        prev = t_l


# ---- routing variants: biased selection, softmax over all experts, expert capacity ----

def _brute_topk(score_row, k):
    """k rounds of arg-max with the lower index winning ties."""
    live = list(range(len(score_row)))
    out = []
    for _ in range(k):
        best = live[0]
        for e in live[1:]:
            if score_row[e] > score_row[best]:
                best = e
        out.append(best)
        live.remove(best)
    return out


def test_route_topk_biased_reduces_to_plain():
    rng = np.random.default_rng(40)
    lg = rng.standard_normal((200, 8)).astype(np.float32)
    i0, w0 = orc.route_topk(lg, 2)
    i1, w1 = orc.route_topk_biased(lg, 2)
    assert np.array_equal(i0, i1) and np.allclose(w0, w1, rtol=1e-15, atol=0)
    i2, w2 = orc.route_topk_biased(lg, 2, bias=np.zeros(8, np.float32), norm="selected")
    assert np.array_equal(i0, i2) and np.array_equal(w1, w2)


def test_route_topk_biased_selection_and_weights():
    from scipy.special import softmax
    rng = np.random.default_rng(41)
    T, E, k = 300, 6, 3
    lg = rng.standard_normal((T, E)).astype(np.float32)
    lg[::7, 2] = lg[::7, 4]  # ties
    bias = np.array([0.5, -0.25, 0.0, 1.0, 0.0, -2.0], np.float32)
    idx, w = orc.route_topk_biased(lg, k, bias, norm="all")
    score = (lg + bias[None, :]).astype(np.float32)
    p = softmax(lg.astype(np.float64), axis=1)
    for t in range(T):
        assert list(idx[t]) == _brute_topk(score[t], k)
        assert np.allclose(w[t], p[t, idx[t]], rtol=1e-14)
    # the bias moves the selection but not the weights of whatever is selected
    idx_s, w_s = orc.route_topk_biased(lg, k, bias, norm="selected")
    assert np.array_equal(idx, idx_s)
    z = np.take_along_axis(lg.astype(np.float64), idx_s.astype(np.int64), axis=1)
    assert np.allclose(w_s, softmax(z, axis=1), rtol=1e-14)
    # all experts selected: the "all" weights are the whole softmax and sum to one
    idx_e, w_e = orc.route_topk_biased(lg, E, bias, norm="all")
    assert np.allclose(w_e.sum(axis=1), 1.0, rtol=1e-14)
    # a large bias forces the expert in
    big = np.zeros(E, np.float32)
    big[5] = 100.0
    assert (orc.route_topk_biased(lg, 1, big)[0][:, 0] == 5).all()


@pytest.mark.parametrize("norm", ["selected", "all"])
def test_route_topk_biased_bwd_matches_autograd(norm):
    import torch
    rng = np.random.default_rng(42)
    T, E, k = 50, 7, 3
    lg = rng.standard_normal((T, E)).astype(np.float32)
    bias = rng.standard_normal(E).astype(np.float32)
    dg = rng.standard_normal((T, k))
    idx, w = orc.route_topk_biased(lg, k, bias, norm)
    x = torch.tensor(lg.astype(np.float64), requires_grad=True)
    ti = torch.tensor(idx.astype(np.int64))
    if norm == "selected":
        g = torch.softmax(torch.gather(x, 1, ti), dim=1)
    else:
        g = torch.gather(torch.softmax(x, dim=1), 1, ti)
    assert np.allclose(g.detach().numpy(), w, rtol=1e-13)
    (g * torch.tensor(dg)).sum().backward()
    got = orc.route_topk_biased_bwd(dg, lg, idx, norm)
    assert np.allclose(got, x.grad.numpy(), rtol=1e-11, atol=1e-13)
    if norm == "selected":  # and the established backward agrees
        assert np.allclose(got, orc.route_topk_bwd(dg, w, idx, E), rtol=1e-12, atol=1e-14)


def test_capacity_drop_hand_and_properties():
    # experts chosen per flat slot: 0 0 1 0 1 1 0 ; capacity 2 -> third and fourth 0 and third 1 are dropped
    ei = np.array([[0, 0], [1, 0], [1, 1], [0, -1]], np.int32)
    kept = orc.capacity_drop(ei, 2, 2)
    assert kept.tolist() == [[0, 0], [1, -1], [1, -1], [-1, -1]]
    assert np.array_equal(orc.capacity_drop(ei, 2, 100), ei)
    assert (orc.capacity_drop(ei, 2, 0) == -1).all()
    rng = np.random.default_rng(43)
    for _ in range(20):
        T, k, E = int(rng.integers(1, 60)), int(rng.integers(1, 4)), int(rng.integers(1, 6))
        ei = rng.integers(-1, E, size=(T, k)).astype(np.int32)
        cap = int(rng.integers(0, T + 2))
        kept = orc.capacity_drop(ei, E, cap)
        flat, kf = ei.reshape(-1), kept.reshape(-1)
        for e in range(E):
            chosen = np.flatnonzero(flat == e)
            survivors = np.flatnonzero(kf == e)
            assert list(survivors) == list(chosen[:cap])  # the earliest `cap` slots stay
        assert ((kf == flat) | (kf == -1)).all()
