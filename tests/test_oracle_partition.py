"""Pins for the oracle's load metrics, partitioner and re-pack (CPU only)."""
import itertools
import os

import numpy as np
import pytest

from oracle import dynmo_oracle as orc


def read_golden(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([c.strip() for c in line.split("|")])
    return rows


def brute_bottleneck(loads, S):
    """Enumerate every contiguous split into S non-empty stages."""
    L = len(loads)
    best = None
    for cuts in itertools.combinations(range(1, L), S - 1):
        b = (0,) + cuts + (L,)
        m = max(sum(loads[b[i]:b[i + 1]]) for i in range(S))
        best = m if best is None else min(best, m)
    return best


def test_imbalance_hand_values(golden_dir):
    for exp, loads in read_golden(os.path.join(golden_dir, "imbalance_hand.txt")):
        L = [float(v) for v in loads.split()]
        assert orc.imbalance(L) == pytest.approx(float(exp), rel=1e-15, abs=1e-15)


def test_partition_hand_values(golden_dir):
    for S, bott, bounds, loads in read_golden(os.path.join(golden_dir, "partition_hand.txt")):
        S = int(S)
        L = [float(v) for v in loads.split()]
        b = orc.partition_dp(L, S)
        assert b == float(bott)
        cb = orc.partition_canonical_bounds(L, S, b)
        assert list(cb) == [int(v) for v in bounds.split()]
        assert orc.stage_loads(L, cb).max() == b


@pytest.mark.parametrize("seed", range(6))
def test_partition_dp_equals_enumeration(seed):
    rng = np.random.default_rng(seed)
    for _ in range(10):
        L = int(rng.integers(1, 12))
        S = int(rng.integers(1, L + 1))
        loads = [float(v) for v in rng.integers(0, 50, size=L)]  # integer-valued: sums are exact
        b = orc.partition_dp(loads, S)
        assert b == brute_bottleneck(loads, S)
        cb = orc.partition_canonical_bounds(loads, S, b)
        assert cb[0] == 0 and cb[-1] == L and all(cb[i] < cb[i + 1] for i in range(S))
        assert orc.stage_loads(loads, cb).max() == b


def test_partition_special_cases():
    assert orc.partition_dp([3.0] * 12, 4) == 9.0
    assert list(orc.partition_canonical_bounds([3.0] * 12, 4, 9.0)) == [0, 3, 6, 9, 12]
    assert orc.partition_dp([1, 1, 50, 1, 1], 5) == 50.0
    assert list(orc.uniform_bounds(10, 4)) == [0, 3, 6, 8, 10]
    # balancing never does worse than the static equal-count split
    rng = np.random.default_rng(1)
    loads = np.sort(rng.integers(1, 100, size=24))[::-1].astype(float)  # early-exit-like decay
    ub = orc.stage_loads(loads, orc.uniform_bounds(24, 6))
    b = orc.partition_dp(loads, 6)
    pb = orc.stage_loads(loads, orc.partition_canonical_bounds(loads, 6, b))
    assert pb.max() <= ub.max()
    assert pb.max() == b
    # fewer layers than stages: trailing stages are empty
    assert orc.partition_dp([5.0, 7.0], 4) == 7.0


def test_repack_hand_trace():
    """Algorithm 2 traced by hand on four workers, MAX_MEM = 10.
    mem = [3,4,2,6], layers = [2,3,1,2], target 2.
    (0,1): 3+4<10, 4>2 -> merge 0 into 1: mem1=7, layers1=5, active=3.
    (1,2): 7+2<10, 3>2 -> merge 1 into 2: mem2=9, layers2=6, active=2.
    (2,3): active == target -> stop."""
    tr, act, mem, nl = orc.repack_first_fit([1, 1, 1, 1], [3, 4, 2, 6], [2, 3, 1, 2], 2, 10)
    assert tr == [(0, 1, 0), (0, 1, 1)] + [(1, 2, i) for i in range(5)]
    assert act == [0, 0, 1, 1] and mem[2] == 9 and nl[2] == 6
    # memory bound blocks every merge
    tr, act, _, _ = orc.repack_first_fit([1, 1, 1], [6, 6, 6], [1, 1, 1], 1, 10)
    assert tr == [] and act == [1, 1, 1]
    # already at the target
    tr, act, _, _ = orc.repack_first_fit([1, 1], [1, 1], [4, 4], 2, 10)
    assert tr == []
    # first fit skips a partner that does not fit and takes the next one
    tr, act, mem, nl = orc.repack_first_fit([1, 1, 1], [5, 6, 2], [1, 1, 1], 2, 10)
    assert tr == [(0, 2, 0)] and act == [0, 1, 1] and mem[2] == 7


def _opt(field, cast):
    return None if field.strip() == "-" else cast(field)


def test_diffusion_hand_traces(golden_dir):
    for S, start, loads, lmem, mmax, final, hist in read_golden(os.path.join(golden_dir, "diffusion_hand.txt")):
        loads = [float(v) for v in loads.split()]
        mem = _opt(lmem, lambda f: [float(v) for v in f.split()])
        cap = _opt(mmax, float)
        b, h = orc.diffusion_balance(loads, [int(v) for v in start.split()], mem,
                                     float("inf") if cap is None else cap)
        assert list(b) == [int(v) for v in final.split()]
        assert h == [float(v) for v in hist.split()]
        assert len(b) == int(S) + 1


def test_potential_closed_form():
    """Sum of pairwise gaps = sum_i (2i - n + 1) x_(i) over the ascending order statistics."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        x = rng.integers(0, 1000, size=int(rng.integers(1, 9))).astype(float)
        xs = np.sort(x)
        n = xs.size
        assert orc.potential(x) == float(sum((2 * i - n + 1) * xs[i] for i in range(n)))
    assert orc.potential([5.0]) == 0.0
    assert orc.potential([3.0, 3.0, 3.0]) == 0.0


@pytest.mark.parametrize("seed", range(5))
def test_diffusion_properties(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(8):
        L = int(rng.integers(2, 14))
        S = int(rng.integers(2, min(L, 6) + 1))
        loads = [float(v) for v in rng.integers(1, 40, size=L)]
        cuts = sorted(rng.choice(np.arange(1, L), size=S - 1, replace=False))
        start = [0] + [int(c) for c in cuts] + [L]
        b, h = orc.diffusion_balance(loads, start)
        # phi falls strictly every round and the stages stay a contiguous, non-empty cover
        assert all(h[i + 1] < h[i] for i in range(len(h) - 1))
        assert b[0] == 0 and b[-1] == L and all(b[i] < b[i + 1] for i in range(S))
        x = orc.stage_loads(loads, b)
        assert h[-1] == orc.potential(x)
        # it never beats the exact optimum of the Partition objective, and it never ends worse than it started
        assert x.max() >= orc.partition_dp(loads, S)
        assert orc.potential(x) <= orc.potential(orc.stage_loads(loads, start))
        # the end state is a local optimum: no single neighbour transfer lowers phi
        for i in range(1, S):
            for d in (-1, 1):
                nb = list(b)
                nb[i] += d
                if nb[i] <= nb[i - 1] or nb[i] >= nb[i + 1]:
                    continue
                assert orc.potential(orc.stage_loads(loads, nb)) >= h[-1]
        # stopping rules
        b0, h0 = orc.diffusion_balance(loads, start, gamma=h[0])
        assert list(b0) == start and h0 == [h[0]]
        b1, h1 = orc.diffusion_balance(loads, start, max_rounds=1)
        assert len(h1) <= 2 and h1 == h[:len(h1)]


def test_diffusion_respects_memory():
    loads = [9.0, 1.0, 1.0, 1.0, 1.0, 1.0]
    mem = [1.0] * 6
    b, _ = orc.diffusion_balance(loads, [0, 3, 6], mem, max_mem=4.0)
    for i in range(2):
        assert b[i + 1] - b[i] <= 4
    free, _ = orc.diffusion_balance(loads, [0, 3, 6])
    assert list(free) == [0, 1, 6]          # 9 | 5 without the cap
    assert list(b) == [0, 2, 6]             # 10 | 4: stage 1 may hold four layers at most


# --------------------------------------------------------------------------
# shadow layers (Sec. 4, Mixture of Depths)
# --------------------------------------------------------------------------

def _shadow_bruteforce(loads, shadow, S):
    """All contiguous splits into S non-empty stages, judged by (bottleneck, most layers on a
    stage), ties by the lexicographically largest bounds (= every stage takes all it can)."""
    import itertools
    L = len(loads)
    eff = [0.0 if shadow[i] else float(loads[i]) for i in range(L)]
    best = None
    for cuts in itertools.combinations(range(1, L), S - 1):
        b = (0,) + cuts + (L,)
        sums = [sum(eff[b[s]:b[s + 1]]) for s in range(S)]
        key = (max(sums), max(b[s + 1] - b[s] for s in range(S)), tuple(-v for v in b))
        if best is None or key < best[0]:
            best = (key, b)
    return best[0][0], best[0][1], list(best[1])


def test_partition_shadow_hand_values(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "partition_shadow_hand.txt")):
        if line.startswith("#") or not line.strip():
            continue
        S, bott, most, bounds, loads, shadow = [f.strip() for f in line.split("|")]
        loads = [float(v) for v in loads.split()]
        shadow = [int(v) for v in shadow.split()]
        got = orc.partition_shadow(loads, shadow, int(S))
        assert got[0] == float(bott) and got[1] == int(most), line
        assert list(got[2]) == [int(v) for v in bounds.split()], line
        n += 1
    assert n >= 5


@pytest.mark.parametrize("seed", range(6))
def test_partition_shadow_equals_enumeration(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(40):
        L = int(rng.integers(2, 11))
        S = int(rng.integers(1, L + 1))
        loads = rng.integers(0, 9, size=L).astype(float)
        shadow = (rng.random(L) < 0.4).astype(int)
        bott, most, bounds = orc.partition_shadow(loads, shadow, S)
        ref = _shadow_bruteforce(loads, shadow, S)
        assert (bott, most, list(bounds)) == ref, (loads, shadow, S)


def test_partition_shadow_reduces_to_partition():
    # with no shadow layer the bottleneck is the Partition balancer's, and flagging a layer as
    # shadow can only lower it
    rng = np.random.default_rng(7)
    for _ in range(30):
        L = int(rng.integers(3, 12))
        S = int(rng.integers(1, L + 1))
        loads = rng.integers(1, 20, size=L).astype(float)
        none = np.zeros(L, int)
        assert orc.partition_shadow(loads, none, S)[0] == orc.partition_dp(loads, S)
        some = (rng.random(L) < 0.5).astype(int)
        assert orc.partition_shadow(loads, some, S)[0] <= orc.partition_dp(loads, S)
