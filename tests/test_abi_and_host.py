"""CPU-only checks of the boundary: the built library exports every symbol the
header declares, and the host-side balancer calls match the oracle."""
import os
import re

import numpy as np
import pytest

from oracle import dynmo_oracle as orc
from paper_2505_14864_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dynmo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dynmo_[a-z0-9_]+)\s*\(", text)))


def declared_arity():
    text = open(os.path.join(ROOT, "include", "dynmo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    out = {}
    for name, args in re.findall(r"\b(dynmo_[a-z0-9_]+)\s*\(([^)]*)\)\s*;", text):
        args = args.strip()
        out[name] = 0 if args in ("", "void") else len(args.split(","))
    return out


def test_binding_arity_matches_header():
    arity = declared_arity()
    for name, (_, argtypes) in B.SIGNATURES.items():
        assert arity[name] == len(argtypes), name


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 20
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.SIGNATURES) == names  # the binding mirrors the header one to one
    assert B.dynmo_version() >= 1


def test_bad_arguments_are_rejected_without_a_gpu():
    lib = B.lib()
    d = B.make_desc(8, 16, 16, 4, 5, "bf16")  # k > E
    assert lib.dynmo_route_topk(B.C.byref(d), None, None, None, None) == -1
    d = B.make_desc(8, 16, 16, 4, 2, "bf16")
    assert lib.dynmo_route_topk(B.C.byref(d), None, None, None, None) == -1  # null pointers
    d = B.make_desc(8, 12, 16, 4, 2, "bf16")  # H not a multiple of 8
    assert lib.dynmo_combine(B.C.byref(d), None, None, None, None, None, None) == -2
    d = B.make_desc(8, 16, 16, 100, 2, "f32")  # too many experts
    assert lib.dynmo_permute_workspace_bytes(B.C.byref(d)) == 0
    with pytest.raises(B.DynmoError):
        B.dynmo_partition([1.0, -2.0], 2)


def read_golden(path):
    rows = []
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([c.strip() for c in line.split("|")])
    return rows


def test_host_balancer_golden(golden_dir):
    for exp, loads in read_golden(os.path.join(golden_dir, "imbalance_hand.txt")):
        assert B.dynmo_imbalance([float(v) for v in loads.split()]) == pytest.approx(float(exp), rel=1e-15, abs=1e-15)
    for S, bott, bounds, loads in read_golden(os.path.join(golden_dir, "partition_hand.txt")):
        L = [float(v) for v in loads.split()]
        b, val = B.dynmo_partition(L, int(S))
        assert val == float(bott) and b == [int(v) for v in bounds.split()]


@pytest.mark.parametrize("seed", range(8))
def test_partition_matches_oracle_dp(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(25):
        L = int(rng.integers(1, 40))
        S = int(rng.integers(1, 12))
        if seed % 2 == 0:
            loads = [float(v) for v in rng.integers(0, 1000, size=L)]  # exact sums
        else:
            loads = [float(v) for v in rng.random(L) * 10.0]
        bounds, val = B.dynmo_partition(loads, S)
        ref = orc.partition_dp(loads, S)
        assert val == ref  # both take stage sums as prefix differences
        assert bounds == list(orc.partition_canonical_bounds(loads, S, ref))
        st = B.dynmo_stage_loads(loads, bounds)
        np.testing.assert_allclose(st, orc.stage_loads(loads, bounds), rtol=1e-13, atol=1e-13)
        if sum(st) > 0:
            assert B.dynmo_imbalance(st) == pytest.approx(orc.imbalance(st), rel=1e-14)
        assert B.dynmo_uniform_bounds(L, S) == list(orc.uniform_bounds(L, S))
