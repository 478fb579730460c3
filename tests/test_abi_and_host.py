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
    d = B.make_desc(8, 16, 16, 4, 2, "bf16")
    assert lib.dynmo_route_topk_ex(B.C.byref(d), None, None, 0, None, None, None) == -1
    assert lib.dynmo_route_topk_all_bwd(B.C.byref(d), None, None, None, None, None) == -1
    assert lib.dynmo_route_drop(B.C.byref(d), None, 4, None, None, 0, None) == -1
    assert lib.dynmo_grouped_ffn_fwd_gather(B.C.byref(d), None, None, None, None, None, None, None, None, None, None, 0,
                                            None) == -1
    big = B.make_desc(300000, 4096, 512, 8, 2, "bf16")  # x is 2.4 GB: beyond the gather call's 32-bit row offsets
    assert lib.dynmo_grouped_ffn_fwd_gather(B.C.byref(big), None, 16, None, None, None, None, None, None, None, None, 0,
                                            None) == -2
    # the folded combine: two slots per token; both or neither row source; too large to gather
    fold = lib.dynmo_grouped_ffn_fwd_combine
    one = B.make_desc(8, 16, 16, 4, 1, "bf16")
    assert fold(B.C.byref(d), 16, None, 16, 16, 16, 16, 16, 16, None, 16, None, 16, 16, 16, 1 << 30, None) == -1
    assert fold(B.C.byref(one), 16, 16, 16, 16, 16, 16, 16, 16, None, 16, None, 16, 16, 16, 1 << 30, None) == -1
    assert fold(B.C.byref(one), None, None, 16, 16, 16, 16, 16, 16, None, 16, None, 16, 16, 16, 1 << 30, None) == -1
    assert fold(B.C.byref(one), 16, None, 16, 16, 16, 16, 16, None, None, 16, None, 16, 16, 16, 1 << 30, None) == -1
    big1 = B.make_desc(300000, 4096, 512, 8, 1, "bf16")
    assert fold(B.C.byref(big1), None, 16, 16, 16, 16, 16, 16, 16, None, 16, None, 16, 16, 16, 1 << 30, None) == -2
    # row data moves in 16-byte pieces: a misaligned activation pointer is refused on the host
    ok = B.make_desc(8, 16, 16, 4, 2, "bf16")
    assert lib.dynmo_combine(B.C.byref(ok), 32, 16, 16, None, 48 + 2, None) == -1
    assert lib.dynmo_permute_bwd(B.C.byref(ok), 32 + 8, 16, None, 64, None) == -1
    assert lib.dynmo_permute(B.C.byref(ok), 32 + 4, 16, 64, 16, 16, 16, 16, 1 << 30, None) == -1
    assert lib.dynmo_grouped_ffn_fwd(B.C.byref(ok), 32, 16, 64, 96, 128 + 2, 160, 192, 224, 256, 1 << 30, None) == -1
    assert lib.dynmo_grouped_ffn_bwd(B.C.byref(ok), 32, 64, 96, 128, 16, 160, 192, 224, 256 + 8, 288, 320, 352, 384,
                                     1 << 30, None) == -1
    assert lib.dynmo_peak_copy(None, None, 16, None) == -1
    assert lib.dynmo_peak_mfma_bf16(0, None, None, None, None) == -1
    assert lib.dynmo_route_drop_workspace_bytes(B.C.byref(d)) > lib.dynmo_permute_workspace_bytes(B.C.byref(d))
    for bad in ([0, 2, 2, 5], [1, 2], [0, 3, 1, 2]):  # wrong end, wrong start, not monotone
        with pytest.raises(B.DynmoError):
            B.dynmo_diffusion([1.0, 2.0], bad)
    with pytest.raises(B.DynmoError):
        B.dynmo_diffusion([1.0, float("nan")], [0, 1, 2])
    with pytest.raises(B.DynmoError):
        B.dynmo_repack([1, 1], [1.0, 1.0], [1, -1], 1, 10.0)


def test_diffusion_and_repack_edge_cases():
    assert B.dynmo_diffusion([5.0], [0, 1]) == ([0, 1], 0, 0.0, 0.0)
    assert B.dynmo_diffusion([5.0, 3.0], [0, 1, 2]) == ([0, 1, 2], 0, 2.0, 2.0)  # one layer each: nothing may move
    # a stage that starts empty is filled (phi 6 -> 4 -> 0), exactly as the oracle does it
    b, rounds, phi0, phi1 = B.dynmo_diffusion([1.0, 2.0, 3.0], [0, 0, 3])
    rb, rh = orc.diffusion_balance([1.0, 2.0, 3.0], [0, 0, 3])
    assert (b, rounds, phi0, phi1) == (list(rb), len(rh) - 1, rh[0], rh[-1]) == ([0, 2, 3], 2, 6.0, 0.0)
    assert B.dynmo_potential([7.0]) == 0.0
    assert B.dynmo_repack([], [], [], 0, 1.0) == ([], [], [], [])
    # nothing to do when the target is already met
    assert B.dynmo_repack([1, 0, 1], [1.0, 9.0, 1.0], [2, 0, 2], 2, 10.0) == ([], [1, 0, 1], [1.0, 9.0, 1.0], [2, 0, 2])


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


def test_diffusion_golden(golden_dir):
    for S, start, loads, lmem, mmax, final, hist in read_golden(os.path.join(golden_dir, "diffusion_hand.txt")):
        loads = [float(v) for v in loads.split()]
        mem = None if lmem == "-" else [float(v) for v in lmem.split()]
        cap = float("inf") if mmax == "-" else float(mmax)
        h = [float(v) for v in hist.split()]
        b, rounds, phi0, phi1 = B.dynmo_diffusion(loads, [int(v) for v in start.split()], mem, cap)
        assert b == [int(v) for v in final.split()]
        assert (rounds, phi0, phi1) == (len(h) - 1, h[0], h[-1])


@pytest.mark.parametrize("seed", range(6))
def test_diffusion_matches_oracle(seed):
    """Same transfers as the oracle on integer-valued loads (every sum is exact, so both
    sides see the same gains and ties); on fractional loads the invariants."""
    rng = np.random.default_rng(300 + seed)
    for _ in range(20):
        L = int(rng.integers(2, 30))
        S = int(rng.integers(2, min(L, 8) + 1))
        cuts = sorted(rng.choice(np.arange(1, L), size=S - 1, replace=False))
        start = [0] + [int(c) for c in cuts] + [L]
        exact = seed % 2 == 0
        loads = [float(v) for v in (rng.integers(0, 60, size=L) if exact else rng.random(L) * 10.0)]
        mem, cap = None, float("inf")
        if seed % 3 == 0:
            mem = [float(v) for v in rng.integers(1, 4, size=L)]
            cap = float(max(sum(mem[start[i]:start[i + 1]]) for i in range(S)) + 2)
        gamma = float(rng.choice([0.0, 5.0, 50.0]))
        limit = int(rng.choice([1, 3, 1000]))
        b, rounds, phi0, phi1 = B.dynmo_diffusion(loads, start, mem, cap, gamma, limit)
        assert b[0] == 0 and b[-1] == L and all(b[i] < b[i + 1] for i in range(S))
        assert B.dynmo_potential(orc.stage_loads(loads, start)) == pytest.approx(phi0, rel=1e-13)
        assert orc.potential(orc.stage_loads(loads, b)) == pytest.approx(phi1, rel=1e-12, abs=1e-12)
        assert phi1 <= phi0 and rounds <= limit
        if mem is not None:
            assert all(sum(mem[b[i]:b[i + 1]]) <= cap for i in range(S))
        if exact:
            rb, rh = orc.diffusion_balance(loads, start, mem, cap, gamma, limit)
            assert b == list(rb) and rounds == len(rh) - 1 and phi0 == rh[0] and phi1 == rh[-1]


def test_repack_matches_oracle():
    cases = [([1, 1, 1, 1], [3, 4, 2, 6], [2, 3, 1, 2], 2, 10), ([1, 1, 1], [6, 6, 6], [1, 1, 1], 1, 10),
             ([1, 1], [1, 1], [4, 4], 2, 10), ([1, 1, 1], [5, 6, 2], [1, 1, 1], 2, 10), ([], [], [], 0, 1.0)]
    rng = np.random.default_rng(7)
    for _ in range(40):
        n = int(rng.integers(1, 9))
        cases.append(([int(v) for v in rng.integers(0, 2, size=n)], [float(v) for v in rng.integers(0, 12, size=n)],
                      [int(v) for v in rng.integers(0, 5, size=n)], int(rng.integers(0, n + 1)),
                      float(rng.integers(4, 30))))
    for act, mem, nl, target, cap in cases:
        got = B.dynmo_repack(act, mem, nl, target, cap)
        ref = orc.repack_first_fit(act, mem, nl, target, cap)
        assert got[0] == [tuple(t) for t in ref[0]]
        assert got[1] == ref[1] and got[2] == ref[2] and got[3] == ref[3]
    # a transfer list that does not fit is reported, with nothing changed
    with pytest.raises(B.DynmoError) as e:
        B.dynmo_repack([1, 1, 1, 1], [3, 4, 2, 6], [2, 3, 1, 2], 2, 10, capacity=1)
    assert e.value.status == -3


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_work_model():
    """The algorithmic work bench.py divides by: flops of the seven products add up to
    18 H F per routed row, and the row movers count each row once per direction."""
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_mod", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    from paper_2505_14864_amd import workloads as wl
    w = wl.CONFIGS[2]
    R = w.T * w.k
    flops = sum(bench.kernel_work(n, w, R, w.T)[1] for n in
                ("ffn_gateup", "ffn_down", "ffn_dA", "ffn_dX", "ffn_dWd", "ffn_dWg", "ffn_dWu"))
    assert flops == 18.0 * w.H * w.F * R
    assert bench.kernel_work("permute_rows", w, R, w.T) == ("hbm", (w.T + R) * w.H * 2 + 4.0 * w.T * w.k)
    assert bench.kernel_work("combine", w, R, w.T)[1] == (R + w.T) * w.H * 2 + 8.0 * w.T * w.k
    w4 = wl.CONFIGS[4]  # residual mode: the pass-through base is read too
    R4 = w4.B * w4.cap
    assert bench.kernel_work("combine", w4, R4, w4.T)[1] == (R4 + 2 * w4.T) * w4.H * 2 + 8.0 * w4.T
    assert bench.kernel_work("route_topk", w, R, w.T) is None


def test_product_and_oracle_do_not_import_each_other():
    """The product path never touches the oracle (no CPU fallback), the oracle never
    touches the product; only the seeded input generators are shared."""
    import ast
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

    def imported(path):
        names = set()
        for node in ast.walk(ast.parse(open(path).read())):
            if isinstance(node, ast.Import):
                names.update(a.name for a in node.names)
            elif isinstance(node, ast.ImportFrom):
                names.add(("." * node.level) + (node.module or ""))
                names.update("%s.%s" % (node.module or "", a.name) for a in node.names)
        return names

    pkg = os.path.join(root, "paper_2505_14864_amd")
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            assert not any("oracle" in n for n in imported(os.path.join(pkg, f))), f
    for f in os.listdir(os.path.join(root, "oracle")):
        if f.endswith(".py"):
            assert not any("paper_2505_14864_amd" in n or "binding" in n for n in imported(os.path.join(root, "oracle", f))), f
    # the input generators hold none of the method's arithmetic: no matmul, softmax, sort or top-k
    src = open(os.path.join(pkg, "workloads.py")).read()
    for word in ("matmul", "argsort", "softmax", "einsum", " @ "):
        assert word not in src, word


def _load_bench():
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_mod2", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    return bench


def test_bench_quotes_measured_traffic_only_for_the_code_it_was_measured_on(tmp_path, monkeypatch):
    """roofline.traffic comes from a counter summary under profiles/ that records the hash of the kernel
    sources it was taken on: the table must parse and give at least the kernel's algorithmic bytes when
    the hash matches the tree, give (None, stale) when it does not, and nothing for a kernel or
    configuration it lacks."""
    bench = _load_bench()
    from paper_2505_14864_amd import workloads as wl
    w = wl.CONFIGS[2]
    R = w.T * w.k
    prof = tmp_path / "profiles"
    prof.mkdir()
    table = ("kernel                            read MB   written MB     total MB algorithmic MB    ratio\n"
             "ffn_dX                             4970.5        126.7       5097.3         2415.9     2.11\n"
             "permute_rows_kernel                  33.7         67.1        100.8          100.7     1.00\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "kernel_sources_hash", lambda: "0123456789abcdef")
    (prof / "hbm_traffic_config2_x.txt").write_text("header\nkernel sources: 0123456789abcdef\n\n" + table)
    assert bench.measured_traffic(2, "ffn_dX") == (5097300000, False)
    rows_moved, stale = bench.measured_traffic(2, "permute_rows")
    assert not stale and abs(rows_moved - bench.kernel_work("permute_rows", w, R, w.T)[1]) < 0.02 * rows_moved
    assert bench.measured_traffic(2, "no_such_kernel") == (None, False)
    assert bench.measured_traffic(1, "ffn_dX") == (None, False)
    # the same summary after the kernels have changed, and one that records no hash at all
    monkeypatch.setattr(bench, "kernel_sources_hash", lambda: "fedcba9876543210")
    assert bench.measured_traffic(2, "ffn_dX") == (None, True)
    (prof / "hbm_traffic_config2_x.txt").write_text("header\n\n" + table)
    assert bench.measured_traffic(2, "ffn_dX") == (None, True)


def test_kernel_sources_hash_follows_the_sources(tmp_path, monkeypatch):
    bench = _load_bench()
    real = bench.kernel_sources_hash()
    assert len(real) == 16 and real == bench.kernel_sources_hash()
    csrc = tmp_path / "paper_2505_14864_amd" / "csrc"
    csrc.mkdir(parents=True)
    (csrc / "a.hip").write_text("one")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    h1 = bench.kernel_sources_hash()
    (csrc / "a.hip").write_text("two")
    assert bench.kernel_sources_hash() != h1


def test_committed_traffic_summaries_name_their_sources():
    """Every committed HBM-traffic summary carries the `kernel sources:` line the bench checks."""
    import glob
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for path in glob.glob(os.path.join(root, "profiles", "hbm_traffic_*.txt")):
        assert any(l.startswith("kernel sources: ") for l in open(path)), path


def test_partition_shadow_matches_oracle():
    """The library's shadow-layer split against the oracle's two dynamic programs (themselves
    pinned by enumeration and hand-worked cases), on random loads, shadow sets and stage counts."""
    rng = np.random.default_rng(5)
    for trial in range(200):
        L = int(rng.integers(0, 40))
        S = int(rng.integers(1, 9))
        integral = trial % 2 == 0
        loads = rng.integers(0, 50, size=L).astype(float) if integral else rng.random(L) * 10
        shadow = (rng.random(L) < rng.random()).astype(int)
        if L == 0:
            bounds, bott, most = B.dynmo_partition_shadow(loads, shadow, S)
            assert bounds == [0] * (S + 1) and bott == 0.0 and most == 0
            continue
        bounds, bott, most = B.dynmo_partition_shadow(loads, shadow, S)
        ref_b, ref_m, ref_bounds = orc.partition_shadow(loads, shadow, S)
        assert bott == ref_b and most == ref_m and bounds == list(ref_bounds), (loads, shadow, S)
    # no shadow flags: the Partition balancer's bottleneck
    loads = [7.0, 2.0, 5.0, 10.0, 8.0]
    assert B.dynmo_partition_shadow(loads, None, 3)[1] == B.dynmo_partition(loads, 3)[1] == 14.0
    with pytest.raises(B.DynmoError):
        B.dynmo_partition_shadow([1.0, float("nan")], [0, 0], 2)
