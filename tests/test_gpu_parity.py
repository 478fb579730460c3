"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs.

Integer results (routing indices, permutation, counts) must match bit for bit;
floating results within the norm-wise tolerance in parity_helpers.TOL.
"""
import numpy as np
import pytest
import torch

from oracle import dynmo_oracle as orc
from paper_2505_14864_amd import binding as B
from paper_2505_14864_amd import workloads as wl
from paper_2505_14864_amd.layer import RoutedFFNLayer, to_device, to_host
from parity_helpers import TOL, assert_close, check_layer_full, check_layer_sampled, f32_inputs, sel

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


# --------------------------------------------------------------------------
# routing
# --------------------------------------------------------------------------

@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (7, 2, 1), (100, 3, 2), (333, 4, 2), (257, 5, 5), (4096, 8, 2), (1000, 16, 4),
                                   (515, 33, 7), (300, 64, 8), (64, 64, 64)])
@pytest.mark.parametrize("ties", [False, True])
def test_route_topk(T, E, k, ties):
    say("route_topk T=%d E=%d k=%d ties=%s" % (T, E, k, ties))
    rng = np.random.default_rng(T * 131 + E * 7 + k)
    if ties:
        logits = (rng.integers(-2, 3, size=(T, E)) * 0.5).astype(np.float32)
        logits[::3] = 0.0
        logits[1::5, ::2] = -0.0
    else:
        logits = rng.standard_normal((T, E)).astype(np.float32)
    d = B.make_desc(T, 8, 8, E, k, "bf16")
    ei = torch.empty((T, k), dtype=torch.int32, device="cuda")
    gw = torch.empty((T, k), dtype=torch.float32, device="cuda")
    B.dynmo_route_topk(d, to_device(logits), ei, gw)
    ref_idx, ref_gate = orc.route_topk(logits, k)
    assert np.array_equal(to_host(ei), ref_idx)
    assert_close("gate_w", to_host(gw), ref_gate, 1e-5)
    # backward
    dgate = rng.standard_normal((T, k)).astype(np.float32)
    dl = torch.empty((T, E), dtype=torch.float32, device="cuda")
    B.dynmo_route_topk_bwd(d, to_device(dgate), gw, ei, dl)
    assert_close("dlogits", to_host(dl), orc.route_topk_bwd(dgate, ref_gate, ref_idx, E), 1e-5)


@pytest.mark.parametrize("Bn,S,cap", [(1, 1, 1), (3, 41, 7), (2, 64, 0), (2, 64, 64), (4, 2048, 256), (2, 1024, 1),
                                      (3, 3000, 1500), (2, 1025, 1024), (2, 4096, 512), (2, 4097, 100),
                                      (1, 10000, 3333), (5, 2049, 2048), (2, 1024, 1023)])
@pytest.mark.parametrize("ties", [False, True])
def test_route_capacity(Bn, S, cap, ties):
    say("route_capacity B=%d S=%d cap=%d ties=%s" % (Bn, S, cap, ties))
    rng = np.random.default_rng(Bn * 1000 + S + cap)
    if ties:
        scores = rng.integers(-3, 4, size=(Bn, S)).astype(np.float32)
        scores[:, ::7] = -0.0
        scores[:, 1::7] = 0.0
    else:
        scores = rng.standard_normal((Bn, S)).astype(np.float32)
    T = Bn * S
    d = B.make_desc(T, 8, 8, 1, 1, "bf16")
    ei = torch.empty((T, 1), dtype=torch.int32, device="cuda")
    gw = torch.empty((T, 1), dtype=torch.float32, device="cuda")
    dsc = to_device(scores)
    B.dynmo_route_capacity(d, dsc, Bn, S, cap, ei, gw)
    ref_idx, ref_gate = orc.route_capacity(scores, cap)
    assert np.array_equal(to_host(ei), ref_idx)
    assert int((to_host(ei) >= 0).sum()) == Bn * cap
    assert_close("gate_w", to_host(gw), ref_gate, 1e-5)
    dgate = rng.standard_normal((T, 1)).astype(np.float32)
    ds = torch.empty((T,), dtype=torch.float32, device="cuda")
    B.dynmo_route_capacity_bwd(d, to_device(dgate), dsc, ei, ds)
    assert_close("dscores", to_host(ds), orc.route_capacity_bwd(dgate, scores, ref_idx), 1e-5)


@pytest.mark.parametrize("S,cap", [(2048, 300), (4096, 4095), (700, 1), (5000, 77)])
def test_route_capacity_degenerate_scores(S, cap):
    """Every score equal (the first cap positions win), then infinities and denormals around the threshold."""
    say("route_capacity degenerate S=%d cap=%d" % (S, cap))
    rng = np.random.default_rng(S + cap)
    rows = [np.zeros(S, np.float32), np.full(S, -2.5, np.float32)]
    r = rng.standard_normal(S).astype(np.float32)
    r[rng.integers(0, S, 5)] = np.inf
    r[rng.integers(0, S, 5)] = -np.inf
    r[rng.integers(0, S, 20)] = 1e-42
    r[rng.integers(0, S, 20)] = -1e-42
    rows.append(r)
    scores = np.stack(rows)
    Bn = len(rows)
    d = B.make_desc(Bn * S, 8, 8, 1, 1, "bf16")
    ei = torch.empty((Bn * S, 1), dtype=torch.int32, device="cuda")
    gw = torch.empty((Bn * S, 1), dtype=torch.float32, device="cuda")
    B.dynmo_route_capacity(d, to_device(scores), Bn, S, cap, ei, gw)
    ref_idx, ref_gate = orc.route_capacity(scores, cap)
    got = to_host(ei)
    assert np.array_equal(got, ref_idx)
    assert np.array_equal(np.nonzero(got.reshape(Bn, S)[0] >= 0)[0], np.arange(cap))
    assert_close("gate_w", to_host(gw), ref_gate, 1e-5)


def test_route_active():
    say("route_active")
    rng = np.random.default_rng(5)
    T = 1000
    ex = rng.geometric(0.3, size=T).astype(np.int32)
    d = B.make_desc(T, 8, 8, 1, 1, "bf16")
    ei = torch.empty((T, 1), dtype=torch.int32, device="cuda")
    gw = torch.empty((T, 1), dtype=torch.float32, device="cuda")
    for l in range(1, 6):
        B.dynmo_route_active(d, to_device(ex), l, ei, gw)
        ref_idx, ref_gate = orc.route_active(ex, l)
        assert np.array_equal(to_host(ei), ref_idx)
        assert np.array_equal(to_host(gw), ref_gate.astype(np.float32))


# --------------------------------------------------------------------------
# permute (integer part bit-exact, rows copied bit for bit)
# --------------------------------------------------------------------------

def run_permute(x, ei, E, dtype):
    T, k = ei.shape
    H = x.shape[1]
    d = B.make_desc(T, H, 8, E, k, dtype)
    dev = "cuda"
    x_p = torch.empty((T * k, H), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=dev)
    seg = torch.empty((E + 1,), dtype=torch.int32, device=dev)
    src = torch.full((max(T * k, 1),), -7, dtype=torch.int32, device=dev)
    dst = torch.empty((T, k), dtype=torch.int32, device=dev)
    ws = torch.empty((max(1, B.dynmo_permute_workspace_bytes(d)),), dtype=torch.uint8, device=dev)
    B.dynmo_permute(d, to_device(x), to_device(ei), x_p, seg, src, dst, ws)
    return x_p, seg, src, dst


@pytest.mark.parametrize("T,E,k,H,dtype", [(1, 1, 1, 8, "bf16"), (256, 4, 2, 128, "f32"), (1000, 8, 2, 64, "bf16"),
                                           (2049, 16, 4, 72, "bf16"), (5000, 64, 8, 8, "bf16"), (777, 3, 3, 12, "f32")])
def test_permute_moe(T, E, k, H, dtype):
    say("permute T=%d E=%d k=%d H=%d %s" % (T, E, k, H, dtype))
    rng = np.random.default_rng(T + E)
    bias = np.asarray([(e + 1.0) ** -1.2 for e in range(E)], np.float32) * 2
    ei, _ = orc.route_topk(rng.standard_normal((T, E)).astype(np.float32) + bias, k)
    x = rng.standard_normal((T, H)).astype(np.float32)
    xs = wl.round_to_bf16_bits(x) if dtype == "bf16" else x
    x_p, seg, src, dst = run_permute(xs, ei, E, dtype)
    rx, rseg, rsrc, rdst = orc.permute(wl.as_f32(xs), ei, E)
    R = int(rseg[-1])
    assert R == T * k
    assert np.array_equal(to_host(seg), rseg)
    assert np.array_equal(to_host(dst), rdst)
    assert np.array_equal(to_host(src)[:R], rsrc)
    assert np.array_equal(to_host(x_p)[:R], rx)


def test_permute_unrouted_empty_and_deterministic():
    say("permute unrouted/empty/determinism")
    rng = np.random.default_rng(9)
    T, H = 6000, 64
    # compaction: most tokens unrouted, E = 1
    ei = np.where(rng.random((T, 1)) < 0.125, 0, -1).astype(np.int32)
    xs = wl.round_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    x_p, seg, src, dst = run_permute(xs, ei, 1, "bf16")
    rx, rseg, rsrc, rdst = orc.permute(wl.as_f32(xs), ei, 1)
    R = int(rseg[-1])
    assert np.array_equal(to_host(seg), rseg) and np.array_equal(to_host(dst), rdst)
    assert np.array_equal(to_host(src)[:R], rsrc) and np.array_equal(to_host(x_p)[:R], rx)
    assert np.all(to_host(src)[R:] == -7)  # nothing written past the routed rows
    # nothing routed at all; and experts 1 and 3 of 5 empty
    ei0 = np.full((T, 1), -1, np.int32)
    _, seg0, _, dst0 = run_permute(xs, ei0, 1, "bf16")
    assert list(to_host(seg0)) == [0, 0] and np.all(to_host(dst0) == -1)
    ei5 = rng.choice(np.asarray([0, 2, 4], np.int32), size=(T, 1))
    x_p, seg, src, dst = run_permute(xs, ei5, 5, "bf16")
    rx, rseg, rsrc, rdst = orc.permute(wl.as_f32(xs), ei5, 5)
    assert np.array_equal(to_host(seg), rseg) and rseg[1] == rseg[2] and rseg[3] == rseg[4]
    assert np.array_equal(to_host(dst), rdst) and np.array_equal(to_host(src), rsrc)
    # repeated runs are bit-identical (no dependence on atomic ordering)
    for _ in range(10):
        _, seg2, src2, dst2 = run_permute(xs, ei5, 5, "bf16")
        assert torch.equal(seg2, seg) and torch.equal(src2, src) and torch.equal(dst2, dst)


# --------------------------------------------------------------------------
# whole layers at small sizes: every tensor compared element by element
# --------------------------------------------------------------------------

def run_moe(w, inp):
    layer = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, "moe")
    dev = {n: to_device(a) for n, a in inp.items()}
    layer.route_topk(dev["logits"])
    layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.route_bwd()
    torch.cuda.synchronize()
    return layer


SMALL_MOE = [
    wl.CONFIGS[1],                                                             # the tiny fp32 config itself
    wl.scaled(wl.CONFIGS[1], T=300, H=36, F=50, seed=11),                      # ragged everything, fp32
    wl.scaled(wl.CONFIGS[2], T=700, H=256, F=448, seed=12),                    # Mixtral recipe, several tiles + tail
    wl.scaled(wl.CONFIGS[3], T=640, H=128, F=88, seed=13),                     # LLaMA-MoE recipe, F not a tile multiple
    wl.scaled(wl.CONFIGS[2], T=33, H=64, F=64, E=8, k=2, seed=14),             # tiny segments, some experts empty
    wl.scaled(wl.CONFIGS[2], T=1, H=8, F=8, E=2, k=1, seed=15),                # a single token
]


@pytest.mark.parametrize("w", SMALL_MOE, ids=lambda w: "%s-T%d-H%d-F%d" % (w.dtype, w.T, w.H, w.F))
def test_moe_layer_small(w):
    say("moe layer %s T=%d H=%d F=%d E=%d k=%d" % (w.dtype, w.T, w.H, w.F, w.E, w.k))
    inp = wl.make_inputs(w, threads=1)
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    assert np.array_equal(to_host(layer.expert_idx), ref["expert_idx"])
    assert_close("gate_w", to_host(layer.gate_w), ref["gate_w"], 1e-5)
    errs = check_layer_full(layer, ref, w.dtype, assert_elementwise=True)
    assert_close("dlogits", to_host(layer.droute), ref["dlogits"], TOL[w.dtype])
    counts, load = layer.load()
    ref_counts, ref_load = orc.layer_load(ref["seg_offsets"], 18.0 * w.H * w.F)
    assert counts == list(ref_counts) and load == ref_load and sum(counts) == w.T * w.k
    say("  errs " + " ".join("%s=%.1e" % kv for kv in errs.items()))


def test_moe_layer_empty_expert_zero_dw():
    say("moe empty expert")
    w = wl.scaled(wl.CONFIGS[2], T=200, H=64, F=96, E=4, k=2, seed=21)
    inp = wl.make_inputs(w, threads=1)
    inp["logits"][:, 2] = -30.0
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    check_layer_full(layer, ref, w.dtype)
    for n in ("dWg", "dWu", "dWd"):
        assert not to_host(getattr(layer, n))[2].any()


@pytest.mark.parametrize("Bn,S,cap,H,F", [(4, 256, 32, 128, 256), (3, 100, 100, 64, 72), (2, 130, 0, 64, 64)])
def test_mod_layer_small(Bn, S, cap, H, F):
    say("mod layer B=%d S=%d cap=%d" % (Bn, S, cap))
    w = wl.scaled(wl.CONFIGS[4], T=Bn * S, B=Bn, S=S, cap=cap, H=H, F=F, seed=31)
    inp = wl.make_inputs(w, threads=1)
    layer = RoutedFFNLayer(w.T, H, F, 1, 1, "bf16", "mod")
    dev = {n: to_device(a) for n, a in inp.items()}
    layer.route_capacity(dev["scores"], cap)
    layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.route_bwd(dev["scores"])
    torch.cuda.synchronize()
    f = f32_inputs(inp)
    ref = orc.mod_layer(f["scores"], cap, f["x"], f["Wg"], f["Wu"], f["Wd"], f["dout"])
    assert np.array_equal(to_host(layer.expert_idx), ref["expert_idx"])
    check_layer_full(layer, ref, "bf16")
    assert_close("dscores", to_host(layer.droute), ref["dscores"], TOL["bf16"])
    counts, load = layer.load()
    assert counts == [Bn * cap]
    assert load == pytest.approx((cap / S) * w.T * 18.0 * H * F)  # Sec. 2.6: fraction x dense cost


def run_stack(w, inp):
    L = w.layers
    layers = [RoutedFFNLayer(w.T, w.H, w.F, 1, 1, "bf16", "early_exit") for _ in range(L)]
    dev = {n: to_device(a) for n, a in inp.items()}
    x = dev["x"]
    xs = [x]
    for l in range(L):
        layers[l].route_active(dev["exit_layer"], l + 1)
        xs.append(layers[l].forward(xs[-1], dev["Wg"][l], dev["Wu"][l], dev["Wd"][l]))
    g = dev["dout"]
    for l in range(L - 1, -1, -1):
        g = layers[l].backward(g, dev["Wg"][l], dev["Wu"][l], dev["Wd"][l])
    torch.cuda.synchronize()
    return layers, xs[-1], g


def test_early_exit_stack_small():
    say("early-exit stack small")
    w = wl.scaled(wl.CONFIGS[5], T=1500, H=128, F=192, seed=41)
    inp = wl.make_inputs(w, threads=1)
    layers, out, dx = run_stack(w, inp)
    f = f32_inputs(inp)
    weights = [(f["Wg"][l], f["Wu"][l], f["Wd"][l]) for l in range(w.layers)]
    ref = orc.early_exit_stack(inp["exit_layer"], f["x"], weights, f["dout"])
    loads = []
    for l in range(w.layers):
        rf, rb = ref["fwd"][l], ref["bwd"][l]
        assert np.array_equal(to_host(layers[l].expert_idx), rf["expert_idx"])
        assert np.array_equal(to_host(layers[l].seg_offsets), rf["seg_offsets"])
        assert np.array_equal(to_host(layers[l].dst_pos), rf["dst_pos"])
        R = int(rf["seg_offsets"][-1])
        assert np.array_equal(to_host(layers[l].src_slot)[:R], rf["src_slot"])
        for n in ("dWg", "dWu", "dWd"):
            assert_close("L%d %s" % (l, n), to_host(getattr(layers[l], n)), rb[n], TOL["bf16"])
        assert_close("L%d out" % l, to_host(layers[l].out), rf["out"], TOL["bf16"])
        counts, load = layers[l].load()
        assert counts == [int(ref["active"][l])]
        loads.append(load)
    assert_close("out", to_host(out), ref["out"], TOL["bf16"])
    assert_close("dx", to_host(dx), ref["dx"], TOL["bf16"])
    assert all(loads[i] >= loads[i + 1] for i in range(len(loads) - 1))  # Sec. 2.5: t_i decreases with depth
    # the exported load vector drives the host balancer
    bounds, bott = B.dynmo_partition(loads, 2)
    assert bott == orc.partition_dp(loads, 2)
    uni = B.dynmo_stage_loads(loads, B.dynmo_uniform_bounds(len(loads), 2))
    bal = B.dynmo_stage_loads(loads, bounds)
    assert max(bal) <= max(uni)


# --------------------------------------------------------------------------
# the benchmark configurations at full size: integer results in full, floating
# results on sampled rows / tokens / weight columns (see check_layer_sampled)
# --------------------------------------------------------------------------

def test_moe_full_size_every_element():
    """Config 2 (the graded workload) against a full oracle run: every element of every tensor,
    hence every 256 x 256 tile of every output, is compared (about ten seconds of float64 numpy)."""
    w = wl.CONFIGS[2]
    say("full-size config 2, every element: %s" % w.name)
    inp = wl.make_inputs(w, threads=16)
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    assert np.array_equal(to_host(layer.expert_idx), ref["expert_idx"])
    assert_close("gate_w", to_host(layer.gate_w), ref["gate_w"], 1e-5)
    errs = check_layer_full(layer, ref, w.dtype, assert_elementwise=True)
    assert_close("dlogits", to_host(layer.droute), ref["dlogits"], TOL[w.dtype])
    say("  " + "  ".join("%s %.1e" % kv for kv in sorted(errs.items())))


def test_mod_full_size_every_element():
    """Config 4 against a full oracle run, every element."""
    w = wl.CONFIGS[4]
    say("full-size config 4, every element: %s" % w.name)
    inp = wl.make_inputs(w, threads=16)
    layer = RoutedFFNLayer(w.T, w.H, w.F, 1, 1, "bf16", "mod")
    dev = {n: to_device(a) for n, a in inp.items()}
    layer.route_capacity(dev["scores"], w.cap)
    layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    torch.cuda.synchronize()
    f = f32_inputs(inp)
    ref = orc.mod_layer(f["scores"], w.cap, f["x"], f["Wg"], f["Wu"], f["Wd"], f["dout"])
    assert np.array_equal(to_host(layer.expert_idx), ref["expert_idx"])
    errs = check_layer_full(layer, ref, "bf16", assert_elementwise=True)
    say("  " + "  ".join("%s %.1e" % kv for kv in sorted(errs.items())))


@pytest.mark.parametrize("cfg", [2, 3])
def test_moe_full_size_sampled(cfg):
    w = wl.CONFIGS[cfg]
    say("full-size config %d: %s" % (cfg, w.name))
    inp = wl.make_inputs(w, threads=16)
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref_idx, ref_gate = orc.route_topk(f["logits"], w.k)
    assert np.array_equal(to_host(layer.expert_idx), ref_idx)
    assert_close("gate_w", to_host(layer.gate_w), ref_gate, 1e-5)
    rng = np.random.default_rng(cfg)
    info = check_layer_sampled(layer, f, ref_idx, ref_gate, False, w.dtype, rng)
    assert int(info["seg"][-1]) == w.T * w.k
    counts, load = layer.load()
    assert counts == list(np.bincount(ref_idx.reshape(-1), minlength=w.E)) and sum(counts) == w.T * w.k
    assert load == w.T * w.k * 18.0 * w.H * w.F
    say("  counts %s" % counts)


def test_mod_full_size_sampled():
    w = wl.CONFIGS[4]
    say("full-size config 4: %s" % w.name)
    inp = wl.make_inputs(w, threads=16)
    layer = RoutedFFNLayer(w.T, w.H, w.F, 1, 1, "bf16", "mod")
    dev = {n: to_device(a) for n, a in inp.items()}
    layer.route_capacity(dev["scores"], w.cap)
    layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    torch.cuda.synchronize()
    f = f32_inputs(inp)
    ref_idx, ref_gate = orc.route_capacity(f["scores"], w.cap)
    assert np.array_equal(to_host(layer.expert_idx), ref_idx)
    rng = np.random.default_rng(4)
    info = check_layer_sampled(layer, f, ref_idx, ref_gate, True, "bf16", rng, n_tokens=64)
    assert int(info["seg"][-1]) == w.B * w.cap
    # unselected tokens pass through bit for bit
    unsel = np.nonzero(ref_idx[:, 0] < 0)[0][:512]
    assert np.array_equal(to_host(layer.out)[unsel], f["x"][unsel])


def test_early_exit_full_size():
    w = wl.CONFIGS[5]
    say("full-size config 5: %s" % w.name)
    inp = wl.make_inputs(w, threads=16)
    layers, out, dx = run_stack(w, inp)
    f = f32_inputs(inp)
    ex = inp["exit_layer"]
    # integer results of every layer in full
    for l in range(w.layers):
        ref_idx, _ = orc.route_active(ex, l + 1)
        _, seg, src, dst = orc.permute(np.zeros((w.T, 1), np.float32), ref_idx, 1)
        assert np.array_equal(to_host(layers[l].expert_idx), ref_idx)
        assert np.array_equal(to_host(layers[l].seg_offsets), seg)
        assert np.array_equal(to_host(layers[l].dst_pos), dst)
        assert np.array_equal(to_host(layers[l].src_slot)[:int(seg[-1])], src)
    # a token's path through the stack depends on that token alone: run the
    # oracle stack on sampled tokens and compare their outputs and gradients
    rng = np.random.default_rng(5)
    toks = np.unique(np.concatenate([rng.integers(0, w.T, size=48), [0, w.T - 1]]))
    weights = [(f["Wg"][l], f["Wu"][l], f["Wd"][l]) for l in range(w.layers)]
    ref = orc.early_exit_stack(ex[toks], f["x"][toks], weights, f["dout"][toks])
    assert_close("out", sel(out, toks), ref["out"], TOL["bf16"])
    assert_close("dx", sel(dx, toks), ref["dx"], TOL["bf16"])
    for l in range(w.layers):
        assert_close("L%d out" % l, sel(layers[l].out, toks), ref["fwd"][l]["out"], TOL["bf16"])
    # layer 1 stands alone at full size (its input is the given x): all kernels
    # of one layer checked with the sampled comparison, upstream gradient = dout
    l1 = RoutedFFNLayer(w.T, w.H, w.F, 1, 1, "bf16", "early_exit")
    dev = {n: to_device(a) for n, a in inp.items()}
    for layer_no in (1, 3):
        l1.route_active(dev["exit_layer"], layer_no)
        l1.forward(dev["x"], dev["Wg"][0], dev["Wu"][0], dev["Wd"][0])
        l1.backward(dev["dout"], dev["Wg"][0], dev["Wu"][0], dev["Wd"][0])
        torch.cuda.synchronize()
        ref_idx, ref_gate = orc.route_active(ex, layer_no)
        f1 = dict(x=f["x"], dout=f["dout"], Wg=f["Wg"][0], Wu=f["Wu"][0], Wd=f["Wd"][0])
        check_layer_sampled(l1, f1, ref_idx, ref_gate, True, "bf16", rng)
    loads = [layers[l].load()[1] for l in range(w.layers)]
    assert all(loads[i] >= loads[i + 1] for i in range(w.layers - 1))
    say("  active rows per layer: %s" % [layers[l].load()[0][0] for l in range(w.layers)])


# --------------------------------------------------------------------------
# limits of the boundary, the profiling step, and a few more edge shapes
# --------------------------------------------------------------------------

def test_many_experts_and_slots():
    """E = 64 (the limit) with k = 8 (the combine limit), bf16, ragged sizes."""
    say("moe E=64 k=8")
    w = wl.scaled(wl.CONFIGS[3], T=300, H=64, F=72, E=64, k=8, seed=51)
    inp = wl.make_inputs(w, threads=1)
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    assert np.array_equal(to_host(layer.expert_idx), ref["expert_idx"])
    check_layer_full(layer, ref, w.dtype)
    assert_close("dlogits", to_host(layer.droute), ref["dlogits"], TOL[w.dtype])


def test_one_expert_takes_more_than_half():
    """An adversarial histogram: one expert gets most rows, one gets none."""
    say("moe adversarial histogram")
    w = wl.scaled(wl.CONFIGS[2], T=1500, H=128, F=256, E=8, k=2, seed=52)
    inp = wl.make_inputs(w, threads=1)
    inp["logits"][:, 3] += 6.0   # everybody's first choice
    inp["logits"][:, 5] -= 40.0  # nobody's choice
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    counts, _ = layer.load()
    assert counts[3] == w.T and counts[5] == 0
    check_layer_full(layer, ref, w.dtype)


def test_profiling_step_reports_every_kernel():
    """The per-kernel event timing of the profiling step: counts match the launches
    made while it was on, durations are positive, and it is off by default."""
    say("profiling step")
    w = wl.scaled(wl.CONFIGS[2], T=512, H=256, F=512, seed=53)
    inp = wl.make_inputs(w, threads=1)
    B.dynmo_profile_enable(False)
    B.dynmo_profile_reset()
    run_moe(w, inp)
    assert all(B.dynmo_profile_read(i)[1] == 0 for i in range(B.dynmo_profile_kernel_count()))
    B.dynmo_profile_enable(True)
    run_moe(w, inp)
    run_moe(w, inp)
    B.dynmo_profile_enable(False)
    got = {B.dynmo_profile_kernel_name(i): B.dynmo_profile_read(i) for i in range(B.dynmo_profile_kernel_count())}
    for name in ("route_topk", "permute_count", "permute_scan", "permute_scatter", "permute_rows", "ffn_gateup", "ffn_down",
                 "combine", "combine_bwd", "ffn_dA", "ffn_dX", "ffn_dWd", "ffn_dWg", "ffn_dWu", "permute_bwd",
                 "route_topk_bwd"):
        ms, n = got[name]
        assert n == 2 and ms > 0.0, name
    assert got["route_capacity"][1] == 0
    by_time = sum(ms for ms, n in got.values()) / 2  # the layer's "by Time" load (Sec. 5)
    assert 0.0 < by_time < 1000.0
    B.dynmo_profile_reset()


def test_bad_arguments_on_the_gpu():
    d = B.make_desc(64, 64, 64, 4, 2, "bf16")
    x = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    ei = torch.zeros((64, 2), dtype=torch.int32, device="cuda")
    small_ws = torch.empty((1,), dtype=torch.uint8, device="cuda")
    big = torch.empty((128, 64), dtype=torch.bfloat16, device="cuda")
    seg = torch.empty((5,), dtype=torch.int32, device="cuda")
    with pytest.raises(B.DynmoError) as e:
        B.dynmo_grouped_ffn_fwd(d, big, seg, big, big, big, big, big, big, small_ws)
    assert e.value.status == -3  # DYNMO_EWORKSPACE
    with pytest.raises(B.DynmoError) as e:
        B.dynmo_combine(d, big, ei, torch.zeros((64, 2), device="cuda"), x, x)
    assert e.value.status == -1  # out aliases base
    d9 = B.make_desc(64, 64, 64, 16, 9, "bf16")
    with pytest.raises(B.DynmoError) as e:
        B.dynmo_combine(d9, big, ei, torch.zeros((64, 2), device="cuda"), None, x)
    assert e.value.status == -2  # more than 8 slots


def test_peak_reference_kernels():
    """The two measurement aids: the copy moves the bytes, the MFMA loop reports its flops."""
    say("peak reference kernels")
    src = torch.arange(0, 1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    assert B.dynmo_peak_copy(dst, src) == 4 << 20
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    tail_src, tail_dst = src[: 1028], torch.zeros(1028, dtype=torch.int32, device="cuda")  # not a multiple of the block
    B.dynmo_peak_copy(tail_dst, tail_src)
    torch.cuda.synchronize()
    assert torch.equal(tail_dst, tail_src)
    sink = torch.zeros(256 * 512, dtype=torch.float32, device="cuda")
    flops = B.dynmo_peak_mfma_bf16(10, sink)
    torch.cuda.synchronize()
    assert flops == 256 * 8 * 10 * 8 * 32768.0
    assert bool(torch.isfinite(sink).all())
    operands = torch.randn(4096, device="cuda").to(torch.bfloat16)
    assert B.dynmo_peak_mfma_bf16(10, sink, operands) == flops
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())


GATHER_CASES = [
    ("moe", wl.CONFIGS[1]),                                                       # fp32, the generic kernels
    ("moe", wl.scaled(wl.CONFIGS[2], T=700, H=256, F=448, seed=61)),              # bf16 MFMA, several tiles + tail
    ("moe", wl.scaled(wl.CONFIGS[3], T=640, H=128, F=88, seed=62)),               # k = 4: four slots share a token row
    ("mod", wl.scaled(wl.CONFIGS[4], T=4 * 256, B=4, S=256, cap=32, H=128, F=256, seed=63)),  # most tokens unrouted
]


@pytest.mark.parametrize("mode,w", GATHER_CASES, ids=lambda v: v if isinstance(v, str) else "%s-T%d" % (v.dtype, v.T))
def test_forward_with_fused_gather(mode, w):
    """The forward pass that reads its rows through src_slot: bit-identical to the
    forward pass over the copied rows (same arithmetic, other addresses), and so within
    tolerance of the oracle; x_p is never written."""
    say("fused gather %s %s T=%d" % (mode, w.dtype, w.T))
    inp = wl.make_inputs(w, threads=1)
    dev = {n: to_device(a) for n, a in inp.items()}
    a = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, mode)
    b = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, mode)
    for layer in (a, b):
        if mode == "moe":
            layer.route_topk(dev["logits"])
        else:
            layer.route_capacity(dev["scores"], w.cap)
    b.x_p.fill_(7.0)
    a.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    b.forward_gather(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    torch.cuda.synchronize()
    R = int(to_host(a.seg_offsets)[-1])
    for n in ("seg_offsets", "src_slot", "dst_pos"):
        assert torch.equal(getattr(a, n)[:R] if n == "src_slot" else getattr(a, n),
                           getattr(b, n)[:R] if n == "src_slot" else getattr(b, n)), n
    for n in ("G", "U", "y_p"):
        assert torch.equal(getattr(a, n)[:R], getattr(b, n)[:R]), n
    assert torch.equal(a.out, b.out)
    assert bool((b.x_p == 7.0).all())
    f = f32_inputs(inp)
    if mode == "moe":
        ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    else:
        ref = orc.mod_layer(f["scores"], w.cap, f["x"], f["Wg"], f["Wu"], f["Wd"], f["dout"])
    assert_close("out", to_host(b.out), ref["out"], TOL[w.dtype])


@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (300, 6, 3), (1000, 8, 2), (513, 16, 4), (257, 64, 8), (64, 5, 5)])
@pytest.mark.parametrize("norm", ["selected", "all"])
def test_route_topk_variants(T, E, k, norm):
    """Biased selection and the two gate normalisations: indices bit-exact (ties and the
    fp32 logit + bias sum included), weights and the all-expert backward in fp32."""
    say("route_topk_ex T=%d E=%d k=%d %s" % (T, E, k, norm))
    rng = np.random.default_rng(700 + T + E)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    if E > 2:
        lg[::5, 1] = lg[::5, E - 1]          # exact ties
        lg[::9] = np.round(lg[::9] * 4) / 4  # many equal values
    bias = (rng.standard_normal(E) * 0.5).astype(np.float32)
    bias[0] = 0.0
    d = B.make_desc(T, 8, 8, E, k, "f32")
    ei = torch.empty((T, k), dtype=torch.int32, device="cuda")
    gw = torch.empty((T, k), dtype=torch.float32, device="cuda")
    dl = torch.empty((T, E), dtype=torch.float32, device="cuda")
    code = B.NORM_SELECTED if norm == "selected" else B.NORM_ALL
    for use_bias in (True, False):
        b = bias if use_bias else None
        B.dynmo_route_topk_ex(d, to_device(lg), to_device(bias) if use_bias else None, code, ei, gw)
        ref_i, ref_w = orc.route_topk_biased(lg, k, b, norm)
        assert np.array_equal(to_host(ei), ref_i)
        assert_close("gate_w", to_host(gw), ref_w, 1e-5)
        dg = rng.standard_normal((T, k)).astype(np.float32)
        if norm == "all":
            B.dynmo_route_topk_all_bwd(d, to_device(dg), to_device(lg), ei, dl)
        else:
            B.dynmo_route_topk_bwd(d, to_device(dg), gw, ei, dl)
        assert_close("dlogits", to_host(dl), orc.route_topk_biased_bwd(dg, lg, ref_i, norm), 1e-4)


@pytest.mark.parametrize("T,E,k,cap", [(1, 1, 1, 0), (50, 4, 2, 7), (3000, 8, 2, 300), (1500, 16, 4, 100000),
                                       (2500, 3, 1, 1)])
def test_route_drop(T, E, k, cap):
    say("route_drop T=%d E=%d k=%d cap=%d" % (T, E, k, cap))
    rng = np.random.default_rng(800 + T)
    ei = rng.integers(-1 if k == 1 else 0, E, size=(T, k)).astype(np.int32)
    d = B.make_desc(T, 8, 8, E, k, "f32")
    kept = torch.full((T, k), 77, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.dynmo_route_drop_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    B.dynmo_route_drop(d, to_device(ei), cap, kept, ws)
    assert np.array_equal(to_host(kept), orc.capacity_drop(ei, E, cap))


def test_moe_layer_with_expert_capacity():
    """Biased selection + capacity dropping + the whole layer, forward and backward: a
    dropped slot contributes nothing to the output and gets dgate = 0, while the routing
    backward still sees its weight."""
    say("moe layer with capacity")
    w = wl.scaled(wl.CONFIGS[2], T=600, H=128, F=192, E=8, k=2, seed=71)
    inp = wl.make_inputs(w, threads=1)
    f = f32_inputs(inp)
    bias = np.linspace(0.4, -0.4, w.E).astype(np.float32)
    cap = 120  # 1200 slots over 8 experts: the popular experts overflow
    layer = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, "moe")
    dev = {n: to_device(a) for n, a in inp.items()}
    chosen = torch.empty((w.T, w.k), dtype=torch.int32, device="cuda")
    B.dynmo_route_topk_ex(layer.d, dev["logits"], to_device(bias), B.NORM_SELECTED, chosen, layer.gate_w)
    ws = torch.empty(B.dynmo_route_drop_workspace_bytes(layer.d), dtype=torch.uint8, device="cuda")
    B.dynmo_route_drop(layer.d, chosen, cap, layer.expert_idx, ws)
    layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    B.dynmo_route_topk_bwd(layer.d, layer.dgate, layer.gate_w, chosen, layer.droute)
    torch.cuda.synchronize()
    idx, gate = orc.route_topk_biased(f["logits"], w.k, bias, "selected")
    kept = orc.capacity_drop(idx, w.E, cap)
    assert (kept == -1).sum() > 50 and np.array_equal(to_host(layer.expert_idx), kept)
    fwd = orc.layer_fwd(f["x"], kept, gate, f["Wg"], f["Wu"], f["Wd"], residual=False)
    bwd = orc.layer_bwd(f["dout"], fwd, gate, f["Wg"], f["Wu"], f["Wd"], residual=False)
    ref = dict(**fwd, **bwd)
    check_layer_full(layer, ref, w.dtype)
    counts, _ = layer.load()
    assert max(counts) <= cap and sum(counts) == int((kept >= 0).sum())
    assert not to_host(layer.dgate)[kept < 0].any()
    assert_close("dlogits", to_host(layer.droute), orc.route_topk_biased_bwd(bwd["dgate"], f["logits"], idx, "selected"),
                 TOL[w.dtype])


def test_moe_full_size_capacity_and_gather():
    """Config 2 at full size through the variants: biased selection, expert capacity that
    makes the two popular experts overflow, the whole layer checked on samples against the
    oracle; then the gather-fused forward must reproduce the copied-rows forward bit for bit."""
    w = wl.CONFIGS[2]
    say("full-size config 2 with capacity and fused gather")
    inp = wl.make_inputs(w, threads=16)
    f = f32_inputs(inp)
    dev = {n: to_device(a) for n, a in inp.items()}
    bias = np.linspace(0.05, -0.05, w.E).astype(np.float32)
    cap = 1100
    layer = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, "moe")
    chosen = torch.empty((w.T, w.k), dtype=torch.int32, device="cuda")
    B.dynmo_route_topk_ex(layer.d, dev["logits"], to_device(bias), B.NORM_SELECTED, chosen, layer.gate_w)
    ws = torch.empty(B.dynmo_route_drop_workspace_bytes(layer.d), dtype=torch.uint8, device="cuda")
    B.dynmo_route_drop(layer.d, chosen, cap, layer.expert_idx, ws)
    layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    torch.cuda.synchronize()
    idx, gate = orc.route_topk_biased(f["logits"], w.k, bias, "selected")
    kept = orc.capacity_drop(idx, w.E, cap)
    assert np.array_equal(to_host(chosen), idx) and np.array_equal(to_host(layer.expert_idx), kept)
    counts, _ = layer.load()
    assert max(counts) == cap and sum(counts) == int((kept >= 0).sum()) < w.T * w.k
    check_layer_sampled(layer, f, kept, gate, False, w.dtype, np.random.default_rng(91))
    other = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, "moe")
    other.expert_idx.copy_(layer.expert_idx)
    other.gate_w.copy_(layer.gate_w)
    other.forward_gather(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    torch.cuda.synchronize()
    R = sum(counts)
    for n in ("G", "U", "y_p"):
        assert torch.equal(getattr(layer, n)[:R], getattr(other, n)[:R]), n
    assert torch.equal(layer.out, other.out)


@pytest.mark.parametrize("H,F", [(512, 1536), (256, 4096), (768, 2048)])
def test_split_last_round_small_problem(H, F):
    """Few output tiles and a long contraction: the down and dX products split their tiles
    along k over the XCDs (for F = 1536 into three chunks, the middle one straddling the
    two phases of dX) and a second pass sums the partial tiles; full check against the oracle."""
    say("split-k small problem H=%d F=%d" % (H, F))
    w = wl.scaled(wl.CONFIGS[2], T=330, H=H, F=F, E=2, k=1, seed=81)
    inp = wl.make_inputs(w, threads=4)
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    check_layer_full(layer, ref, w.dtype)
    again = run_moe(w, inp)  # the split sums in a fixed order: bit-identical from run to run
    for n in ("y_p", "dx_p", "out", "dx"):
        assert torch.equal(getattr(layer, n), getattr(again, n)), n


@pytest.mark.parametrize("T", [1, 15, 16, 17, 63, 64, 65, 127, 129, 191, 193, 255, 256, 257, 300, 511])
def test_ragged_row_tile_every_row_block_count(T):
    """One expert with T rows: the last row tile holds T mod 256 valid rows, and a wavefront of the grouped
    GEMM has work in ceil((valid 16-row blocks - its position) / 4) of its four row blocks -- every count
    from none to four occurs over these T, in all seven products; full check against the oracle."""
    say("ragged row tile T=%d" % T)
    w = wl.scaled(wl.CONFIGS[2], T=T, H=128, F=320, E=1, k=1, seed=8300 + T)
    inp = wl.make_inputs(w, threads=2)
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    check_layer_full(layer, ref, w.dtype)


@pytest.mark.parametrize("counts", [(100, 300, 700, 1300, 1800, 3400), (3329, 257, 0, 1, 2049, 1537)])
def test_tile_order_mixed_row_tile_counts(counts):
    """Experts with 0, 1, 2, 3, 6, 7, 8, 9 and 14 row tiles in one layer whose products have 8 or 16 column
    tiles: the grouped GEMM walks an expert's tiles in one chunk, in several chunks of about four (or eight) row
    tiles, or in column groups, depending on its row-tile count, deals runs of 32 tiles round robin to the XCDs,
    and every workgroup works out from the run it is in which operand lines it prefetches; a tile left out or
    done twice by any of that shows in the full check against the oracle (top-1 routing with exactly these
    rows per expert, tokens in random order)."""
    say("tile order counts=%s" % (counts,))
    T, E = sum(counts), len(counts)
    w = wl.scaled(wl.CONFIGS[2], T=T, H=2048, F=2048, E=E, k=1, seed=8400 + counts[0])
    inp = wl.make_inputs(w, threads=4)
    rng = np.random.default_rng(w.seed)
    expert_of = rng.permutation(np.repeat(np.arange(E), counts))
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[np.arange(T), expert_of] += 20.0
    inp["logits"] = logits
    layer = run_moe(w, inp)
    assert to_host(layer.seg_offsets).tolist() == np.concatenate([[0], np.cumsum(counts)]).tolist()
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    check_layer_full(layer, ref, w.dtype)


def test_layer_load_in_two_halves():
    """dynmo_layer_load_begin / _end (copy enqueued behind the permutation, read after an event) give the
    counts and the load of the synchronising dynmo_layer_load, also with more work queued behind the copy."""
    say("layer load in two halves")
    w = wl.scaled(wl.CONFIGS[2], T=700, H=128, F=256, E=5, k=2, seed=8600)
    inp = wl.make_inputs(w, threads=2)
    dev = {n: to_device(a) for n, a in inp.items()}
    layer = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, "moe")
    layer.route_topk(dev["logits"])
    layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    layer.load_begin()
    layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])  # queued behind the copy
    counts, load = layer.load_end()
    ref_counts, ref_load = layer.load()
    assert counts == ref_counts and load == ref_load
    assert sum(counts) == w.T * w.k
    f = f32_inputs(inp)
    ref_idx, _ = orc.route_topk(f["logits"], w.k)
    assert counts == np.bincount(ref_idx.ravel(), minlength=w.E).tolist()
    with pytest.raises(ValueError):  # the landing place must be pinned host memory
        B.dynmo_layer_load_begin(layer.d, layer.seg_offsets, torch.empty(w.E + 1, dtype=torch.int32))


def test_layer_under_graph_capture():
    """Forward + backward of a layer captured into a HIP graph (no call on the path
    allocates, synchronises or issues a memset) and replayed three times with eager work
    and synchronisations in between; every replay must reproduce the eager results bit
    for bit, also after the inputs changed in place."""
    say("graph capture")
    w = wl.scaled(wl.CONFIGS[2], T=900, H=256, F=2048, E=4, k=2, seed=95)  # down and dX split their tiles
    inp = wl.make_inputs(w, threads=2)
    dev = {n: to_device(a) for n, a in inp.items()}
    layer = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, "moe")
    layer.alloc_backward()
    names = ("expert_idx", "gate_w", "seg_offsets", "dst_pos", "y_p", "G", "U", "out", "dgate", "dx", "dWg", "dWu", "dWd",
             "droute")

    def run():
        layer.route_topk(dev["logits"])
        layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
        layer.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
        layer.route_bwd()

    def snapshot():
        torch.cuda.synchronize()
        return {n: getattr(layer, n).clone() for n in names}

    B.dynmo_profile_enable(False)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run()  # warm-up outside the capture (function attributes are set on first use)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    x0, l0 = dev["x"].clone(), dev["logits"].clone()
    for trial in range(3):
        if trial == 1:  # new inputs, written in place: the graph reads the same buffers
            dev["x"].copy_(torch.roll(x0, 7, dims=0))
            dev["logits"].copy_(torch.roll(l0, 3, dims=1))
        if trial == 2:
            dev["x"].copy_(x0)
            dev["logits"].copy_(l0)
        run()
        eager = snapshot()
        for n in names:
            if getattr(layer, n).dtype.is_floating_point:
                getattr(layer, n).fill_(-3.0)
            else:
                getattr(layer, n).fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        replayed = snapshot()
        R = int(eager["seg_offsets"][-1])
        for n in names:
            a, b = (eager[n][:R], replayed[n][:R]) if n in ("y_p", "G", "U") else (eager[n], replayed[n])
            assert torch.equal(a, b), "%s differs on replay %d" % (n, trial)


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes(seed):
    """Seeded random shapes (expert counts 1..64, 1..8 slots, sizes on and off the tile
    boundaries, flat to very skewed routing) through the bf16 layer, full check."""
    rng = np.random.default_rng(4000 + seed)
    E = int(rng.choice([1, 2, 3, 5, 8, 16, 33, 64]))
    k = int(rng.integers(1, min(E, 8) + 1))
    T = int(rng.choice([1, 7, 64, 255, 256, 257, 600, 1500]))
    H = int(rng.choice([8, 24, 64, 136, 256, 520, 1024]))
    F = int(rng.choice([8, 40, 128, 264, 688, 1032, 2048]))
    if T * k * (H + F) * E > 4e8:
        T = 256
    w = wl.scaled(wl.CONFIGS[2], T=T, H=H, F=F, E=E, k=k, seed=4100 + seed, zipf_s=float(rng.choice([0.0, 1.1, 2.5])))
    say("random shape %d: T=%d H=%d F=%d E=%d k=%d zipf=%.1f" % (seed, T, H, F, E, k, w.zipf_s))
    inp = wl.make_inputs(w, threads=2)
    layer = run_moe(w, inp)
    f = f32_inputs(inp)
    ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    assert np.array_equal(to_host(layer.expert_idx), ref["expert_idx"])
    check_layer_full(layer, ref, w.dtype)


# --------------------------------------------------------------------------
# one-slot layers with the combine folded into the last product
# --------------------------------------------------------------------------

FOLDED_CASES = [
    ("mod", wl.scaled(wl.CONFIGS[4], T=4 * 256, B=4, S=256, cap=32, H=128, F=256, seed=91)),     # one ragged tile
    ("mod", wl.scaled(wl.CONFIGS[4], T=3 * 400, B=3, S=400, cap=230, H=520, F=328, seed=92)),    # several tiles, tails
    ("mod", wl.scaled(wl.CONFIGS[4], T=2 * 330, B=2, S=330, cap=165, H=512, F=1536, seed=93)),   # last product splits k
    ("mod", wl.scaled(wl.CONFIGS[4], T=2 * 130, B=2, S=130, cap=0, H=64, F=64, seed=94)),        # nothing routed
    ("mod", wl.scaled(wl.CONFIGS[4], T=2 * 100, B=2, S=100, cap=100, H=36, F=50, dtype="f32", seed=95)),  # fp32 kernels
    ("moe", wl.scaled(wl.CONFIGS[2], T=330, H=256, F=4096, E=2, k=1, seed=96)),                  # top-1, no residual, split
    ("moe", wl.scaled(wl.CONFIGS[1], T=300, H=36, F=50, E=4, k=1, seed=97)),                     # top-1 fp32
]


def route_for(layer, mode, w, dev):
    if mode == "moe":
        layer.route_topk(dev["logits"])
    else:
        layer.route_capacity(dev["scores"], w.cap)


@pytest.mark.parametrize("mode,w", FOLDED_CASES,
                         ids=lambda v: v if isinstance(v, str) else "%s-T%d-H%d-F%d" % (v.dtype, v.T, v.H, v.F))
def test_forward_with_folded_combine(mode, w):
    """k = 1: the last product stores res + gate_w * Y straight into the token rows.  Checked
    against the oracle's layer output; rows of tokens without a routed row keep their bits; the
    saved tensors are those of the plain forward pass bit for bit, so the backward pass that
    follows gives identical gradients."""
    say("folded combine %s %s T=%d H=%d F=%d" % (mode, w.dtype, w.T, w.H, w.F))
    inp = wl.make_inputs(w, threads=1)
    dev = {n: to_device(a) for n, a in inp.items()}
    a = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, mode)
    b = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, mode)
    for layer in (a, b):
        route_for(layer, mode, w, dev)
    a.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    a.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    x_b = dev["x"].clone()
    out_b = b.forward_folded(x_b, dev["Wg"], dev["Wu"], dev["Wd"])
    assert (out_b is x_b) == (mode != "moe")
    b.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    torch.cuda.synchronize()
    f = f32_inputs(inp)
    if mode == "moe":
        ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    else:
        ref = orc.mod_layer(f["scores"], w.cap, f["x"], f["Wg"], f["Wu"], f["Wd"], f["dout"])
    assert np.array_equal(to_host(b.expert_idx), ref["expert_idx"])
    e_out = assert_close("out", to_host(out_b), ref["out"], TOL[w.dtype])
    unrouted = torch.as_tensor(ref["expert_idx"][:, 0] < 0, device="cuda")
    if mode != "moe":
        assert torch.equal(x_b[unrouted], dev["x"][unrouted])
    else:
        assert not bool(unrouted.any())
    # one rounding instead of two: never further from the plain result than two output steps
    step = 2.0 ** -7 if w.dtype == "bf16" else 2.0 ** -22
    assert_close("out vs plain", to_host(out_b), to_host(a.out), 2 * step)
    R = int(to_host(a.seg_offsets)[-1])
    for n in ("G", "U", "y_p", "x_p"):
        assert torch.equal(getattr(a, n)[:R], getattr(b, n)[:R]), n
    for n in ("dx", "dWg", "dWu", "dWd", "dgate"):
        assert torch.equal(getattr(a, n), getattr(b, n)), n
    say("  out err %.1e" % e_out)

    # the same call reading its rows through src_slot, without the unweighted rows, in place
    x_c = dev["x"].clone()
    res = x_c if mode != "moe" else None
    out_c = x_c if mode != "moe" else torch.zeros_like(a.out)
    G = torch.empty_like(b.G)
    U = torch.empty_like(b.U)
    B.dynmo_grouped_ffn_fwd_combine(b.d, None, x_c, b.src_slot, b.seg_offsets, dev["Wg"], dev["Wu"], dev["Wd"],
                                    b.gate_w, res, out_c, None, G, U, b.ws_fwd)
    torch.cuda.synchronize()
    assert torch.equal(out_c, out_b)
    assert torch.equal(G[:R], b.G[:R]) and torch.equal(U[:R], b.U[:R])


@pytest.mark.parametrize("mode,w", FOLDED_CASES,
                         ids=lambda v: v if isinstance(v, str) else "%s-T%d-H%d-F%d" % (v.dtype, v.T, v.H, v.F))
def test_backward_with_folded_scatter(mode, w):
    """k = 1: the dX product stores dbase + dX straight into the token rows (the scatter back to
    token order folded into its stores).  Checked against the oracle's dx; the gradient rows of
    tokens without a routed row keep their bits; the weight gradients and the gate gradient are
    those of the plain backward pass bit for bit."""
    say("folded scatter %s %s T=%d H=%d F=%d" % (mode, w.dtype, w.T, w.H, w.F))
    inp = wl.make_inputs(w, threads=1)
    dev = {n: to_device(a) for n, a in inp.items()}
    a = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, mode)
    b = RoutedFFNLayer(w.T, w.H, w.F, w.E, w.k, w.dtype, mode)
    for layer in (a, b):
        route_for(layer, mode, w, dev)
        layer.forward(dev["x"], dev["Wg"], dev["Wu"], dev["Wd"])
    dx_a = a.backward(dev["dout"], dev["Wg"], dev["Wu"], dev["Wd"])
    g_b = dev["dout"].clone()
    dx_b = b.backward_folded(g_b, dev["Wg"], dev["Wu"], dev["Wd"])
    assert (dx_b is g_b) == (mode != "moe")
    torch.cuda.synchronize()
    f = f32_inputs(inp)
    if mode == "moe":
        ref = orc.moe_layer(f["logits"], f["x"], f["Wg"], f["Wu"], f["Wd"], w.k, f["dout"])
    else:
        ref = orc.mod_layer(f["scores"], w.cap, f["x"], f["Wg"], f["Wu"], f["Wd"], f["dout"])
    e_dx = assert_close("dx", to_host(dx_b), ref["dx"], TOL[w.dtype])
    unrouted = torch.as_tensor(ref["expert_idx"][:, 0] < 0, device="cuda")
    if mode != "moe":
        assert torch.equal(dx_b[unrouted], dev["dout"][unrouted])
    else:
        assert not bool(unrouted.any())
    # one rounding instead of two: never further from the plain result than two output steps
    step = 2.0 ** -7 if w.dtype == "bf16" else 2.0 ** -22
    assert_close("dx vs plain", to_host(dx_b), to_host(dx_a), 2 * step)
    for n in ("dWg", "dWu", "dWd", "dgate"):
        assert torch.equal(getattr(a, n), getattr(b, n)), n
    R = int(to_host(a.seg_offsets)[-1])
    assert torch.equal(a.dy_p[:R], b.dy_p[:R])
    say("  dx err %.1e" % e_dx)

    # a separate dx with dbase given, and the rows in expert order asked for as well
    dx_c = torch.full_like(dev["dout"], 3.0)
    dx_p = torch.empty_like(b.dx_p)
    B.dynmo_grouped_ffn_bwd_scatter(b.d, b.dy_p, b.x_p, b.G, b.U, b.seg_offsets, b.src_slot, dev["Wg"], dev["Wu"],
                                    dev["Wd"], dev["dout"] if mode != "moe" else None, dx_c, dx_p, b.dWg, b.dWu, b.dWd,
                                    b.ws_bwd)
    torch.cuda.synchronize()
    routed = ~unrouted
    assert torch.equal(dx_c[routed], dx_b[routed])
    assert bool((dx_c[unrouted] == 3.0).all())
    assert torch.equal(dx_p[:R], a.dx_p[:R])
    d2 = B.make_desc(w.T, w.H, w.F, max(2, w.E), 2, w.dtype)
    with pytest.raises(B.DynmoError):
        B.dynmo_grouped_ffn_bwd_scatter(d2, b.dy_p, b.x_p, b.G, b.U, b.seg_offsets, b.src_slot, dev["Wg"], dev["Wu"],
                                        dev["Wd"], None, dx_c, None, b.dWg, b.dWu, b.dWd, b.ws_bwd)


def test_folded_combine_early_exit_stack_in_place():
    """Sec. 2.5's shrinking stack with the residual stream updated in place, layer after layer."""
    say("folded combine, early-exit stack in place")
    w = wl.scaled(wl.CONFIGS[5], T=1500, H=128, F=192, seed=98)
    inp = wl.make_inputs(w, threads=1)
    dev = {n: to_device(a) for n, a in inp.items()}
    layers = [RoutedFFNLayer(w.T, w.H, w.F, 1, 1, "bf16", "early_exit") for _ in range(w.layers)]
    x = dev["x"].clone()
    for l, layer in enumerate(layers):
        layer.route_active(dev["exit_layer"], l + 1)
        assert layer.forward_folded(x, dev["Wg"][l], dev["Wu"][l], dev["Wd"][l]) is x
    g = dev["dout"].clone()
    for l in range(w.layers - 1, -1, -1):
        assert layers[l].backward_folded(g, dev["Wg"][l], dev["Wu"][l], dev["Wd"][l]) is g
    torch.cuda.synchronize()
    plain_layers, plain_out, plain_dx = run_stack(w, inp)
    f = f32_inputs(inp)
    weights = [(f["Wg"][l], f["Wu"][l], f["Wd"][l]) for l in range(w.layers)]
    ref = orc.early_exit_stack(inp["exit_layer"], f["x"], weights, f["dout"])
    assert_close("out", to_host(x), ref["out"], TOL["bf16"])
    assert_close("dx", to_host(g), ref["dx"], TOL["bf16"])
    # the in-place stream rounds once per layer where the plain one rounds twice
    assert_close("out vs plain", to_host(x), to_host(plain_out), 4 * 2.0 ** -7)
    assert_close("dx vs plain", to_host(g), to_host(plain_dx), 4 * 2.0 ** -7)
    assert [l.load()[0] for l in layers] == [l.load()[0] for l in plain_layers]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_zero_tokens(dtype):
    """T = 0: every call on the path returns without touching its (dummy) buffers; the segment
    offsets come back as zeros, the weight gradients as zeros, the load as zero."""
    say("zero tokens %s" % dtype)
    H, F, E, k = 64, 96, 4, 2
    d = B.make_desc(0, H, F, E, k, dtype)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dummy = lambda: torch.full((64,), 7, dtype=td, device="cuda")
    dummy_f = lambda: torch.full((64,), 7.0, dtype=torch.float32, device="cuda")
    dummy_i = lambda: torch.full((64,), 7, dtype=torch.int32, device="cuda")
    ei, gw, seg, src, dst = dummy_i(), dummy_f(), dummy_i(), dummy_i(), dummy_i()
    x, x_p, y_p, G, U, out = dummy(), dummy(), dummy(), dummy(), dummy(), dummy()
    W = [(torch.randn(E, F, H, device="cuda") * 0.02).to(td), (torch.randn(E, F, H, device="cuda") * 0.02).to(td),
         (torch.randn(E, H, F, device="cuda") * 0.02).to(td)]
    ws_p = torch.empty((max(64, B.dynmo_permute_workspace_bytes(d)),), dtype=torch.uint8, device="cuda")
    ws_f = torch.empty((B.dynmo_grouped_ffn_fwd_workspace_bytes(d),), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty((B.dynmo_grouped_ffn_bwd_workspace_bytes(d),), dtype=torch.uint8, device="cuda")
    B.dynmo_route_topk(d, dummy_f(), ei, gw)
    B.dynmo_permute(d, x, ei, x_p, seg, src, dst, ws_p)
    B.dynmo_grouped_ffn_fwd(d, x_p, seg, W[0], W[1], W[2], y_p, G, U, ws_f)
    B.dynmo_combine(d, y_p, dst, gw, None, out)
    dy_p, dgate, dx_p, dx, dl = dummy(), dummy_f(), dummy(), dummy(), dummy_f()
    dW = [torch.full_like(w, 7) for w in W]
    B.dynmo_combine_bwd(d, out, y_p, dst, gw, dy_p, dgate)
    B.dynmo_grouped_ffn_bwd(d, dy_p, x_p, G, U, seg, W[0], W[1], W[2], dx_p, dW[0], dW[1], dW[2], ws_b)
    B.dynmo_permute_bwd(d, dx_p, dst, None, dx)
    B.dynmo_route_topk_bwd(d, dgate, gw, ei, dl)
    counts, load = B.dynmo_layer_load(d, seg, 1.0)
    torch.cuda.synchronize()
    assert counts == [0] * E and load == 0.0
    assert to_host(seg)[:E + 1].tolist() == [0] * (E + 1)
    for t in (ei, src, dst, x_p, y_p, G, U, out, dy_p, dx_p, dx):
        assert bool((t == 7).all())
    for g in dW:
        assert not bool(g.any())
