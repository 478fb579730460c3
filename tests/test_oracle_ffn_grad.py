"""Pins for the oracle's FFN values and gradients (CPU only).

The reference here is never the oracle's own route: it is the dense masked
equivalent (every expert applied to every token, no permutation), evaluated
and differentiated by torch in float64 (library matmul, library silu,
autograd), plus central finite differences and closed special cases.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as Fnn

from oracle import dynmo_oracle as orc

torch.set_default_dtype(torch.float64)


def rand_problem(T, H, F, E, seed, scale=0.3):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, H)).astype(np.float32)
    Wg = (rng.standard_normal((E, F, H)) * scale).astype(np.float32)
    Wu = (rng.standard_normal((E, F, H)) * scale).astype(np.float32)
    Wd = (rng.standard_normal((E, H, F)) * scale).astype(np.float32)
    dout = rng.standard_normal((T, H)).astype(np.float32)
    return rng, x, Wg, Wu, Wd, dout


def dense_masked_moe(logits, x, Wg, Wu, Wd, k):
    """out[t] = sum_e m[t,e] * FFN_e(x[t]); m = softmax over the top-k logits,
    built with torch.topk + scatter.  (Logits used here have no ties.)"""
    E = Wg.shape[0]
    vals, idx = torch.topk(logits, k, dim=1)
    w = torch.softmax(vals, dim=1)
    m = torch.zeros_like(logits).scatter(1, idx, w)
    out = torch.zeros_like(x)
    for e in range(E):
        h = Fnn.silu(x @ Wg[e].T) * (x @ Wu[e].T)
        out = out + m[:, e:e + 1] * (h @ Wd[e].T)
    return out


@pytest.mark.parametrize("T,H,F,E,k,seed", [(24, 8, 12, 4, 2, 0), (17, 6, 10, 5, 3, 1), (12, 4, 6, 3, 1, 2), (9, 5, 7, 3, 3, 3)])
def test_moe_layer_equals_dense_masked_and_autograd(T, H, F, E, k, seed):
    rng, x, Wg, Wu, Wd, dout = rand_problem(T, H, F, E, seed)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    res = orc.moe_layer(logits, x, Wg, Wu, Wd, k, dout)

    tl, tx, tg, tu, td = (torch.tensor(a.astype(np.float64), requires_grad=True) for a in (logits, x, Wg, Wu, Wd))
    out = dense_masked_moe(tl, tx, tg, tu, td, k)
    (out * torch.tensor(dout.astype(np.float64))).sum().backward()

    def close(a, b):
        np.testing.assert_allclose(a, b.detach().numpy(), rtol=1e-10, atol=1e-12)

    close(res["out"], out)
    close(res["dx"], tx.grad)
    close(res["dWg"], tg.grad)
    close(res["dWu"], tu.grad)
    close(res["dWd"], td.grad)
    close(res["dlogits"], tl.grad)


def test_moe_gradients_by_finite_differences():
    T, H, F, E, k = 8, 4, 6, 3, 2
    rng, x, Wg, Wu, Wd, dout = rand_problem(T, H, F, E, 7)
    # well-separated logits: the selection cannot flip under the FD step
    logits = (rng.permuted(np.tile(np.arange(E, dtype=np.float64), (T, 1)), axis=1) * 1.5
              + rng.uniform(-0.2, 0.2, (T, E)))
    args = dict(logits=logits.astype(np.float64), x=x.astype(np.float64), Wg=Wg.astype(np.float64),
                Wu=Wu.astype(np.float64), Wd=Wd.astype(np.float64))

    def loss(a):
        r = orc.moe_layer(a["logits"], a["x"], a["Wg"], a["Wu"], a["Wd"], k, dout)
        return float((r["out"] * dout).sum())

    res = orc.moe_layer(args["logits"], args["x"], args["Wg"], args["Wu"], args["Wd"], k, dout)
    grads = dict(logits=res["dlogits"], x=res["dx"], Wg=res["dWg"], Wu=res["dWu"], Wd=res["dWd"])
    eps = 1e-6
    for name, g in grads.items():
        flat_idx = rng.choice(args[name].size, size=min(20, args[name].size), replace=False)
        for fi in flat_idx:
            pos = np.unravel_index(fi, args[name].shape)
            keep = args[name][pos]
            args[name][pos] = keep + eps
            lp = loss(args)
            args[name][pos] = keep - eps
            lm = loss(args)
            args[name][pos] = keep
            fd = (lp - lm) / (2 * eps)
            assert g[pos] == pytest.approx(fd, rel=2e-6, abs=2e-8), (name, pos)


def test_single_expert_is_a_dense_swiglu_mlp():
    T, H, F = 19, 8, 11
    rng, x, Wg, Wu, Wd, dout = rand_problem(T, H, F, 1, 11)
    logits = rng.standard_normal((T, 1)).astype(np.float32)
    res = orc.moe_layer(logits, x, Wg, Wu, Wd, 1, dout)
    tx = torch.tensor(x.astype(np.float64))
    ref = (Fnn.silu(tx @ torch.tensor(Wg[0].astype(np.float64)).T) * (tx @ torch.tensor(Wu[0].astype(np.float64)).T)) \
        @ torch.tensor(Wd[0].astype(np.float64)).T
    np.testing.assert_allclose(res["out"], ref.numpy(), rtol=1e-11, atol=1e-13)
    assert np.all(res["gate_w"] == 1.0)
    assert np.all(res["dlogits"] == 0.0)  # softmax over one logit is constant


def test_zero_down_projection_gives_base():
    T, H, F, E = 10, 4, 6, 2
    rng, x, Wg, Wu, Wd, dout = rand_problem(T, H, F, E, 13)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    res = orc.moe_layer(logits, x, Wg, Wu, np.zeros_like(Wd), 2, dout)
    assert np.all(res["out"] == 0.0)
    scores = rng.standard_normal((2, 5)).astype(np.float32)
    res = orc.mod_layer(scores, 2, x, Wg[:1], Wu[:1], np.zeros_like(Wd[:1]), dout)
    np.testing.assert_array_equal(res["out"], x.astype(np.float64))


def test_empty_expert_gets_zero_weight_gradients():
    T, H, F, E = 12, 4, 6, 4
    rng, x, Wg, Wu, Wd, dout = rand_problem(T, H, F, E, 17)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[:, 2] = -50.0  # expert 2 is never in the top-2
    res = orc.moe_layer(logits, x, Wg, Wu, Wd, 2, dout)
    assert res["seg_offsets"][3] == res["seg_offsets"][2]
    for name in ("dWg", "dWu", "dWd"):
        assert np.all(res[name][2] == 0.0)
        assert np.any(res[name][0] != 0.0)


def test_mod_layer_against_autograd():
    B, S, H, F, cap = 3, 10, 6, 8, 4
    T = B * S
    rng, x, Wg, Wu, Wd, dout = rand_problem(T, H, F, 1, 19)
    scores = rng.standard_normal((B, S)).astype(np.float32)
    res = orc.mod_layer(scores, cap, x, Wg, Wu, Wd, dout)
    ts, tx, tg, tu, td = (torch.tensor(a.astype(np.float64), requires_grad=True) for a in (scores, x, Wg, Wu, Wd))
    # mask from torch.topk (scores drawn without ties)
    _, top = torch.topk(ts, cap, dim=1)
    mask = torch.zeros(B, S).scatter(1, top, 1.0).reshape(T, 1)
    ffn = (Fnn.silu(tx @ tg[0].T) * (tx @ tu[0].T)) @ td[0].T
    out = tx + mask * torch.sigmoid(ts).reshape(T, 1) * ffn
    (out * torch.tensor(dout.astype(np.float64))).sum().backward()
    for a, b in ((res["out"], out), (res["dx"], tx.grad), (res["dWg"], tg.grad), (res["dWu"], tu.grad),
                 (res["dWd"], td.grad), (res["dscores"].reshape(B, S), ts.grad)):
        np.testing.assert_allclose(a, b.detach().numpy(), rtol=1e-10, atol=1e-12)
    assert int(res["seg_offsets"][1]) == B * cap
    # cap = S with very large scores: every token gets x + FFN(x)
    big = np.full((B, S), 40.0, np.float32)
    res = orc.mod_layer(big, S, x, Wg, Wu, Wd, dout)
    np.testing.assert_allclose(res["out"], (tx + ffn).detach().numpy(), rtol=1e-12, atol=1e-13)


def _dense_stack(tx, ws, active_masks):
    h = tx
    for (g, u, d), m in zip(ws, active_masks):
        h = h + m * ((Fnn.silu(h @ g[0].T) * (h @ u[0].T)) @ d[0].T)
    return h


def test_early_exit_stack_against_autograd_and_limits():
    T, H, F, L = 30, 6, 8, 4
    rng = np.random.default_rng(23)
    x = rng.standard_normal((T, H)).astype(np.float32)
    dout = rng.standard_normal((T, H)).astype(np.float32)
    ws = [tuple((rng.standard_normal(s) * 0.3).astype(np.float32) for s in ((1, F, H), (1, F, H), (1, H, F)))
          for _ in range(L)]
    ex = rng.geometric(0.3, size=T).astype(np.int32)
    res = orc.early_exit_stack(ex, x, ws, dout)
    tx = torch.tensor(x.astype(np.float64), requires_grad=True)
    tws = [tuple(torch.tensor(w.astype(np.float64), requires_grad=True) for w in trip) for trip in ws]
    masks = [torch.tensor((ex >= l).astype(np.float64)).reshape(T, 1) for l in range(1, L + 1)]
    out = _dense_stack(tx, tws, masks)
    (out * torch.tensor(dout.astype(np.float64))).sum().backward()
    np.testing.assert_allclose(res["out"], out.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(res["dx"], tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    for l in range(L):
        for name, t in zip(("dWg", "dWu", "dWd"), tws[l]):
            np.testing.assert_allclose(res["bwd"][l][name], t.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert list(res["active"]) == [int((ex >= l).sum()) for l in range(1, L + 1)]
    assert all(res["active"][l] >= res["active"][l + 1] for l in range(L - 1))
    # nobody exits -> plain dense residual MLP stack (all masks one)
    res = orc.early_exit_stack(np.full(T, 99, np.int32), x, ws, dout)
    ref = _dense_stack(torch.tensor(x.astype(np.float64)), [tuple(torch.tensor(w.astype(np.float64)) for w in t) for t in ws],
                       [1.0] * L)
    np.testing.assert_allclose(res["out"], ref.numpy(), rtol=1e-10, atol=1e-12)
    # everybody exits at layer 1 -> layers 2..L are the identity with zero dW
    res = orc.early_exit_stack(np.ones(T, np.int32), x, ws, dout)
    np.testing.assert_array_equal(res["out"], res["fwd"][0]["out"])
    for l in range(1, L):
        assert all(np.all(res["bwd"][l][n] == 0.0) for n in ("dWg", "dWu", "dWd"))
        np.testing.assert_array_equal(res["bwd"][l]["dx"], dout.astype(np.float64))


def _pin_moe(seed=29):
    T, H, F, E, k = 10, 4, 6, 3, 2
    test_moe_layer_equals_dense_masked_and_autograd(T, H, F, E, k, seed)


def test_planted_mistakes_are_caught(monkeypatch):
    """Mutate the oracle one slip at a time (on the CPU) and require the
    autograd pin to fail for each mutant, then pass again unmutated."""
    real = {n: getattr(orc, n) for n in ("_sigmoid", "combine", "permute_bwd", "route_topk_bwd", "grouped_ffn_bwd",
                                          "combine_bwd", "grouped_ffn_fwd")}

    def drop_second_slot(y_p, dst_pos, gate_w, base, T):
        dp = np.array(dst_pos)
        dp[:, 1:] = -1
        return real["combine"](y_p, dp, gate_w, base, T)

    def no_slot_sum(dx_p, dst_pos, dbase):
        dp = np.array(dst_pos)
        dp[:, :1] = -1
        return real["permute_bwd"](dx_p, dp, dbase)

    def sign_flip(dgate, gate_w, expert_idx, E):
        return -real["route_topk_bwd"](dgate, gate_w, expert_idx, E)

    def swapped_gate_up(dy_p, x_p, G, U, seg, Wg, Wu, Wd):
        dx, dWg, dWu, dWd = real["grouped_ffn_bwd"](dy_p, x_p, G, U, seg, Wg, Wu, Wd)
        return dx, dWu, dWg, dWd

    def unweighted_dy(dout, y_p, dst_pos, gate_w):
        return real["combine_bwd"](dout, y_p, dst_pos, np.ones_like(gate_w))

    def transposed_down(x_p, seg, Wg, Wu, Wd):
        y, G, U = real["grouped_ffn_fwd"](x_p, seg, Wg, Wu, Wd)
        return y[:, ::-1].copy(), G, U

    mutants = {
        "_sigmoid": lambda z: 1.0 / (1.0 + np.exp(z)),
        "combine": drop_second_slot,
        "permute_bwd": no_slot_sum,
        "route_topk_bwd": sign_flip,
        "grouped_ffn_bwd": swapped_gate_up,
        "combine_bwd": unweighted_dy,
        "grouped_ffn_fwd": transposed_down,
    }
    for name, mutant in mutants.items():
        monkeypatch.setattr(orc, name, mutant)
        with pytest.raises(AssertionError):
            _pin_moe()
        monkeypatch.setattr(orc, name, real[name])
    _pin_moe()
