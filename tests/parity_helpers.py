"""Shared helpers for the GPU parity tests: error metrics, tolerances, the full
element-by-element comparison and the sampled one (kept for the two configurations whose
full oracle run does not fit the test budget)."""
import numpy as np

from oracle import dynmo_oracle as orc
from paper_2505_14864_amd import workloads as wl
from paper_2505_14864_amd.layer import to_host

# Norm-wise tolerance per tensor: max|gpu - oracle| / max|oracle|.
# bf16: inputs, saved activations and outputs are rounded to 8 significant bits
# (relative step 2^-8 = 3.9e-3); a few roundings in sequence stay below 2e-2.
# fp32: dot products of length <= a few hundred in fp32 against fp64: ~1e-6.
TOL = {"bf16": 2e-2, "f32": 1e-4}
# Element-wise secondary measure |g - o| / (|o| + rms(o)).  The norm-wise measure divides by
# max|o|, which is 4 to 5 rms(o) for these tensors; this one divides by about rms(o) at
# elements near zero and is that much stricter there.  An element of a bf16 result is a sum
# of terms that each carry about five independent roundings of relative size <= 2^-9
# (standard deviation 2^-9 / sqrt(3) = 1.1e-3 each; the SwiGLU derivative amplifies those of
# G by up to 2), so its error has a standard deviation of about 5e-3 rms(o); the largest of
# up to 5e8 elements lies about 6.3 standard deviations out, 3.2e-2.  Bound: twice the
# norm-wise tolerance.
ELEMENT_TOL = {"bf16": 4e-2, "f32": 2e-4}


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    scale = np.abs(ref).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / scale)


def assert_close(name, got, ref, tol):
    e = rel_err(got, ref)
    assert e <= tol, "%s: max rel err %.3e > %.1e" % (name, e, tol)
    return e


def group_rel_err(got, ref, bounds):
    """Largest norm-wise error over groups of leading indices [bounds[g], bounds[g+1]): each
    group is scaled by its own largest reference magnitude, so an error confined to a small
    expert (or to the rows of one segment) is not hidden under the largest group's scale.
    A group whose reference is all zero must be reproduced exactly."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    worst = 0.0
    for g in range(len(bounds) - 1):
        a, b = int(bounds[g]), int(bounds[g + 1])
        if b <= a:
            continue
        scale = np.abs(ref[a:b]).max()
        diff = np.abs(got[a:b] - ref[a:b]).max()
        worst = max(worst, float(diff) if scale == 0.0 else float(diff / scale))
    return worst


def elementwise_excess(got, ref):
    """The secondary, element-wise measure: max over elements of |g - o| / (|o| + rms(o))."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.abs(got).max())
    return float((np.abs(got - ref) / (np.abs(ref) + rms)).max())


def sel(t, idx, dim=0):
    """Rows / columns of a GPU tensor, selected on the device, as numpy."""
    import torch
    i = torch.as_tensor(np.asarray(idx, dtype=np.int64), device=t.device)
    return to_host(t.index_select(dim, i))


def f32_inputs(inp):
    return {n: wl.as_f32(a) for n, a in inp.items()}


def sub_segments(rows, seg):
    """Segment offsets of a sorted subset of permuted rows."""
    rows = np.asarray(rows)
    return np.asarray([int(np.searchsorted(rows, s, side="left")) for s in seg], dtype=np.int32)


def pick_rows(seg, rng, extra):
    """Rows at both ends of every segment plus `extra` random ones (sorted, unique)."""
    R = int(seg[-1])
    rows = set()
    for e in range(len(seg) - 1):
        a, b = int(seg[e]), int(seg[e + 1])
        if b > a:
            rows.update((a, b - 1))
    if R > 0:
        rows.update(int(v) for v in rng.integers(0, R, size=extra))
    return np.asarray(sorted(rows), dtype=np.int64)


def pick_cols(n, tile, rng, extra):
    """First, last, tile-edge and a few random column indices."""
    cols = {0, n - 1, min(n - 1, tile - 1), min(n - 1, tile), (n - 1) // tile * tile}
    cols.update(int(v) for v in rng.integers(0, n, size=extra))
    return np.asarray(sorted(cols), dtype=np.int64)


def check_layer_sampled(layer, f, expert_idx_ref, gate_ref, residual, dtype, rng, n_tokens=24, n_cols=6):
    """Compares one layer's GPU results (already computed, forward and backward)
    with the oracle on sampled rows / tokens / weight columns.

    f: dict of fp32 host inputs (x, dout, Wg, Wu, Wd with leading E).
    Integer results are compared in full; y_p, G, U, dx_p on sampled rows; out,
    dx, dgate on sampled tokens; dWg/dWu rows and dWd columns on a sampled subset
    of the F dimension (exact, because the FFN separates over F for those).
    """
    tol = TOL[dtype]
    T, k = expert_idx_ref.shape
    E = f["Wg"].shape[0]
    x, dout, Wg, Wu, Wd = f["x"], f["dout"], f["Wg"], f["Wu"], f["Wd"]
    x_p_ref, seg, src_slot, dst_pos = orc.permute(x, expert_idx_ref, E)
    R = int(seg[-1])
    assert np.array_equal(to_host(layer.seg_offsets), seg)
    assert np.array_equal(to_host(layer.dst_pos), dst_pos)
    assert np.array_equal(to_host(layer.src_slot)[:R], src_slot)
    assert np.array_equal(to_host(layer.x_p)[:R], x_p_ref)  # rows are copied bits

    # sampled tokens -> their rows, plus segment-edge rows
    toks = np.unique(np.concatenate([rng.integers(0, T, size=n_tokens), [0, T - 1]]))
    tok_rows = dst_pos[toks].reshape(-1)
    rows = np.unique(np.concatenate([tok_rows[tok_rows >= 0], pick_rows(seg, rng, 8)])).astype(np.int64)
    sseg = sub_segments(rows, seg)
    y_s, G_s, U_s = orc.grouped_ffn_fwd(x_p_ref[rows], sseg, Wg, Wu, Wd)
    assert_close("y_p", sel(layer.y_p, rows), y_s, tol)
    assert_close("G", sel(layer.G, rows), G_s, tol)
    assert_close("U", sel(layer.U, rows), U_s, tol)

    # out / dgate on the sampled tokens: remap their slots into the row subset
    pos_in_sub = {int(r): i for i, r in enumerate(rows)}
    dp_sub = np.asarray([[pos_in_sub[int(p)] if p >= 0 else -1 for p in dst_pos[t]] for t in toks], dtype=np.int32)
    base = x[toks] if residual else None
    out_s = orc.combine(y_s, dp_sub, gate_ref[toks], base, len(toks))
    assert_close("out", sel(layer.out, toks), out_s, tol)

    # backward on the row subset: dy rows come from the owning token's dout
    owner = src_slot[rows] // k
    slot = src_slot[rows] % k
    dy_s = gate_ref[owner, slot][:, None] * dout[owner].astype(np.float64)
    assert_close("dy_p", sel(layer.dy_p, rows), dy_s, tol)
    dgate_s = np.einsum("rh,rh->r", dout[owner].astype(np.float64), y_s)
    got_dgate = to_host(layer.dgate)[owner, slot]
    assert_close("dgate", got_dgate, dgate_s, tol)
    dx_s, _, _, _ = orc.grouped_ffn_bwd(dy_s, x_p_ref[rows], G_s, U_s, sseg, Wg, Wu, Wd)
    assert_close("dx_p", sel(layer.dx_p, rows), dx_s, tol)
    dx_t = orc.permute_bwd(dx_s, dp_sub, dout[toks] if residual else None)
    assert_close("dx", sel(layer.dx, toks), dx_t, tol)

    # weight gradients on a subset of the F dimension, all rows
    cols = pick_cols(Wg.shape[1], 128, rng, n_cols)
    Wg_c, Wu_c, Wd_c = Wg[:, cols, :], Wu[:, cols, :], Wd[:, :, cols]
    own_all = src_slot // k
    dy_all = gate_ref[own_all, src_slot % k][:, None] * dout[own_all].astype(np.float64)
    _, G_c, U_c = orc.grouped_ffn_fwd(x_p_ref, seg, Wg_c, Wu_c, Wd_c)
    _, dWg_c, dWu_c, dWd_c = orc.grouped_ffn_bwd(dy_all, x_p_ref, G_c, U_c, seg, Wg_c, Wu_c, Wd_c)
    assert_close("dWg", sel(layer.dWg, cols, 1), dWg_c, tol)
    assert_close("dWu", sel(layer.dWu, cols, 1), dWu_c, tol)
    assert_close("dWd", sel(layer.dWd, cols, 2), dWd_c, tol)
    for e in range(E):
        if seg[e + 1] == seg[e]:  # an expert with no rows gets exactly zero
            assert not to_host(layer.dWg[e]).any() and not to_host(layer.dWd[e]).any()
    return dict(seg=seg, dst_pos=dst_pos, rows=rows, toks=toks)


def check_layer_full(layer, ref, dtype, names=("y_p", "G", "U", "out", "dy_p", "dgate", "dx_p", "dx", "dWg", "dWu", "dWd"),
                     assert_elementwise=False):
    """Element-by-element comparison of every tensor with a full oracle run.

    Three measures per tensor, all against the same tolerance: the norm-wise error over the
    whole tensor; the same error with every expert's weight gradient and every expert's row
    segment scaled on its own; and the element-wise |g - o| / (|o| + rms(o)), which is always
    reported and, with assert_elementwise, held to ELEMENT_TOL (the benchmark configurations,
    whose sums are long enough for that bound's derivation; an expert with a few dozen rows
    has weight-gradient elements that are sums of a few dozen terms, with a heavier tail)."""
    tol = TOL[dtype]
    seg = ref["seg_offsets"]
    R = int(seg[-1])
    assert np.array_equal(to_host(layer.seg_offsets), seg)
    assert np.array_equal(to_host(layer.dst_pos), ref["dst_pos"])
    assert np.array_equal(to_host(layer.src_slot)[:R], ref["src_slot"])
    assert np.array_equal(to_host(layer.x_p)[:R], np.asarray(ref["x_p"], dtype=np.float32))
    errs = {}
    for n in names:
        got = to_host(getattr(layer, n))
        if n in ("y_p", "G", "U", "dy_p", "dx_p"):
            got = got[:R]
        errs[n] = assert_close(n, got, ref[n], tol)
        if n in ("dWg", "dWu", "dWd"):
            g = group_rel_err(got, ref[n], range(got.shape[0] + 1))
            assert g <= tol, "%s: per-expert rel err %.3e > %.1e" % (n, g, tol)
            errs[n + "/expert"] = g
        elif n in ("y_p", "G", "U", "dy_p", "dx_p"):
            g = group_rel_err(got, ref[n], seg)
            assert g <= tol, "%s: per-segment rel err %.3e > %.1e" % (n, g, tol)
            errs[n + "/segment"] = g
        x = elementwise_excess(got, ref[n])
        if assert_elementwise:
            assert x <= ELEMENT_TOL[dtype], "%s: element-wise |g-o| / (|o| + rms) = %.3e > %.1e" % (n, x, ELEMENT_TOL[dtype])
        errs[n + "/element"] = x
    return errs
