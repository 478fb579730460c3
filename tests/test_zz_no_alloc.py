"""dynmo_permute_static (the permutation for callers that cannot allocate) against
dynmo_permute, through the C ABI: two calls in a row on the same GPU, the second with a
smaller input, each compared bit for bit with the workspace-taking entry point (whose own
parity with the oracle test_gpu_parity.py covers) and with the oracle."""
import numpy as np
import pytest
import torch

from oracle import dynmo_oracle as orc
from paper_2505_14864_amd import binding as B
from paper_2505_14864_amd.layer import to_device, to_host

pytestmark = pytest.mark.gpu


def _run_both(T, H, E, k, seed):
    print("permute_static T=%d H=%d E=%d k=%d" % (T, H, E, k), flush=True)
    rng = np.random.default_rng(seed)
    ei = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32) if T else np.zeros((0, k), np.int32)
    if T:
        ei[rng.random((T, k)) < 0.1] = -1  # some unrouted slots
    x = rng.standard_normal((T, H)).astype(np.float32)
    d = B.make_desc(T, H, 8, E, k, "f32")
    dev = "cuda"
    xd, eid = to_device(x), to_device(ei)
    out = {}
    for name in ("ws", "static"):
        x_p = torch.full((max(T * k, 1), H), 7.0, dtype=torch.float32, device=dev)
        seg = torch.full((E + 1,), -5, dtype=torch.int32, device=dev)
        src = torch.full((max(T * k, 1),), -5, dtype=torch.int32, device=dev)
        dst = torch.full((max(T, 1), k), -5, dtype=torch.int32, device=dev)
        # an empty torch tensor has a null data pointer: with no tokens only the indices are asked for
        rows_in, rows_out = (xd, x_p) if T else (None, None)
        if name == "ws":
            ws = torch.empty(B.dynmo_permute_workspace_bytes(d), dtype=torch.uint8, device=dev)
            B.dynmo_permute(d, rows_in, eid if T else seg, rows_out, seg, src, dst, ws)
        else:
            B.dynmo_permute_static(d, rows_in, eid if T else seg, rows_out, seg, src, dst)
        torch.cuda.synchronize()
        out[name] = (to_host(seg), to_host(src), to_host(dst), to_host(x_p))
    ref_x_p, ref_seg, ref_src, ref_dst = orc.permute(x, ei, E)
    R = int(ref_seg[-1])
    for name in ("ws", "static"):
        seg, src, dst, x_p = out[name]
        assert np.array_equal(seg, ref_seg), name
        assert np.array_equal(src[:R], ref_src[:R]), name
        assert np.array_equal(dst[:T], ref_dst), name
        assert np.array_equal(x_p[:R], ref_x_p[:R]), name
        assert np.all(x_p[R:] == 7.0), name  # nothing written past R
    for a, b in zip(out["ws"], out["static"]):
        assert np.array_equal(a, b)


def test_permute_static_two_calls_second_smaller():
    # the second call reuses the scratch the first one left behind, with fewer chunks and experts
    _run_both(T=5000, H=64, E=16, k=4, seed=1)
    _run_both(T=700, H=32, E=5, k=2, seed=2)
    _run_both(T=0, H=32, E=3, k=1, seed=3)
    _run_both(T=1, H=16, E=1, k=1, seed=4)


def test_permute_static_limit():
    E = 64
    max_slots = B.dynmo_permute_static_max_slots(E)
    assert max_slots == (1 << 18) // E * 1024
    assert B.dynmo_permute_static_max_slots(0) == 0 and B.dynmo_permute_static_max_slots(65) == 0
    # one chunk beyond the limit is refused before anything is launched (no buffer is touched)
    T = max_slots + 1
    d = B.make_desc(T, 8, 8, E, 1, "bf16")
    dummy = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(B.DynmoError) as ei:
        B.dynmo_permute_static(d, None, dummy, None, dummy, dummy, dummy)
    assert ei.value.status == -3
