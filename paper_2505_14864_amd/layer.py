"""Call sequences of the routed FFN layer over the C-ABI binding.

Holds the device buffers of one layer and issues the library calls in order:
  forward : route -> permute -> grouped_ffn_fwd -> combine
            (or permute indices only -> grouped_ffn_fwd_gather -> combine,
             or, for k = 1, permute -> grouped_ffn_fwd_combine)
  backward: combine_bwd -> grouped_ffn_bwd -> permute_bwd -> route_bwd
Buffers come from torch (device memory only); every step is a library kernel.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def to_device(a: np.ndarray, device="cuda"):
    """numpy -> GPU tensor; uint16 arrays are bf16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """GPU tensor -> numpy float32/int32 (bf16 widened exactly)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.numpy()


class RoutedFFNLayer:
    """Buffers and call order for one layer.  mode: "moe" | "mod" | "early_exit"."""

    def __init__(self, T, H, F, E=1, k=1, dtype="bf16", mode="moe", device="cuda"):
        self.T, self.H, self.F, self.E, self.k = T, H, F, E, k
        self.mode = mode
        self.residual = mode != "moe"
        self.dtype = dtype
        self.td = _TORCH_DTYPE[dtype]
        self.d = B.make_desc(T, H, F, E, k, dtype)
        dev = device
        R = T * k
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        act = dict(dtype=self.td, device=dev)
        self.expert_idx = torch.empty((T, k), **i32)
        self.gate_w = torch.empty((T, k), **f32)
        self.seg_offsets = torch.empty((E + 1,), **i32)
        self.src_slot = torch.empty((R,), **i32)
        self.dst_pos = torch.empty((T, k), **i32)
        self.x_p = torch.empty((R, H), **act)
        self.y_p = torch.empty((R, H), **act)
        self.G = torch.empty((R, F), **act)
        self.U = torch.empty((R, F), **act)
        self.out = torch.empty((T, H), **act)
        self.ws_permute = torch.empty((max(1, B.dynmo_permute_workspace_bytes(self.d)),), dtype=torch.uint8, device=dev)
        self.ws_fwd = torch.empty((B.dynmo_grouped_ffn_fwd_workspace_bytes(self.d),), dtype=torch.uint8, device=dev)
        # the load export's landing place on the host (pinned, so that the copy does not stall the stream)
        self._seg_host = torch.empty(E + 1, dtype=torch.int32, pin_memory=True)
        self._seg_event = torch.cuda.Event()
        self._bwd_ready = False
        self._dev = dev

    def alloc_backward(self):
        if self._bwd_ready:
            return
        T, H, F, E, k = self.T, self.H, self.F, self.E, self.k
        act = dict(dtype=self.td, device=self._dev)
        f32 = dict(dtype=torch.float32, device=self._dev)
        self.dy_p = torch.empty((T * k, H), **act)
        self.dx_p = torch.empty((T * k, H), **act)
        self.dgate = torch.empty((T, k), **f32)
        self.dx = torch.empty((T, H), **act)
        self.dWg = torch.empty((E, F, H), **act)
        self.dWu = torch.empty((E, F, H), **act)
        self.dWd = torch.empty((E, H, F), **act)
        self.droute = torch.empty((T, E) if self.mode == "moe" else (T,), **f32)
        self.ws_bwd = torch.empty((B.dynmo_grouped_ffn_bwd_workspace_bytes(self.d),), dtype=torch.uint8, device=self._dev)
        self._bwd_ready = True

    # ---- routing ----
    def route_topk(self, logits):
        B.dynmo_route_topk(self.d, logits, self.expert_idx, self.gate_w)

    def route_capacity(self, scores, cap):
        Bn, S = scores.shape
        B.dynmo_route_capacity(self.d, scores, Bn, S, cap, self.expert_idx, self.gate_w)

    def route_active(self, exit_layer, layer):
        B.dynmo_route_active(self.d, exit_layer, layer, self.expert_idx, self.gate_w)

    # ---- forward / backward after routing ----
    def forward(self, x, Wg, Wu, Wd, out=None):
        d = self.d
        out = self.out if out is None else out
        B.dynmo_permute(d, x, self.expert_idx, self.x_p, self.seg_offsets, self.src_slot, self.dst_pos, self.ws_permute)
        B.dynmo_grouped_ffn_fwd(d, self.x_p, self.seg_offsets, Wg, Wu, Wd, self.y_p, self.G, self.U, self.ws_fwd)
        B.dynmo_combine(d, self.y_p, self.dst_pos, self.gate_w, x if self.residual else None, out)
        return out

    def forward_gather(self, x, Wg, Wu, Wd, out=None):
        """Forward without the row copy: the first product reads its rows from x through
        src_slot (x_p is not written, so backward() cannot follow this call)."""
        d = self.d
        out = self.out if out is None else out
        B.dynmo_permute(d, None, self.expert_idx, None, self.seg_offsets, self.src_slot, self.dst_pos, self.ws_permute)
        B.dynmo_grouped_ffn_fwd_gather(d, x, self.src_slot, self.seg_offsets, Wg, Wu, Wd, self.y_p, self.G, self.U,
                                       self.ws_fwd)
        B.dynmo_combine(d, self.y_p, self.dst_pos, self.gate_w, x if self.residual else None, out)
        return out

    def forward_folded(self, x, Wg, Wu, Wd, out=None):
        """k = 1 only: the combine folded into the last product's stores.  A layer with a
        residual ("mod", "early_exit") updates x in place and returns it: tokens without a
        routed row are not touched; with `out` given it writes the routed tokens' rows of
        `out` instead (res = x) and the other rows of `out` are the caller's.  A top-1 "moe"
        layer writes self.out (every token has a row).  x_p and y_p are still written, so
        backward() may follow."""
        d = self.d
        if out is None:
            out = x if self.residual else self.out
        B.dynmo_permute(d, x, self.expert_idx, self.x_p, self.seg_offsets, self.src_slot, self.dst_pos, self.ws_permute)
        B.dynmo_grouped_ffn_fwd_combine(d, self.x_p, None, self.src_slot, self.seg_offsets, Wg, Wu, Wd, self.gate_w,
                                        x if self.residual else None, out, self.y_p, self.G, self.U, self.ws_fwd)
        return out

    def backward(self, dout, Wg, Wu, Wd, dx=None):
        self.alloc_backward()
        d = self.d
        dx = self.dx if dx is None else dx
        B.dynmo_combine_bwd(d, dout, self.y_p, self.dst_pos, self.gate_w, self.dy_p, self.dgate)
        B.dynmo_grouped_ffn_bwd(d, self.dy_p, self.x_p, self.G, self.U, self.seg_offsets, Wg, Wu, Wd, self.dx_p,
                                self.dWg, self.dWu, self.dWd, self.ws_bwd)
        B.dynmo_permute_bwd(d, self.dx_p, self.dst_pos, dout if self.residual else None, dx)
        return dx

    def backward_folded(self, dout, Wg, Wu, Wd, dx=None):
        """k = 1 only: the scatter back to token order folded into the stores of the dX product.
        A layer with a residual ("mod", "early_exit") updates dout in place and returns it (the
        gradient of a token without a routed row passes through untouched); with `dx` given it
        writes the routed tokens' rows of `dx` instead (dbase = dout) and the other rows of
        `dx` are the caller's.  A top-1 "moe" layer writes self.dx (every token has a row)."""
        self.alloc_backward()
        d = self.d
        if dx is None:
            dx = dout if self.residual else self.dx
        B.dynmo_combine_bwd(d, dout, self.y_p, self.dst_pos, self.gate_w, self.dy_p, self.dgate)
        B.dynmo_grouped_ffn_bwd_scatter(d, self.dy_p, self.x_p, self.G, self.U, self.seg_offsets, self.src_slot, Wg, Wu,
                                        Wd, dout if self.residual else None, dx, None, self.dWg, self.dWu, self.dWd,
                                        self.ws_bwd)
        return dx

    def route_bwd(self, scores=None):
        self.alloc_backward()
        if self.mode == "moe":
            B.dynmo_route_topk_bwd(self.d, self.dgate, self.gate_w, self.expert_idx, self.droute)
        elif self.mode == "mod":
            B.dynmo_route_capacity_bwd(self.d, self.dgate, scores, self.expert_idx, self.droute)
        return self.droute

    def load(self, cost_per_row=None):
        c = 18.0 * self.H * self.F if cost_per_row is None else cost_per_row
        return B.dynmo_layer_load(self.d, self.seg_offsets, c)

    def load_begin(self):
        """The load export without a stall: enqueues the copy of the segment offsets (final once the rows
        are permuted) into pinned host memory and records an event behind it; load_end() waits for that
        event only, not for whatever the stream was given since."""
        B.dynmo_layer_load_begin(self.d, self.seg_offsets, self._seg_host)
        self._seg_event.record()

    def load_end(self, cost_per_row=None):
        c = 18.0 * self.H * self.F if cost_per_row is None else cost_per_row
        self._seg_event.synchronize()
        return B.dynmo_layer_load_end(self.d, self._seg_host, c)
