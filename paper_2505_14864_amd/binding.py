"""ctypes binding of libdynmo.so: one Python function per C-ABI call, same names.

Argument marshalling only.  Tensors are torch tensors on the GPU (torch is used
for device memory and streams, nothing else); every step runs in the library's
kernels.  There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdynmo.so")

DYNMO_F32, DYNMO_BF16 = 0, 1
_STATUS = {0: "DYNMO_OK", -1: "DYNMO_EINVAL", -2: "DYNMO_EUNSUPPORTED", -3: "DYNMO_EWORKSPACE", -4: "DYNMO_EHIP"}


class DynmoError(RuntimeError):
    def __init__(self, call, status, hip_error=0):
        self.status = status
        self.hip_error = hip_error
        msg = "%s returned %s" % (call, _STATUS.get(status, status))
        if status == -4:
            msg += " (hipError_t %d)" % hip_error
        super().__init__(msg)


class Desc(C.Structure):
    _fields_ = [("T", C.c_int32), ("H", C.c_int32), ("F", C.c_int32), ("E", C.c_int32), ("k", C.c_int32),
                ("dtype", C.c_int32)]


_P = C.c_void_p
_I = C.c_int32
_D = C.POINTER(Desc)

# name -> (restype, argtypes); mirrors include/dynmo.h one to one
SIGNATURES = {
    "dynmo_version": (_I, []),
    "dynmo_last_hip_error": (_I, []),
    "dynmo_route_topk": (_I, [_D, _P, _P, _P, _P]),
    "dynmo_route_capacity": (_I, [_D, _P, _I, _I, _I, _P, _P, _P]),
    "dynmo_route_active": (_I, [_D, _P, _I, _P, _P, _P]),
    "dynmo_route_topk_bwd": (_I, [_D, _P, _P, _P, _P, _P]),
    "dynmo_route_capacity_bwd": (_I, [_D, _P, _P, _P, _P, _P]),
    "dynmo_route_topk_ex": (_I, [_D, _P, _P, _I, _P, _P, _P]),
    "dynmo_route_topk_all_bwd": (_I, [_D, _P, _P, _P, _P, _P]),
    "dynmo_route_drop_workspace_bytes": (C.c_size_t, [_D]),
    "dynmo_route_drop": (_I, [_D, _P, _I, _P, _P, C.c_size_t, _P]),
    "dynmo_permute_workspace_bytes": (C.c_size_t, [_D]),
    "dynmo_permute": (_I, [_D, _P, _P, _P, _P, _P, _P, _P, C.c_size_t, _P]),
    "dynmo_permute_static_max_slots": (C.c_size_t, [_I]),
    "dynmo_permute_static": (_I, [_D, _P, _P, _P, _P, _P, _P, _P]),
    "dynmo_permute_bwd": (_I, [_D, _P, _P, _P, _P, _P]),
    "dynmo_grouped_ffn_fwd_workspace_bytes": (C.c_size_t, [_D]),
    "dynmo_grouped_ffn_fwd": (_I, [_D, _P, _P, _P, _P, _P, _P, _P, _P, _P, C.c_size_t, _P]),
    "dynmo_grouped_ffn_fwd_gather": (_I, [_D, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, C.c_size_t, _P]),
    "dynmo_grouped_ffn_fwd_combine": (_I, [_D] + [_P] * 14 + [C.c_size_t, _P]),
    "dynmo_grouped_ffn_bwd_workspace_bytes": (C.c_size_t, [_D]),
    "dynmo_grouped_ffn_bwd": (_I, [_D] + [_P] * 13 + [C.c_size_t, _P]),
    "dynmo_grouped_ffn_bwd_scatter": (_I, [_D] + [_P] * 16 + [C.c_size_t, _P]),
    "dynmo_combine": (_I, [_D, _P, _P, _P, _P, _P, _P]),
    "dynmo_combine_bwd": (_I, [_D, _P, _P, _P, _P, _P, _P, _P]),
    "dynmo_layer_load": (_I, [_D, _P, C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_double), _P]),
    "dynmo_layer_load_begin": (_I, [_D, _P, _P, _P]),
    "dynmo_layer_load_end": (_I, [_D, _P, C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "dynmo_partition": (_I, [C.POINTER(C.c_double), _I, _I, C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "dynmo_partition_shadow": (_I, [C.POINTER(C.c_double), C.POINTER(C.c_int32), _I, _I, C.POINTER(C.c_int32),
                                    C.POINTER(C.c_double), C.POINTER(C.c_int32)]),
    "dynmo_uniform_bounds": (_I, [_I, _I, C.POINTER(C.c_int32)]),
    "dynmo_stage_loads": (_I, [C.POINTER(C.c_double), _I, C.POINTER(C.c_int32), _I, C.POINTER(C.c_double)]),
    "dynmo_imbalance": (_I, [C.POINTER(C.c_double), _I, C.POINTER(C.c_double)]),
    "dynmo_potential": (_I, [C.POINTER(C.c_double), _I, C.POINTER(C.c_double)]),
    "dynmo_diffusion": (_I, [C.POINTER(C.c_double), _I, _I, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.c_double,
                             C.c_double, _I, C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "dynmo_repack": (_I, [_I, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_int32), _I, C.c_double,
                          C.POINTER(C.c_int32), _I, C.POINTER(C.c_int32)]),
    "dynmo_profile_enable": (_I, [_I]),
    "dynmo_profile_reset": (_I, []),
    "dynmo_profile_kernel_count": (_I, []),
    "dynmo_profile_kernel_name": (C.c_char_p, [_I]),
    "dynmo_profile_read": (_I, [_I, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "dynmo_peak_mfma_bf16": (_I, [_I, _P, _P, C.POINTER(C.c_double), _P]),
    "dynmo_peak_copy": (_I, [_P, _P, C.c_size_t, _P]),
}

_lib = None


def lib():
    """Loads the built library (never builds, never falls back)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdynmo.so is not built: run `python -m paper_2505_14864_amd.build` "
                               "(or __graft_entry__.build()); there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def make_desc(T, H, F, E, k, dtype):
    code = {"f32": DYNMO_F32, "bf16": DYNMO_BF16, torch.float32: DYNMO_F32, torch.bfloat16: DYNMO_BF16}.get(dtype, dtype)
    return Desc(int(T), int(H), int(F), int(E), int(k), int(code))


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return t.data_ptr()


def _pinned_ptr(t, n):
    if t.is_cuda or not t.is_pinned() or not t.is_contiguous() or t.dtype != torch.int32 or t.numel() < n:
        raise ValueError("expected a contiguous pinned int32 host tensor of at least %d elements" % n)
    return t.data_ptr()


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _check(call, rc):
    if rc != 0:
        raise DynmoError(call, rc, lib().dynmo_last_hip_error())


def dynmo_version():
    return lib().dynmo_version()


def dynmo_route_topk(d, logits, expert_idx, gate_w, stream=None):
    _check("dynmo_route_topk", lib().dynmo_route_topk(C.byref(d), _ptr(logits), _ptr(expert_idx), _ptr(gate_w), _stream(stream)))


def dynmo_route_capacity(d, scores, B, S, cap, expert_idx, gate_w, stream=None):
    _check("dynmo_route_capacity", lib().dynmo_route_capacity(C.byref(d), _ptr(scores), B, S, cap, _ptr(expert_idx),
                                                              _ptr(gate_w), _stream(stream)))


def dynmo_route_active(d, exit_layer, layer, expert_idx, gate_w, stream=None):
    _check("dynmo_route_active", lib().dynmo_route_active(C.byref(d), _ptr(exit_layer), layer, _ptr(expert_idx),
                                                          _ptr(gate_w), _stream(stream)))


def dynmo_route_topk_bwd(d, dgate, gate_w, expert_idx, dlogits, stream=None):
    _check("dynmo_route_topk_bwd", lib().dynmo_route_topk_bwd(C.byref(d), _ptr(dgate), _ptr(gate_w), _ptr(expert_idx),
                                                              _ptr(dlogits), _stream(stream)))


def dynmo_route_capacity_bwd(d, dgate, scores, expert_idx, dscores, stream=None):
    _check("dynmo_route_capacity_bwd", lib().dynmo_route_capacity_bwd(C.byref(d), _ptr(dgate), _ptr(scores),
                                                                      _ptr(expert_idx), _ptr(dscores), _stream(stream)))


NORM_SELECTED, NORM_ALL = 0, 1


def dynmo_route_topk_ex(d, logits, bias, gate_norm, expert_idx, gate_w, stream=None):
    _check("dynmo_route_topk_ex", lib().dynmo_route_topk_ex(C.byref(d), _ptr(logits), _ptr(bias), int(gate_norm),
                                                            _ptr(expert_idx), _ptr(gate_w), _stream(stream)))


def dynmo_route_topk_all_bwd(d, dgate, logits, expert_idx, dlogits, stream=None):
    _check("dynmo_route_topk_all_bwd", lib().dynmo_route_topk_all_bwd(C.byref(d), _ptr(dgate), _ptr(logits),
                                                                      _ptr(expert_idx), _ptr(dlogits), _stream(stream)))


def dynmo_route_drop_workspace_bytes(d):
    return int(lib().dynmo_route_drop_workspace_bytes(C.byref(d)))


def dynmo_route_drop(d, expert_idx, capacity, expert_idx_kept, workspace, stream=None):
    _check("dynmo_route_drop", lib().dynmo_route_drop(C.byref(d), _ptr(expert_idx), int(capacity), _ptr(expert_idx_kept),
                                                      _ptr(workspace), workspace.numel(), _stream(stream)))


def dynmo_permute_workspace_bytes(d):
    return lib().dynmo_permute_workspace_bytes(C.byref(d))


def dynmo_permute(d, x, expert_idx, x_p, seg_offsets, src_slot, dst_pos, workspace, stream=None):
    _check("dynmo_permute", lib().dynmo_permute(C.byref(d), _ptr(x), _ptr(expert_idx), _ptr(x_p), _ptr(seg_offsets),
                                                _ptr(src_slot), _ptr(dst_pos), _ptr(workspace), workspace.numel(),
                                                _stream(stream)))


def dynmo_permute_static_max_slots(E):
    return lib().dynmo_permute_static_max_slots(int(E))


def dynmo_permute_static(d, x, expert_idx, x_p, seg_offsets, src_slot, dst_pos, stream=None):
    _check("dynmo_permute_static", lib().dynmo_permute_static(C.byref(d), _ptr(x), _ptr(expert_idx), _ptr(x_p),
                                                              _ptr(seg_offsets), _ptr(src_slot), _ptr(dst_pos),
                                                              _stream(stream)))


def dynmo_permute_bwd(d, dx_p, dst_pos, dbase, dx, stream=None):
    _check("dynmo_permute_bwd", lib().dynmo_permute_bwd(C.byref(d), _ptr(dx_p), _ptr(dst_pos), _ptr(dbase), _ptr(dx),
                                                        _stream(stream)))


def dynmo_grouped_ffn_fwd_workspace_bytes(d):
    return lib().dynmo_grouped_ffn_fwd_workspace_bytes(C.byref(d))


def dynmo_grouped_ffn_fwd(d, x_p, seg_offsets, Wg, Wu, Wd, y_p, G_save, U_save, workspace, stream=None):
    _check("dynmo_grouped_ffn_fwd", lib().dynmo_grouped_ffn_fwd(
        C.byref(d), _ptr(x_p), _ptr(seg_offsets), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(y_p), _ptr(G_save), _ptr(U_save),
        _ptr(workspace), workspace.numel(), _stream(stream)))


def dynmo_grouped_ffn_fwd_gather(d, x, src_slot, seg_offsets, Wg, Wu, Wd, y_p, G_save, U_save, workspace, stream=None):
    _check("dynmo_grouped_ffn_fwd_gather", lib().dynmo_grouped_ffn_fwd_gather(
        C.byref(d), _ptr(x), _ptr(src_slot), _ptr(seg_offsets), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(y_p),
        _ptr(G_save), _ptr(U_save), _ptr(workspace), workspace.numel(), _stream(stream)))


def dynmo_grouped_ffn_fwd_combine(d, x_p, x, src_slot, seg_offsets, Wg, Wu, Wd, gate_w, res, out, y_p, G_save, U_save,
                                  workspace, stream=None):
    _check("dynmo_grouped_ffn_fwd_combine", lib().dynmo_grouped_ffn_fwd_combine(
        C.byref(d), _ptr(x_p), _ptr(x), _ptr(src_slot), _ptr(seg_offsets), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(gate_w),
        _ptr(res), _ptr(out), _ptr(y_p), _ptr(G_save), _ptr(U_save), _ptr(workspace), workspace.numel(),
        _stream(stream)))


def dynmo_grouped_ffn_bwd_workspace_bytes(d):
    return lib().dynmo_grouped_ffn_bwd_workspace_bytes(C.byref(d))


def dynmo_grouped_ffn_bwd(d, dy_p, x_p, G_save, U_save, seg_offsets, Wg, Wu, Wd, dx_p, dWg, dWu, dWd, workspace,
                          stream=None):
    _check("dynmo_grouped_ffn_bwd", lib().dynmo_grouped_ffn_bwd(
        C.byref(d), _ptr(dy_p), _ptr(x_p), _ptr(G_save), _ptr(U_save), _ptr(seg_offsets), _ptr(Wg), _ptr(Wu), _ptr(Wd),
        _ptr(dx_p), _ptr(dWg), _ptr(dWu), _ptr(dWd), _ptr(workspace), workspace.numel(), _stream(stream)))


def dynmo_grouped_ffn_bwd_scatter(d, dy_p, x_p, G_save, U_save, seg_offsets, src_slot, Wg, Wu, Wd, dbase, dx, dx_p, dWg,
                                  dWu, dWd, workspace, stream=None):
    _check("dynmo_grouped_ffn_bwd_scatter", lib().dynmo_grouped_ffn_bwd_scatter(
        C.byref(d), _ptr(dy_p), _ptr(x_p), _ptr(G_save), _ptr(U_save), _ptr(seg_offsets), _ptr(src_slot), _ptr(Wg),
        _ptr(Wu), _ptr(Wd), _ptr(dbase), _ptr(dx), _ptr(dx_p), _ptr(dWg), _ptr(dWu), _ptr(dWd), _ptr(workspace),
        workspace.numel(), _stream(stream)))


def dynmo_combine(d, y_p, dst_pos, gate_w, base, out, stream=None):
    _check("dynmo_combine", lib().dynmo_combine(C.byref(d), _ptr(y_p), _ptr(dst_pos), _ptr(gate_w), _ptr(base), _ptr(out),
                                                _stream(stream)))


def dynmo_combine_bwd(d, dout, y_p, dst_pos, gate_w, dy_p, dgate, stream=None):
    _check("dynmo_combine_bwd", lib().dynmo_combine_bwd(C.byref(d), _ptr(dout), _ptr(y_p), _ptr(dst_pos), _ptr(gate_w),
                                                        _ptr(dy_p), _ptr(dgate), _stream(stream)))


def dynmo_layer_load(d, seg_offsets, cost_per_row, stream=None):
    """Returns (counts list[E], load float).  Synchronises the stream."""
    counts = (C.c_int32 * d.E)()
    load = C.c_double()
    _check("dynmo_layer_load", lib().dynmo_layer_load(C.byref(d), _ptr(seg_offsets), float(cost_per_row), counts,
                                                      C.byref(load), _stream(stream)))
    return list(counts), load.value


def dynmo_layer_load_begin(d, seg_offsets, seg_host, stream=None):
    """Enqueues the copy of seg_offsets into seg_host (a pinned int32 host tensor of E+1 elements); no wait."""
    _check("dynmo_layer_load_begin", lib().dynmo_layer_load_begin(C.byref(d), _ptr(seg_offsets), _pinned_ptr(seg_host, d.E + 1),
                                                                  _stream(stream)))


def dynmo_layer_load_end(d, seg_host, cost_per_row):
    """Returns (counts list[E], load float) from seg_host once its copy has completed.  No GPU call."""
    counts = (C.c_int32 * d.E)()
    load = C.c_double()
    _check("dynmo_layer_load_end", lib().dynmo_layer_load_end(C.byref(d), _pinned_ptr(seg_host, d.E + 1), float(cost_per_row), counts,
                                                              C.byref(load)))
    return list(counts), load.value


# ---- host-only calls (plain Python sequences in, lists out) -----------------

def _darr(v):
    return (C.c_double * len(v))(*[float(a) for a in v])


def _iarr(v):
    return (C.c_int32 * len(v))(*[int(a) for a in v])


def dynmo_partition(loads, S):
    """Returns (bounds list[S+1], bottleneck)."""
    bounds = (C.c_int32 * (S + 1))()
    b = C.c_double()
    _check("dynmo_partition", lib().dynmo_partition(_darr(loads), len(loads), S, bounds, C.byref(b)))
    return list(bounds), b.value


def dynmo_partition_shadow(loads, shadow, S):
    """Returns (bounds list[S+1], bottleneck, most layers on one stage)."""
    bounds = (C.c_int32 * (S + 1))()
    b = C.c_double()
    m = C.c_int32()
    sh = None if shadow is None else (C.c_int32 * len(loads))(*[int(v) for v in shadow])
    _check("dynmo_partition_shadow", lib().dynmo_partition_shadow(_darr(loads), sh, len(loads), S, bounds, C.byref(b),
                                                                  C.byref(m)))
    return list(bounds), b.value, m.value


def dynmo_uniform_bounds(L, S):
    bounds = (C.c_int32 * (S + 1))()
    _check("dynmo_uniform_bounds", lib().dynmo_uniform_bounds(L, S, bounds))
    return list(bounds)


def dynmo_stage_loads(loads, bounds):
    S = len(bounds) - 1
    out = (C.c_double * S)()
    _check("dynmo_stage_loads", lib().dynmo_stage_loads(_darr(loads), len(loads), _iarr(bounds), S, out))
    return list(out)


def dynmo_imbalance(stage_loads):
    r = C.c_double()
    _check("dynmo_imbalance", lib().dynmo_imbalance(_darr(stage_loads), len(stage_loads), C.byref(r)))
    return r.value


# ---- profiling step ---------------------------------------------------------

def dynmo_potential(stage_loads):
    a = _darr(stage_loads)
    out = C.c_double()
    _check("dynmo_potential", lib().dynmo_potential(a, len(stage_loads), C.byref(out)))
    return out.value


def dynmo_diffusion(loads, bounds, layer_mem=None, max_mem=float("inf"), gamma=0.0, max_rounds=1 << 30):
    """Returns (bounds, rounds, phi_before, phi_after)."""
    la, ba = _darr(loads), _iarr(bounds)
    ma = _darr(layer_mem) if layer_mem is not None else None
    rounds, phi = C.c_int32(), (C.c_double * 2)()
    _check("dynmo_diffusion", lib().dynmo_diffusion(la, len(loads), len(bounds) - 1, ba, ma, float(max_mem),
                                                    float(gamma), int(max_rounds), C.byref(rounds), phi))
    return list(ba), rounds.value, phi[0], phi[1]


def dynmo_repack(active_workers, mem_usage, num_layers, target_num_workers, max_mem, capacity=None):
    """Returns (transfers, active_workers, mem_usage, num_layers) like the listing's state after the run."""
    n = len(active_workers)
    act, mem, nl = _iarr(active_workers), _darr(mem_usage), _iarr(num_layers)
    cap = n * max(1, sum(int(v) for v in num_layers)) if capacity is None else int(capacity)
    tr = (C.c_int32 * max(1, 3 * cap))()
    cnt = C.c_int32()
    _check("dynmo_repack", lib().dynmo_repack(n, act, mem, nl, int(target_num_workers), float(max_mem), tr, cap,
                                              C.byref(cnt)))
    return [tuple(tr[3 * i:3 * i + 3]) for i in range(cnt.value)], list(act), list(mem), list(nl)


def dynmo_profile_enable(on):
    _check("dynmo_profile_enable", lib().dynmo_profile_enable(1 if on else 0))


def dynmo_profile_reset():
    _check("dynmo_profile_reset", lib().dynmo_profile_reset())


def dynmo_profile_kernel_count():
    return lib().dynmo_profile_kernel_count()


def dynmo_profile_kernel_name(i):
    return lib().dynmo_profile_kernel_name(i).decode()


def dynmo_profile_read(i):
    """Returns (total_ms, launches) of kernel role i; waits for those launches."""
    ms = C.c_double()
    n = C.c_int64()
    _check("dynmo_profile_read", lib().dynmo_profile_read(i, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def dynmo_peak_mfma_bf16(iters, sink, operands=None, stream=None):
    """Launches the register-resident MFMA loop; returns the launch's flop count."""
    fl = C.c_double()
    _check("dynmo_peak_mfma_bf16", lib().dynmo_peak_mfma_bf16(int(iters), _ptr(operands), _ptr(sink), C.byref(fl),
                                                              _stream(stream)))
    return fl.value


def dynmo_peak_copy(dst, src, stream=None):
    nbytes = src.numel() * src.element_size()
    _check("dynmo_peak_copy", lib().dynmo_peak_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)))
    return nbytes
