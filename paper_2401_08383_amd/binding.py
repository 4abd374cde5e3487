"""Thin ctypes binding of ``libexflow_moe.so`` (the C ABI declared in ``include/exflow_moe.h``).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch
is used for device memory (``torch.empty(..., device="cuda")``, ``.data_ptr()``) and for the
current HIP stream.  There is no CPU fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libexflow_moe.so")

EXF_OK = 0
EXF_ERR_NULL_PTR = -1
EXF_ERR_BAD_SHAPE = -2
EXF_ERR_BAD_DTYPE = -3
EXF_ERR_WORKSPACE_TOO_SMALL = -4
EXF_ERR_HIP = -5
EXF_ERR_NOT_IMPLEMENTED = -6
EXF_ERR_MISALIGNED = -7
EXF_F32 = 0
EXF_BF16 = 1
EXF_ACT_GELU_ERF = 0
EXF_ACT_GELU_TANH = 1

_vp, _i, _i64, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t

# name -> (restype, argtypes); mirrors include/exflow_moe.h one to one
SIGNATURES = {
    "exf_version": (_i, []),
    "exf_last_error": (ctypes.c_char_p, []),
    "exf_check_placement": (_i, [_vp, _i, _i, _i]),
    "exf_comm_volume": (_i, [_i, _i64, _i, ctypes.c_double, ctypes.c_double, _vp]),
    "exf_transfer_ratios": (_i, [_vp, _vp, _i, _i64, _vp, _vp]),
    "moe_gate_topk": (_i, [_vp, _vp, _i64, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "moe_topk_from_logits": (_i, [_vp, _i64, _i, _i, _i, _vp, _vp, _vp]),
    "moe_dispatch_workspace_bytes": (_sz, [_i64, _i, _i]),
    "moe_dispatch": (_i, [_vp, _vp, _vp, _i64, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moe_dispatch_static": (_i, [_vp, _vp, _vp, _i64, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_expert_ffn_workspace_bytes": (_sz, [_i64, _i, _i, _i, _i]),
    "moe_expert_ffn": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp]),
    "moe_expert_ffn_fused_workspace_bytes": (_sz, [_i64, _i, _i, _i, _i, _i]),
    "moe_expert_ffn_fused": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp]),
    "moe_combine": (_i, [_vp, _vp, _vp, _i64, _i, _i, _i, _vp, _vp]),
    "affinity_histogram_workspace_bytes": (_sz, [_i, _i64, _i]),
    "affinity_histogram": (_i, [_vp, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "affinity_statistics_workspace_bytes": (_sz, [_i, _i64, _i]),
    "affinity_statistics": (_i, [_vp, _vp, _i, _i64, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "placement_locality_workspace_bytes": (_sz, [_i, _i64]),
    "placement_locality": (_i, [_vp, _vp, _i, _i64, _i, _i, _vp, _vp, _sz, _vp]),
    "affinity_multihop_workspace_bytes": (_sz, [_i, _i64, _i]),
    "affinity_multihop": (_i, [_vp, _i, _i64, _i, _vp, _vp, _vp, _sz, _vp]),
    "routing_transfers_workspace_bytes": (_sz, [_i, _i64]),
    "routing_transfers": (_i, [_vp, _vp, _vp, _i, _i64, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "placement_locality_from_counts": (_i, [_vp, _vp, _i, _i, _i, _vp, _vp]),
    "exf_placement_search": (_i, [_vp, _i, _i, _i, _i, _i, ctypes.c_uint64, _vp]),
    "exf_probe_copy": (_i, [_vp, _vp, _sz, _vp]),
    "exf_probe_mfma": (_i, [_i, _i, _vp, _vp]),
    "exf_probe_gemm_loop_bytes": (_sz, []),
    "exf_probe_gemm_loop": (_i, [_vp, _sz, _i, _vp, _vp]),
    "exf_probe_ffn_timeline": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i, _i, _i, _i, _vp, _vp, _sz, _vp, _i, _vp]),
}

_lib = None


class ExflowError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"exflow_moe error {code}: {message}")
        self.code = code


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2401_08383_amd.build` (there is no fallback path)")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def last_error() -> str:
    return lib().exf_last_error().decode()


def _check(rc: int) -> None:
    if rc != EXF_OK:
        raise ExflowError(rc, last_error())


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return EXF_F32
    if t.dtype == torch.bfloat16:
        return EXF_BF16
    raise ExflowError(EXF_ERR_BAD_DTYPE, f"unsupported dtype {t.dtype}")


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ----------------------------------------------------------------------------------------------
def moe_gate_topk(x, w_gate, k, renormalize=False, want_logits=False):
    """-> (topk_idx int32 [T,k], topk_w fp32 [T,k], logits fp32 [T,E] or None)."""
    T, d = x.shape
    E = w_gate.shape[0]
    assert w_gate.shape[1] == d and x.is_contiguous() and w_gate.is_contiguous() and x.dtype == w_gate.dtype
    idx = torch.empty((T, k), dtype=torch.int32, device=x.device)
    w = torch.empty((T, k), dtype=torch.float32, device=x.device)
    logits = torch.empty((T, E), dtype=torch.float32, device=x.device) if want_logits else None
    _check(lib().moe_gate_topk(_ptr(x), _ptr(w_gate), T, d, E, k, int(bool(renormalize)), dtype_code(x), _ptr(logits),
                               _ptr(idx), _ptr(w), _stream()))
    return idx, w, logits


def moe_topk_from_logits(logits, k, renormalize=False):
    T, E = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    idx = torch.empty((T, k), dtype=torch.int32, device=logits.device)
    w = torch.empty((T, k), dtype=torch.float32, device=logits.device)
    _check(lib().moe_topk_from_logits(_ptr(logits), T, E, k, int(bool(renormalize)), _ptr(idx), _ptr(w), _stream()))
    return idx, w


class DispatchResult:
    __slots__ = ("x_sorted", "src_of_sorted", "sorted_of_src", "expert_counts", "expert_offsets")

    def __init__(self, x_sorted, src_of_sorted, sorted_of_src, expert_counts, expert_offsets):
        self.x_sorted = x_sorted
        self.src_of_sorted = src_of_sorted
        self.sorted_of_src = sorted_of_src
        self.expert_counts = expert_counts
        self.expert_offsets = expert_offsets


def moe_dispatch(x, topk_idx, E, E_local=None, expert_map=None, out=None, workspace=None, gather=True):
    """Stable dispatch of the assignments; returns a DispatchResult of device tensors.

    Entries of ``src_of_sorted`` / rows of ``x_sorted`` at or beyond ``expert_offsets[E_local]``
    are left untouched by the library.  ``out`` may carry a previous DispatchResult to reuse.
    """
    T, k = topk_idx.shape
    d = x.shape[1]
    E_local = E if E_local is None else E_local
    A = T * k
    dev = topk_idx.device
    assert topk_idx.dtype == torch.int32 and topk_idx.is_contiguous() and x.is_contiguous()
    if out is None:
        out = DispatchResult(
            torch.empty((A, d), dtype=x.dtype, device=dev) if gather else None,
            torch.empty(A, dtype=torch.int32, device=dev),
            torch.empty(A, dtype=torch.int32, device=dev),
            torch.empty(E_local, dtype=torch.int32, device=dev),
            torch.empty(E_local + 1, dtype=torch.int32, device=dev),
        )
    nbytes = lib().moe_dispatch_workspace_bytes(T, k, E_local)
    if workspace is None:
        workspace = _workspace(nbytes, dev)
    _check(lib().moe_dispatch(_ptr(x), _ptr(topk_idx), _ptr(expert_map), T, d, k, E, E_local, dtype_code(x),
                              _ptr(out.x_sorted), _ptr(out.src_of_sorted), _ptr(out.sorted_of_src),
                              _ptr(out.expert_counts), _ptr(out.expert_offsets), _ptr(workspace), workspace.numel(), _stream()))
    return out


def moe_dispatch_static(x, topk_idx, E, out, E_local=None, expert_map=None):
    """moe_dispatch without a workspace and without any allocation: every output tensor comes from the
    caller (``out``: a DispatchResult; ``x_sorted`` None skips the row gather)."""
    T, k = topk_idx.shape
    d = x.shape[1]
    E_local = E if E_local is None else E_local
    assert topk_idx.dtype == torch.int32 and topk_idx.is_contiguous() and x.is_contiguous()
    _check(lib().moe_dispatch_static(_ptr(x), _ptr(topk_idx), _ptr(expert_map), T, d, k, E, E_local, dtype_code(x),
                                     _ptr(out.x_sorted), _ptr(out.src_of_sorted), _ptr(out.sorted_of_src),
                                     _ptr(out.expert_counts), _ptr(out.expert_offsets), _stream()))
    return out


def moe_expert_ffn(x_sorted, expert_offsets, w1, w2, b1=None, b2=None, act=EXF_ACT_GELU_ERF, out=None, workspace=None):
    A, d = x_sorted.shape
    E_local, f, d2 = w1.shape
    assert d2 == d and tuple(w2.shape) == (E_local, d, f) and expert_offsets.numel() == E_local + 1
    assert x_sorted.is_contiguous() and w1.is_contiguous() and w2.is_contiguous()
    assert expert_offsets.dtype == torch.int32
    dt = dtype_code(x_sorted)
    if out is None:
        out = torch.empty((A, d), dtype=x_sorted.dtype, device=x_sorted.device)
    nbytes = lib().moe_expert_ffn_workspace_bytes(A, d, f, E_local, dt)
    if workspace is None:
        workspace = _workspace(nbytes, x_sorted.device)
    _check(lib().moe_expert_ffn(_ptr(x_sorted), _ptr(expert_offsets), _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2), A, d, f,
                                E_local, act, dt, _ptr(out), _ptr(workspace), workspace.numel(), _stream()))
    return out


def moe_expert_ffn_fused(x, src_of_sorted, sorted_of_src, topk_w, expert_offsets, w1, w2, b1=None, b2=None,
                         act=EXF_ACT_GELU_ERF, out=None, workspace=None):
    """Expert FFN + combine straight from / to the unsorted token rows (bf16)."""
    T, d = x.shape
    k = topk_w.shape[1]
    E_local, f, d2 = w1.shape
    assert d2 == d and tuple(w2.shape) == (E_local, d, f) and expert_offsets.numel() == E_local + 1
    assert x.is_contiguous() and w1.is_contiguous() and w2.is_contiguous() and topk_w.is_contiguous()
    assert tuple(topk_w.shape) == (T, k) and topk_w.dtype == torch.float32
    assert src_of_sorted.numel() == T * k and sorted_of_src.numel() == T * k
    assert src_of_sorted.dtype == torch.int32 and sorted_of_src.dtype == torch.int32 and expert_offsets.dtype == torch.int32
    dt = dtype_code(x)
    if out is None:
        out = torch.empty((T, d), dtype=x.dtype, device=x.device)
    nbytes = lib().moe_expert_ffn_fused_workspace_bytes(T, k, d, f, E_local, dt)
    if workspace is None:
        workspace = _workspace(nbytes, x.device)
    _check(lib().moe_expert_ffn_fused(_ptr(x), _ptr(src_of_sorted), _ptr(sorted_of_src), _ptr(topk_w), _ptr(expert_offsets),
                                      _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2), T, k, d, f, E_local, act, dt, _ptr(out),
                                      _ptr(workspace), workspace.numel(), _stream()))
    return out


def moe_combine(y_sorted, sorted_of_src, topk_w, out=None):
    T, k = topk_w.shape
    d = y_sorted.shape[1]
    assert sorted_of_src.numel() == T * k and y_sorted.is_contiguous() and topk_w.dtype == torch.float32
    if out is None:
        out = torch.empty((T, d), dtype=y_sorted.dtype, device=y_sorted.device)
    _check(lib().moe_combine(_ptr(y_sorted), _ptr(sorted_of_src), _ptr(topk_w), T, d, k, dtype_code(y_sorted), _ptr(out),
                             _stream()))
    return out


def affinity_histogram(trace, E, want_loads=True, want_prob=True, want_invalid=True, workspace=None, out=None):
    """trace int32 [L,N] on the device -> dict(counts, loads, cond_prob, n_invalid) of device tensors."""
    L, N = trace.shape
    assert trace.dtype == torch.int32 and trace.is_contiguous()
    dev = trace.device
    if out is None:
        out = dict(
            counts=torch.empty((max(L - 1, 0), E, E), dtype=torch.int64, device=dev),
            loads=torch.empty((L, E), dtype=torch.int64, device=dev) if want_loads else None,
            cond_prob=torch.empty((max(L - 1, 0), E, E), dtype=torch.float32, device=dev) if want_prob else None,
            n_invalid=torch.empty(1, dtype=torch.int64, device=dev) if want_invalid else None,
        )
    nbytes = lib().affinity_histogram_workspace_bytes(L, N, E)
    if workspace is None:
        workspace = _workspace(nbytes, dev)
    _check(lib().affinity_histogram(_ptr(trace), L, N, E, _ptr(out["counts"]), _ptr(out["loads"]), _ptr(out["cond_prob"]),
                                    _ptr(out["n_invalid"]), _ptr(workspace), workspace.numel(), _stream()))
    return out


def affinity_statistics(trace, placement, G, want_loads=True, want_prob=True, want_invalid=True, workspace=None, out=None):
    """One pass over the trace -> dict(counts, loads, cond_prob, n_invalid, local_per_pair) of device tensors."""
    L, N = trace.shape
    E = placement.shape[1]
    assert placement.shape[0] == L and placement.dtype == torch.int32 and trace.dtype == torch.int32
    assert trace.is_contiguous() and placement.is_contiguous()
    dev = trace.device
    if out is None:
        out = dict(
            counts=torch.empty((max(L - 1, 0), E, E), dtype=torch.int64, device=dev),
            loads=torch.empty((L, E), dtype=torch.int64, device=dev) if want_loads else None,
            cond_prob=torch.empty((max(L - 1, 0), E, E), dtype=torch.float32, device=dev) if want_prob else None,
            n_invalid=torch.empty(1, dtype=torch.int64, device=dev) if want_invalid else None,
            local_per_pair=torch.empty(max(L - 1, 0), dtype=torch.int64, device=dev),
        )
    nbytes = lib().affinity_statistics_workspace_bytes(L, N, E)
    if workspace is None:
        workspace = _workspace(nbytes, dev)
    _check(lib().affinity_statistics(_ptr(trace), _ptr(placement), L, N, E, G, _ptr(out["counts"]), _ptr(out["loads"]),
                                     _ptr(out["cond_prob"]), _ptr(out["n_invalid"]), _ptr(out["local_per_pair"]), _ptr(workspace),
                                     workspace.numel(), _stream()))
    return out


def placement_locality(trace, placement, G, workspace=None, out=None):
    """-> local_per_pair int64 [L-1] (device); fraction = sum / (N*(L-1))."""
    L, N = trace.shape
    E = placement.shape[1]
    assert placement.shape[0] == L and placement.dtype == torch.int32 and trace.dtype == torch.int32
    assert trace.is_contiguous() and placement.is_contiguous()
    if out is None:
        out = torch.empty(max(L - 1, 0), dtype=torch.int64, device=trace.device)
    nbytes = lib().placement_locality_workspace_bytes(L, N)
    if workspace is None:
        workspace = _workspace(nbytes, trace.device)
    _check(lib().placement_locality(_ptr(trace), _ptr(placement), L, N, E, G, _ptr(out), _ptr(workspace), workspace.numel(),
                                    _stream()))
    return out


def affinity_multihop(trace, E, want_prob=True, workspace=None):
    """-> dict(counts int64 [L(L-1)/2,E,E], cond_prob fp32 or None) on the device, pairs source layer first."""
    L, N = trace.shape
    assert trace.dtype == torch.int32 and trace.is_contiguous()
    P = L * (L - 1) // 2
    counts = torch.empty((P, E, E), dtype=torch.int64, device=trace.device)
    prob = torch.empty((P, E, E), dtype=torch.float32, device=trace.device) if want_prob else None
    nbytes = lib().affinity_multihop_workspace_bytes(L, N, E)
    if workspace is None:
        workspace = _workspace(nbytes, trace.device)
    _check(lib().affinity_multihop(_ptr(trace), L, N, E, _ptr(counts), _ptr(prob), _ptr(workspace), workspace.numel(), _stream()))
    return {"counts": counts, "cond_prob": prob}


def routing_transfers(trace, placement, home, G, workspace=None):
    """-> (local_per_pair int64 [L-1], away_per_layer int64 [L]) on the device."""
    L, N = trace.shape
    E = placement.shape[1]
    assert placement.shape[0] == L and home.shape == (N,)
    assert trace.dtype == placement.dtype == home.dtype == torch.int32
    assert trace.is_contiguous() and placement.is_contiguous() and home.is_contiguous()
    local = torch.empty(max(L - 1, 0), dtype=torch.int64, device=trace.device)
    away = torch.empty(L, dtype=torch.int64, device=trace.device)
    nbytes = lib().routing_transfers_workspace_bytes(L, N)
    if workspace is None:
        workspace = _workspace(nbytes, trace.device)
    _check(lib().routing_transfers(_ptr(trace), _ptr(placement), _ptr(home), L, N, E, G, _ptr(local), _ptr(away), _ptr(workspace),
                                   workspace.numel(), _stream()))
    return local, away


def placement_locality_from_counts(counts, placements, out=None):
    """counts int64 [L-1,E,E] (device), placements int32 [B,L,E] (device) -> local int64 [B,L-1] (device)."""
    B, L, E = placements.shape
    assert counts.shape == (L - 1, E, E) and counts.dtype == torch.int64 and placements.dtype == torch.int32
    assert counts.is_contiguous() and placements.is_contiguous()
    if out is None:
        out = torch.empty((B, max(L - 1, 0)), dtype=torch.int64, device=counts.device)
    _check(lib().placement_locality_from_counts(_ptr(counts), _ptr(placements), B, L, E, _ptr(out), _stream()))
    return out


def placement_search(counts_host, G, nodes=1, restarts=4, seed=0):
    """counts_host int64 [L-1,E,E] (torch CPU) -> placement int32 [L,E] (torch CPU): the host solver."""
    assert counts_host.device.type == "cpu" and counts_host.dtype == torch.int64 and counts_host.is_contiguous()
    Lm1, E, _ = counts_host.shape
    out = torch.empty((Lm1 + 1, E), dtype=torch.int32)
    _check(lib().exf_placement_search(counts_host.data_ptr(), Lm1 + 1, E, G, nodes, restarts, seed, out.data_ptr()))
    return out


def check_placement(placement_host, G) -> bool:
    """Load-balance and exclusivity constraints of a HOST placement (torch CPU int32 [L,E])."""
    assert placement_host.device.type == "cpu" and placement_host.dtype == torch.int32 and placement_host.is_contiguous()
    L, E = placement_host.shape
    return lib().exf_check_placement(placement_host.data_ptr(), L, E, G) == EXF_OK


def comm_volume(G, N, L, p, p_star):
    """Forward communication of the paper's comparison table, in tokens:
    dict(vanilla_top1, vanilla_top2, coherent_top1, coherent_top2)."""
    out = (ctypes.c_double * 4)()
    _check(lib().exf_comm_volume(int(G), int(N), int(L), float(p), float(p_star), ctypes.addressof(out)))
    return dict(vanilla_top1=out[0], vanilla_top2=out[1], coherent_top1=out[2], coherent_top2=out[3])


def transfer_ratios(away_per_layer_host, local_per_pair_host, tokens):
    """(p, p_star) from HOST copies (torch CPU int64) of the counters routing_transfers returns."""
    assert away_per_layer_host.device.type == "cpu" and away_per_layer_host.dtype == torch.int64 and away_per_layer_host.is_contiguous()
    L = away_per_layer_host.numel()
    if L > 1:
        assert local_per_pair_host.device.type == "cpu" and local_per_pair_host.dtype == torch.int64
        assert local_per_pair_host.is_contiguous() and local_per_pair_host.numel() == L - 1
    p, p_star = ctypes.c_double(), ctypes.c_double()
    _check(lib().exf_transfer_ratios(away_per_layer_host.data_ptr(), local_per_pair_host.data_ptr() if L > 1 else None, L, int(tokens),
                                     ctypes.addressof(p), ctypes.addressof(p_star)))
    return p.value, p_star.value
