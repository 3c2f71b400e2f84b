"""Thin ctypes binding of the C2R HIP library (include/c2r.h).

Argument marshalling only: torch provides device memory and the current stream;
every step of the path runs in the library's kernels.  There is no CPU or
PyTorch fallback: if libc2r_hip.so is missing, importing the functions raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libc2r_hip.so")

F32, BF16 = 0, 1
STAGE_COACTIVATION, STAGE_ROUTE, STAGE_PERMUTE, STAGE_EXPERT_FFN, STAGE_DEDUP_DISPATCH = 0, 1, 2, 3, 4
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH = 0, -1, -2, -3, -4
_ERRNAMES = {-1: "C2R_ERR_INVALID_ARG", -2: "C2R_ERR_UNSUPPORTED", -3: "C2R_ERR_WORKSPACE",
             -4: "C2R_ERR_LAUNCH"}

EXPORTS = ["c2r_version", "c2r_route_chunk", "c2r_workspace_bytes", "c2r_build_coactivation",
           "c2r_collaborators", "c2r_route", "c2r_route_from_logits", "c2r_profile_from_logits", "c2r_permute", "c2r_permute_noalloc", "c2r_expert_ffn",
           "c2r_expert_ffn_gate_up", "c2r_expert_ffn_gate_up_gather", "c2r_expert_ffn_gather", "c2r_expert_ffn_down",
           "c2r_expert_ffn_gate_up_with_shared", "c2r_expert_ffn_down_with_shared", "c2r_combine",
           "c2r_place_experts", "c2r_dedup_dispatch", "c2r_combine_partial", "c2r_combine_copies",
           "c2r_collaboration_degree", "c2r_distinct_devices"]


class C2RError(RuntimeError):
    def __init__(self, fn, code):
        super().__init__(f"{fn} failed: {_ERRNAMES.get(code, code)}")
        self.code = code


_lib = None


def lib():
    """Load the HIP library; raise loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2504_01337_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
        L.c2r_version.restype = i32
        L.c2r_route_chunk.restype = i32
        L.c2r_workspace_bytes.restype = sz
        L.c2r_workspace_bytes.argtypes = [i32, i64, i32, i32, i32, i32, i32]
        L.c2r_build_coactivation.argtypes = [vp, i64, i32, i32, vp, vp]
        L.c2r_collaborators.argtypes = [vp, i32, i32, vp, vp, vp]
        L.c2r_route.argtypes = [vp, i32, vp, vp, i64, i32, i32, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        L.c2r_route_from_logits.argtypes = [vp, i64, i32, i32, vp, i32, vp, vp, vp]
        L.c2r_profile_from_logits.argtypes = [vp, i64, i32, i32, vp, i32, vp, vp, vp, vp]
        L.c2r_permute.argtypes = [vp, i32, vp, i64, i32, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.c2r_permute_noalloc.argtypes = [vp, i32, vp, i64, i32, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp]
        L.c2r_expert_ffn.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.c2r_expert_ffn_gate_up.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, vp, vp]
        L.c2r_expert_ffn_gate_up_gather.argtypes = [vp, i32, vp, i64, i32, vp, i32, i64, i32, i32, vp, vp, vp, vp]
        L.c2r_expert_ffn_gather.argtypes = [vp, i32, vp, i64, i32, vp, i32, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.c2r_expert_ffn_down.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, vp]
        L.c2r_expert_ffn_gate_up_with_shared.argtypes = [vp, i32, vp, i64, i32, vp, i32, i64, i32, i32, vp, vp, vp,
                                                         i32, vp, vp, vp, vp]
        L.c2r_expert_ffn_down_with_shared.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, i64, i32, vp, vp, vp, vp]
        L.c2r_combine.argtypes = [vp, i32, vp, vp, i64, i32, i32, vp, vp, vp]
        L.c2r_place_experts.argtypes = [vp, i32, i32, vp, vp]
        L.c2r_dedup_dispatch.argtypes = [vp, i64, i32, i32, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.c2r_combine_partial.argtypes = [vp, i32, vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, vp]
        L.c2r_combine_copies.argtypes = [vp, i32, vp, i64, i64, i32, i32, vp, vp, vp]
        L.c2r_collaboration_degree.argtypes = [vp, i32, vp, vp]
        L.c2r_distinct_devices.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp, vp, vp]
        for name in EXPORTS[3:]:
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(fn, rc):
    if rc != OK:
        raise C2RError(fn, rc)


def _ws(nbytes: int, device, ws: Optional[torch.Tensor]):
    if ws is not None:
        return ws
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def version() -> int:
    return lib().c2r_version()


def route_chunk() -> int:
    return lib().c2r_route_chunk()


def workspace_bytes(stage, T, d, E, K, F, dt) -> int:
    return int(lib().c2r_workspace_bytes(stage, T, d, E, K, F, dt))


def build_coactivation(topk_idx: torch.Tensor, E: int, Cm: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 2.  Accumulates into Cm (int32[E,E]); a zeroed matrix is made if None."""
    T, K = topk_idx.shape
    if Cm is None:
        Cm = torch.zeros((E, E), dtype=torch.int32, device=topk_idx.device)
    _check("c2r_build_coactivation",
           lib().c2r_build_coactivation(_ptr(topk_idx), T, K, E, _ptr(Cm), _stream()))
    return Cm


def collaborators(Cm: torch.Tensor, Tc: int, out=None):
    """Eq. 4.  Returns (collab_idx int32[E, min(Tc,E-1)], collab_mask int64[E])."""
    E = Cm.shape[0]
    n = min(Tc, E - 1)
    if out is None:
        idx = torch.empty((E, n), dtype=torch.int32, device=Cm.device)
        mask = torch.empty((E,), dtype=torch.int64, device=Cm.device)
    else:
        idx, mask = out
    _check("c2r_collaborators", lib().c2r_collaborators(_ptr(Cm), E, Tc, _ptr(idx), _ptr(mask), _stream()))
    return idx, mask


def route(x, Wg, bias, K, collab_idx=None, want_logits=False, ws=None, out=None):
    """Eq. 1 + Sec. 3.3 selection.  Returns (topk_idx, gates, logits or None)."""
    T, d = x.shape
    E = Wg.shape[1]
    assert Wg.shape[0] == d and Wg.dtype == torch.float32
    dev = x.device
    if out is None:
        idx = torch.empty((T, K), dtype=torch.int32, device=dev)
        gates = torch.empty((T, K), dtype=torch.float32, device=dev)
    else:
        idx, gates = out
    logits = torch.empty((T, E), dtype=torch.float32, device=dev) if want_logits else None
    Tc = 0 if collab_idx is None else collab_idx.shape[1]
    ws = _ws(workspace_bytes(STAGE_ROUTE, T, d, E, K, 0, _dt(x)), dev, ws)
    _check("c2r_route", lib().c2r_route(_ptr(x), _dt(x), _ptr(Wg), _ptr(bias), T, d, E, K, _ptr(collab_idx), Tc,
                                        _ptr(idx), _ptr(gates), _ptr(logits), _ptr(ws), ws.numel(), _stream()))
    return idx, gates, logits


def route_from_logits(logits, K, collab_idx=None, out=None):
    T, E = logits.shape
    if out is None:
        idx = torch.empty((T, K), dtype=torch.int32, device=logits.device)
        gates = torch.empty((T, K), dtype=torch.float32, device=logits.device)
    else:
        idx, gates = out
    Tc = 0 if collab_idx is None else collab_idx.shape[1]
    _check("c2r_route_from_logits", lib().c2r_route_from_logits(_ptr(logits), T, E, K, _ptr(collab_idx), Tc,
                                                                 _ptr(idx), _ptr(gates), _stream()))
    return idx, gates


def profile_from_logits(logits, K, Cm, collab_idx=None, out=None, want_selection=False):
    """Selection from stored logits and co-activation counts (added to Cm, int32[E, E]) in one launch.
    out = (topk_idx, gates) to have the selections written as well (or want_selection=True to have
    them allocated); returns (Cm, topk_idx or None, gates or None)."""
    T, E = logits.shape
    idx = gates = None
    if out is not None:
        idx, gates = out
    elif want_selection:
        idx = torch.empty((T, K), dtype=torch.int32, device=logits.device)
        gates = torch.empty((T, K), dtype=torch.float32, device=logits.device)
    Tc = 0 if collab_idx is None else collab_idx.shape[1]
    _check("c2r_profile_from_logits", lib().c2r_profile_from_logits(_ptr(logits), T, E, K, _ptr(collab_idx), Tc,
                                                                     _ptr(idx), _ptr(gates), _ptr(Cm), _stream()))
    return Cm, idx, gates


def permute(x, topk_idx, E, local_slot=None, E_local=None, ws=None, out=None, rows=True):
    """Dispatch.  Returns (counts, offsets, perm, inv_perm, x_perm)."""
    T, K = topk_idx.shape
    dev = topk_idx.device
    E_local = E if E_local is None else E_local
    d = x.shape[1] if x is not None else 0
    if out is None:
        counts = torch.empty((E_local,), dtype=torch.int32, device=dev)
        offsets = torch.empty((E_local + 1,), dtype=torch.int32, device=dev)
        perm = torch.full((T * K,), -1, dtype=torch.int32, device=dev)
        inv_perm = torch.empty((T * K,), dtype=torch.int32, device=dev)
        x_perm = torch.empty((T * K, d), dtype=x.dtype, device=dev) if (rows and x is not None) else None
    else:
        counts, offsets, perm, inv_perm, x_perm = out
    dt = _dt(x) if x is not None else F32
    ws = _ws(workspace_bytes(STAGE_PERMUTE, T, d, E, K, 0, dt), dev, ws)
    _check("c2r_permute", lib().c2r_permute(_ptr(x), dt, _ptr(topk_idx), T, d, E, K, _ptr(local_slot), E_local,
                                            _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(x_perm),
                                            _ptr(ws), ws.numel(), _stream()))
    return counts, offsets, perm, inv_perm, x_perm


def permute_noalloc(x, topk_idx, E, local_slot, E_local, out):
    """c2r_permute without a workspace (static device scratch); the caller passes every output:
    out = (counts, offsets, perm, inv_perm, x_perm or None).  Nothing is allocated."""
    T, K = topk_idx.shape
    counts, offsets, perm, inv_perm, x_perm = out
    d = x.shape[1] if x is not None else 0
    dt = _dt(x) if x is not None else F32
    _check("c2r_permute_noalloc", lib().c2r_permute_noalloc(
        _ptr(x), dt, _ptr(topk_idx), T, d, E, K, _ptr(local_slot), E_local, _ptr(counts), _ptr(offsets),
        _ptr(perm), _ptr(inv_perm), _ptr(x_perm), _stream()))
    return out


def expert_ffn(x_perm, offsets, w_gate, w_up, w_down, ws=None, out=None):
    """Grouped SwiGLU FFN over the rows of each expert.  Returns y_perm."""
    A_cap, d = x_perm.shape
    E_local, F, _ = w_gate.shape
    assert offsets.numel() == E_local + 1 and offsets.dtype == torch.int32
    assert w_up.shape == (E_local, F, d) and w_down.shape == (E_local, d, F)
    assert w_gate.dtype == x_perm.dtype == w_up.dtype == w_down.dtype
    y_perm = torch.empty_like(x_perm) if out is None else out
    ws = _ws(workspace_bytes(STAGE_EXPERT_FFN, A_cap, d, E_local, 1, F, _dt(x_perm)), x_perm.device, ws)
    _check("c2r_expert_ffn", lib().c2r_expert_ffn(_ptr(x_perm), _dt(x_perm), _ptr(offsets), E_local, A_cap, d, F,
                                                  _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(y_perm), _ptr(ws),
                                                  ws.numel(), _stream()))
    return y_perm


def expert_ffn_gate_up(x_perm, offsets, w_gate, w_up, h):
    """First pass of the expert FFN: h = silu(x W_gate^T) * (x W_up^T)."""
    A_cap, d = x_perm.shape
    E_local, F, _ = w_gate.shape
    assert h.shape == (A_cap, F) and h.dtype == x_perm.dtype
    _check("c2r_expert_ffn_gate_up", lib().c2r_expert_ffn_gate_up(
        _ptr(x_perm), _dt(x_perm), _ptr(offsets), E_local, A_cap, d, F, _ptr(w_gate), _ptr(w_up), _ptr(h), _stream()))
    return h


def expert_ffn_gate_up_gather(x, perm, K, offsets, w_gate, w_up, h):
    """First FFN pass reading row p as x[perm[p] // K] (dispatch gather folded in)."""
    T, d = x.shape
    A_cap = perm.numel()
    E_local, F, _ = w_gate.shape
    assert h.shape == (A_cap, F) and h.dtype == x.dtype and perm.dtype == torch.int32
    _check("c2r_expert_ffn_gate_up_gather", lib().c2r_expert_ffn_gate_up_gather(
        _ptr(x), _dt(x), _ptr(perm), T, K, _ptr(offsets), E_local, A_cap, d, F, _ptr(w_gate), _ptr(w_up), _ptr(h),
        _stream()))
    return h


def expert_ffn_gather(x, perm, K, offsets, w_gate, w_up, w_down, ws=None, out=None):
    """Both FFN passes, the first reading row p as x[perm[p] // K]; h lives in the workspace, any F % 8 == 0."""
    T, d = x.shape
    A_cap = perm.numel()
    E_local, F, _ = w_gate.shape
    assert w_up.shape == (E_local, F, d) and w_down.shape == (E_local, d, F) and perm.dtype == torch.int32
    y_perm = torch.empty((A_cap, d), dtype=x.dtype, device=x.device) if out is None else out
    ws = _ws(workspace_bytes(STAGE_EXPERT_FFN, A_cap, d, E_local, 1, F, _dt(x)), x.device, ws)
    _check("c2r_expert_ffn_gather", lib().c2r_expert_ffn_gather(
        _ptr(x), _dt(x), _ptr(perm), T, K, _ptr(offsets), E_local, A_cap, d, F, _ptr(w_gate), _ptr(w_up), _ptr(w_down),
        _ptr(y_perm), _ptr(ws), ws.numel(), _stream()))
    return y_perm


def gather_fusable(dtype, d, F) -> bool:
    """Whether c2r_expert_ffn_gate_up_gather takes this shape (bf16, d and F multiples of 64)."""
    return dtype == torch.bfloat16 and d % 64 == 0 and F % 64 == 0


def expert_ffn_down(h, offsets, w_down, y_perm):
    """Second pass of the expert FFN: y_perm = h W_down^T."""
    A_cap, F = h.shape
    E_local, d, _ = w_down.shape
    assert y_perm.shape == (A_cap, d)
    _check("c2r_expert_ffn_down", lib().c2r_expert_ffn_down(
        _ptr(h), _dt(h), _ptr(offsets), E_local, A_cap, d, F, _ptr(w_down), _ptr(y_perm), _stream()))
    return y_perm


def expert_ffn_gate_up_with_shared(x, perm, K, offsets, w_gate, w_up, h, ws_gate, ws_up, h_shared):
    """First FFN pass of the routed groups (rows read through perm) and of the shared expert, one launch."""
    T, d = x.shape
    A_cap = perm.numel()
    E_local, F, _ = w_gate.shape
    Fs = ws_gate.shape[-2]
    assert h.shape == (A_cap, F) and h_shared.shape == (T, Fs) and perm.dtype == torch.int32
    assert ws_gate.shape[-1] == d and ws_up.shape[-2:] == (Fs, d)
    _check("c2r_expert_ffn_gate_up_with_shared", lib().c2r_expert_ffn_gate_up_with_shared(
        _ptr(x), _dt(x), _ptr(perm), T, K, _ptr(offsets), E_local, A_cap, d, F, _ptr(w_gate), _ptr(w_up), _ptr(h),
        Fs, _ptr(ws_gate), _ptr(ws_up), _ptr(h_shared), _stream()))
    return h, h_shared


def expert_ffn_down_with_shared(h, offsets, w_down, y_perm, h_shared, ws_down, y_shared):
    """Second FFN pass of the routed groups and of the shared expert, one launch."""
    A_cap, F = h.shape
    E_local, d, _ = w_down.shape
    T, Fs = h_shared.shape
    assert y_perm.shape == (A_cap, d) and y_shared.shape == (T, d) and ws_down.shape[-2:] == (d, Fs)
    _check("c2r_expert_ffn_down_with_shared", lib().c2r_expert_ffn_down_with_shared(
        _ptr(h), _dt(h), _ptr(offsets), E_local, A_cap, d, F, _ptr(w_down), _ptr(y_perm), T, Fs, _ptr(h_shared),
        _ptr(ws_down), _ptr(y_shared), _stream()))
    return y_perm, y_shared


def combine(y_perm, gates, inv_perm, y_shared=None, out=None):
    """Un-permute + gate-weighted sum.  Returns y[T, d]."""
    T, K = gates.shape
    d = y_perm.shape[1]
    y = torch.empty((T, d), dtype=y_perm.dtype, device=y_perm.device) if out is None else out
    _check("c2r_combine", lib().c2r_combine(_ptr(y_perm), _dt(y_perm), _ptr(gates), _ptr(inv_perm), T, d, K,
                                            _ptr(y_shared), _ptr(y), _stream()))
    return y


def place_experts(Cm, n_dev):
    """Sec. 3.4: greedy co-location of collaborating experts.  Returns int32[E] expert -> device."""
    E = Cm.shape[0]
    out = torch.empty((E,), dtype=torch.int32, device=Cm.device)
    _check("c2r_place_experts", lib().c2r_place_experts(_ptr(Cm), E, n_dev, _ptr(out), _stream()))
    return out


def dedup_dispatch(topk_idx, E, expert_device, n_dev, ws=None):
    """Sec. 3.4: one copy of a token per destination device.
    Returns (send_counts[n_dev], send_offsets[n_dev+1], send_token[T*K], send_row[T*K])."""
    T, K = topk_idx.shape
    dev = topk_idx.device
    i32 = dict(dtype=torch.int32, device=dev)
    counts, offsets = torch.empty((n_dev,), **i32), torch.empty((n_dev + 1,), **i32)
    tok, row = torch.full((T * K,), -1, **i32), torch.empty((T * K,), **i32)
    ws = _ws(workspace_bytes(STAGE_DEDUP_DISPATCH, T, 0, n_dev, K, 0, F32), dev, ws)
    _check("c2r_dedup_dispatch", lib().c2r_dedup_dispatch(_ptr(topk_idx), T, K, E, _ptr(expert_device), n_dev,
                                                        _ptr(counts), _ptr(offsets), _ptr(tok), _ptr(row),
                                                        _ptr(ws), ws.numel(), _stream()))
    return counts, offsets, tok, row


def combine_partial(y_perm, gates, inv_perm, send_token, send_row, send_offsets, y_part=None):
    """What an expert device returns: one gate-weighted partial row per token copy."""
    T, K = gates.shape
    d = y_perm.shape[1]
    if y_part is None:
        y_part = torch.empty((T * K, d), dtype=y_perm.dtype, device=y_perm.device)
    n_send = send_offsets[-1:]
    _check("c2r_combine_partial", lib().c2r_combine_partial(_ptr(y_perm), _dt(y_perm), _ptr(gates), _ptr(inv_perm),
                                                          _ptr(send_token), _ptr(send_row), _ptr(n_send), T,
                                                          y_part.shape[0], d, K, _ptr(y_part), _stream()))
    return y_part


def combine_copies(y_part, send_row, T, K, y_shared=None, out=None):
    """What the token's home device does: add the partial rows of its copies (+ shared)."""
    d = y_part.shape[1]
    y = torch.empty((T, d), dtype=y_part.dtype, device=y_part.device) if out is None else out
    _check("c2r_combine_copies", lib().c2r_combine_copies(_ptr(y_part), _dt(y_part), _ptr(send_row), T,
                                                        y_part.shape[0], d, K, _ptr(y_shared), _ptr(y), _stream()))
    return y


def collaboration_degree(Cm):
    """Eq. 3: fp64[E], the entropy of each expert's co-activation frequencies with the others."""
    E = Cm.shape[0]
    P = torch.empty((E,), dtype=torch.float64, device=Cm.device)
    _check("c2r_collaboration_degree", lib().c2r_collaboration_degree(_ptr(Cm), E, _ptr(P), _stream()))
    return P


def distinct_devices(topk_idx, E, expert_device, n_dev, per_token=False):
    """Sec. 4.1: for every row of expert_device (int32[n_maps, E] or int32[E]) the number of
    (token, device) copies a zero-redundancy dispatch sends.  Returns int64[n_maps] totals
    (and int32[n_maps, T] per-token counts if asked); redundancy = 1 - totals / (T*K)."""
    T, K = topk_idx.shape
    maps = expert_device.reshape(-1, E)
    n_maps = maps.shape[0]
    totals = torch.empty((n_maps,), dtype=torch.int64, device=topk_idx.device)
    pt = torch.empty((n_maps, T), dtype=torch.int32, device=topk_idx.device) if per_token else None
    _check("c2r_distinct_devices", lib().c2r_distinct_devices(_ptr(topk_idx), T, K, E, _ptr(maps), n_maps, n_dev,
                                                            _ptr(pt), _ptr(totals), _stream()))
    return (totals, pt) if per_token else totals


class C2RLayer:
    """One C2R MoE layer with all buffers allocated up front: forward() only
    enqueues the library's stages (no allocation, no host synchronisation).

    overlap=True (needs a shared always-on expert) spreads the work over two streams of
    default priority, because the shared expert needs neither the routing nor the dispatch:
        side stream : shared gate/up ........................ shared down
        main stream : route, permute | routed gate/up | routed down | combine
    Measured at the Qwen-MoE shape, clocks settled, this is 1.1 % faster than one stream (13 of
    the 72 us of route + permute are hidden: the router's fp32 FMAs and the GEMM's MFMAs share
    the SIMDs' issue slots, so most of what route and permute save, the shared gate/up pass
    beside them loses again).  The default is one stream: kernels that run alone can be timed."""

    def __init__(self, T, d, E, K, F, dtype, Wg, bias, collab_idx, w_gate, w_up, w_down,
                 local_slot=None, E_local=None, shared=None, device="cuda", fuse_gather=None, overlap=False,
                 fuse_shared=None):
        self.T, self.d, self.E, self.K, self.F = T, d, E, K, F
        self.E_local = E if E_local is None else E_local
        self.Wg, self.bias, self.collab_idx = Wg, bias, collab_idx
        self.w = (w_gate, w_up, w_down)
        self.local_slot, self.shared = local_slot, shared
        dev = device
        dt = F32 if dtype == torch.float32 else BF16
        i32 = dict(dtype=torch.int32, device=dev)
        self.idx = torch.empty((T, K), **i32)
        self.gates = torch.empty((T, K), dtype=torch.float32, device=dev)
        self.counts = torch.empty((self.E_local,), **i32)
        self.offsets = torch.empty((self.E_local + 1,), **i32)
        self.perm = torch.full((T * K,), -1, **i32)
        self.inv_perm = torch.empty((T * K,), **i32)
        # fold the dispatch's row gather into the first FFN pass when the shape allows it:
        # x_perm is then never written
        self.fuse_gather = gather_fusable(dtype, d, F) if fuse_gather is None else fuse_gather
        # ... or, when only F stands in the way (h needs a padded pitch), into c2r_expert_ffn_gather,
        # which runs both passes out of its workspace
        self.gather_both = (fuse_gather is None and not self.fuse_gather and dtype == torch.bfloat16
                            and d % 64 == 0 and T * d * 2 < (1 << 32))
        self.x_perm = None if self.fuse_gather or self.gather_both else torch.empty((T * K, d), dtype=dtype, device=dev)
        # the two FFN passes are enqueued as calls of their own when h needs no padded pitch
        # (then the layer owns h); otherwise c2r_expert_ffn runs both out of its workspace
        self.h = torch.empty((T * K, F), dtype=dtype, device=dev) if self.fuse_gather else None
        self.y_perm = torch.empty((T * K, d), dtype=dtype, device=dev)
        self.y = torch.empty((T, d), dtype=dtype, device=dev)
        u8 = dict(dtype=torch.uint8, device=dev)
        self.ws_route = torch.empty(max(256, workspace_bytes(STAGE_ROUTE, T, d, E, K, 0, dt)), **u8)
        self.ws_perm = torch.empty(max(256, workspace_bytes(STAGE_PERMUTE, T, d, E, K, 0, dt)), **u8)
        if not self.fuse_gather:
            self.ws_ffn = torch.empty(max(256, workspace_bytes(STAGE_EXPERT_FFN, T * K, d, self.E_local, 1, F, dt)), **u8)
        self.overlap = bool(overlap) and shared is not None
        if shared is not None:
            Fs = shared[0].shape[1]
            self.off_shared = torch.tensor([0, T], **i32)
            self.split_shared = gather_fusable(dtype, d, Fs)
            if self.split_shared:
                self.h_shared = torch.empty((T, Fs), dtype=dtype, device=dev)
            else:
                self.ws_shared = torch.empty(max(256, workspace_bytes(STAGE_EXPERT_FFN, T, d, 1, 1, Fs, dt)), **u8)
            self.y_shared = torch.empty((T, d), dtype=dtype, device=dev)
        else:
            self.y_shared = None
        # routed groups and shared expert in ONE launch per FFN pass (c2r_expert_ffn_*_with_shared):
        # the shared expert's uniform tiles fill the compute units that the ragged groups' last
        # tiles leave idle.  Needs the split, gather-fused form of both and a single stream.
        can_fuse_shared = (shared is not None and self.fuse_gather and self.split_shared and not self.overlap
                           and T * d * 2 < (1 << 32))
        self.fuse_shared = can_fuse_shared if fuse_shared is None else (bool(fuse_shared) and can_fuse_shared)
        if self.overlap:
            self.side = torch.cuda.Stream(device=dev)          # default priority
            self.ev = {k: torch.cuda.Event() for k in ("x", "shared_gate_up", "gate_up", "shared_down")}

    # names of the stages forward() may run, in the order a trace lists them
    STAGES = ("route", "permute", "ffn_gate_up", "ffn_down", "shared_gate_up", "shared_down", "combine")

    def stage_names(self):
        """The stages this layer's forward() runs (with fuse_shared the shared expert is part of
        ffn_gate_up and ffn_down)."""
        if self.shared is None or self.fuse_shared:
            return tuple(s for s in self.STAGES if not s.startswith("shared"))
        return self.STAGES

    def forward(self, x, trace=None, only=None):
        """y = layer(x).  trace: optional {stage: (start_event, end_event)} for any subset of
        STAGES; each pair is recorded on the stream its stage runs on (timing events, made by
        the caller).  only: run just that stage on the buffers a previous full call left
        (for timing a stage on its own)."""
        main = torch.cuda.current_stream()
        side = self.side if self.overlap else main

        def run(name, stream, fn):
            if only is not None and name != only:
                return
            pair = trace.get(name) if trace is not None else None
            with torch.cuda.stream(stream):
                if pair is not None:
                    pair[0].record(stream)
                fn()
                if pair is not None:
                    pair[1].record(stream)

        def gate_up():
            if self.fuse_shared:
                expert_ffn_gate_up_with_shared(x, self.perm, self.K, self.offsets, self.w[0], self.w[1], self.h,
                                               self.shared[0], self.shared[1], self.h_shared)
            elif self.fuse_gather:
                expert_ffn_gate_up_gather(x, self.perm, self.K, self.offsets, self.w[0], self.w[1], self.h)
            elif self.gather_both:   # both passes, rows read through perm
                expert_ffn_gather(x, self.perm, self.K, self.offsets, *self.w, ws=self.ws_ffn, out=self.y_perm)
            else:   # both passes
                expert_ffn(self.x_perm, self.offsets, *self.w, ws=self.ws_ffn, out=self.y_perm)

        def down():
            if self.fuse_shared:
                expert_ffn_down_with_shared(self.h, self.offsets, self.w[2], self.y_perm, self.h_shared,
                                            self.shared[2], self.y_shared)
            elif self.fuse_gather:
                expert_ffn_down(self.h, self.offsets, self.w[2], self.y_perm)

        def shared_gate_up():
            if self.split_shared:
                expert_ffn_gate_up(x, self.off_shared, self.shared[0], self.shared[1], self.h_shared)
            else:   # both passes
                expert_ffn(x, self.off_shared, *self.shared, ws=self.ws_shared, out=self.y_shared)

        def shared_down():
            if self.split_shared:
                expert_ffn_down(self.h_shared, self.off_shared, self.shared[2], self.y_shared)

        if self.overlap:
            self.ev["x"].record(main)                # x is ready, the previous call's combine has read y_shared
            side.wait_event(self.ev["x"])
        if self.shared is not None and not self.fuse_shared:
            run("shared_gate_up", side, shared_gate_up)
            if self.overlap:
                self.ev["shared_gate_up"].record(side)
        run("route", main, lambda: route(x, self.Wg, self.bias, self.K, self.collab_idx, ws=self.ws_route,
                                         out=(self.idx, self.gates)))
        run("permute", main, lambda: permute(x, self.idx, self.E, self.local_slot, self.E_local, ws=self.ws_perm,
                                             out=(self.counts, self.offsets, self.perm, self.inv_perm, self.x_perm)))
        if self.overlap:
            main.wait_event(self.ev["shared_gate_up"])
        run("ffn_gate_up", main, gate_up)
        if self.overlap:
            self.ev["gate_up"].record(main)
            side.wait_event(self.ev["gate_up"])
        if self.shared is not None and not self.fuse_shared:
            run("shared_down", side, shared_down)
            if self.overlap:
                self.ev["shared_down"].record(side)
        run("ffn_down", main, down)
        if self.overlap:
            main.wait_event(self.ev["shared_down"])
        run("combine", main, lambda: combine(self.y_perm, self.gates, self.inv_perm, self.y_shared, out=self.y))
        return self.y
