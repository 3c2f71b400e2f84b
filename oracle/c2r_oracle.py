"""ctypes front end of the CPU oracle (oracle/c2r_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg.  It marshals numpy arrays and nothing else; all arithmetic is
in the C file.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_route.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


CANON_CHUNK = 256   # the library's declared k-chunk length (stated in include/c2r.h)


def logits_f64(x, Wg, bias=None):
    x, Wg, bias = _f32(x), _f32(Wg), _f32(bias)
    T, d = x.shape
    E = Wg.shape[1]
    out = np.empty((T, E), dtype=np.float64)
    lib().orc_logits_f64(_p(x), _p(Wg), _p(bias), C.c_int64(T), d, E, _p(out))
    return out


def logits_canon_f32(x, Wg, bias=None, chunk=CANON_CHUNK):
    x, Wg, bias = _f32(x), _f32(Wg), _f32(bias)
    T, d = x.shape
    E = Wg.shape[1]
    out = np.empty((T, E), dtype=np.float32)
    lib().orc_logits_canon_f32(_p(x), _p(Wg), _p(bias), C.c_int64(T), d, E, int(chunk), _p(out))
    return out


def route(logits, K, collab_idx=None):
    """(topk_idx int32[T,K], gates f64[T,K]); collab_idx=None is conventional top-K."""
    logits = _f32(logits)
    T, E = logits.shape
    ci = _i32(collab_idx)
    Tc = 0 if ci is None else ci.shape[1]
    idx = np.empty((T, K), dtype=np.int32)
    gates = np.empty((T, K), dtype=np.float64)
    rc = lib().orc_route(_p(logits), C.c_int64(T), E, K, _p(ci), Tc, _p(idx), _p(gates))
    if rc != 0:
        raise ValueError("collaborator list too short for K-1 distinct experts")
    return idx, gates


def coactivation(topk_idx, E, C_in=None):
    idx = _i32(topk_idx)
    T, K = idx.shape
    Cm = np.zeros((E, E), dtype=np.int64) if C_in is None else np.ascontiguousarray(C_in, dtype=np.int64).copy()
    lib().orc_coactivation(_p(idx), C.c_int64(T), K, E, _p(Cm))
    return Cm


def collaborators(Cm, Tc):
    Cm = np.ascontiguousarray(Cm, dtype=np.int64)
    E = Cm.shape[0]
    n = min(Tc, E - 1)
    out = np.empty((E, n), dtype=np.int32)
    lib().orc_collaborators(_p(Cm), E, int(Tc), _p(out))
    return out


def permute(topk_idx, E, local_slot=None, E_local=None):
    idx = _i32(topk_idx)
    T, K = idx.shape
    ls = _i32(local_slot)
    E_local = E if E_local is None else E_local
    counts = np.empty(E_local, dtype=np.int32)
    offsets = np.empty(E_local + 1, dtype=np.int32)
    perm = np.full(T * K, -1, dtype=np.int32)
    inv = np.empty(T * K, dtype=np.int32)
    lib().orc_permute(_p(idx), C.c_int64(T), K, E, _p(ls), E_local, _p(counts), _p(offsets), _p(perm), _p(inv))
    return counts, offsets, perm[: offsets[-1]].copy(), inv


def expert_ffn_rows(x_rows, expert_of_row, w_gate, w_up, w_down):
    x_rows = _f32(x_rows)
    n, d = x_rows.shape
    F = w_gate.shape[1]
    eo = _i32(expert_of_row)
    wg, wu, wd = _f32(w_gate), _f32(w_up), _f32(w_down)
    y = np.empty((n, d), dtype=np.float64)
    lib().orc_expert_ffn_rows(_p(x_rows), _p(eo), C.c_int64(n), d, F, _p(wg), _p(wu), _p(wd), _p(y))
    return y


def layer_tokens(x, tokens, topk_idx, gates, w_gate, w_up, w_down, E, local_slot=None, shared=None):
    """fp64 layer output y[len(tokens), d] for the listed tokens."""
    x = _f32(x)
    d = x.shape[1]
    tokens = np.ascontiguousarray(tokens, dtype=np.int64)
    idx = _i32(topk_idx)
    K = idx.shape[1]
    g = np.ascontiguousarray(gates, dtype=np.float64)
    wg, wu, wd = _f32(w_gate), _f32(w_up), _f32(w_down)
    F = wg.shape[1]
    ls = _i32(local_slot)
    if shared is not None:
        sg, su, sd = (_f32(a) for a in shared)
        Fs = sg.shape[-2]
    else:
        sg = su = sd = None
        Fs = 0
    y = np.empty((len(tokens), d), dtype=np.float64)
    lib().orc_layer_tokens(_p(x), _p(tokens), C.c_int64(len(tokens)), d, E, K, F, _p(idx), _p(g), _p(ls),
                           _p(wg), _p(wu), _p(wd), Fs, _p(sg), _p(su), _p(sd), _p(y))
    return y


def combine(y_perm, gates, inv_perm, T, K, y_shared=None):
    yp = np.ascontiguousarray(y_perm, dtype=np.float64)
    d = yp.shape[1]
    g = np.ascontiguousarray(gates, dtype=np.float64)
    inv = _i32(inv_perm)
    ys = None if y_shared is None else np.ascontiguousarray(y_shared, dtype=np.float64)
    y = np.empty((T, d), dtype=np.float64)
    lib().orc_combine(_p(yp), _p(g), _p(inv), C.c_int64(T), d, K, _p(ys), _p(y))
    return y


def distinct_devices(topk_idx, dev_of_expert):
    idx = _i32(topk_idx)
    T, K = idx.shape
    dev = _i32(dev_of_expert)
    out = np.empty(T, dtype=np.int32)
    lib().orc_distinct_devices(_p(idx), C.c_int64(T), K, _p(dev), _p(out))
    return out


# ---- host-side metrics of Sec. 3.2 / Sec. 4.1 (plain numpy, fp64) ----

def collaboration_degree(Cm):
    """Eq. 3: entropy of each expert's co-activation frequencies with the others
    (diagonal left out of both the sum and the normalisation; natural log)."""
    Cm = np.asarray(Cm, dtype=np.float64).copy()
    np.fill_diagonal(Cm, 0.0)
    P = np.zeros(Cm.shape[0])
    for i in range(Cm.shape[0]):
        s = Cm[i].sum()
        if s <= 0:
            continue
        p = Cm[i] / s
        nz = p > 0
        P[i] = -(p[nz] * np.log(p[nz])).sum()
    return P


def redundancy(distinct, K):
    """Share of (token, expert) copies a zero-redundancy dispatch does not send."""
    distinct = np.asarray(distinct, dtype=np.float64)
    return 1.0 - distinct.sum() / (distinct.size * K)


def estimated_speedup(all_to_all_share, redundancy_share):
    """Sec. 4.1: estimated speed-up = all-to-all time share x token redundancy."""
    return all_to_all_share * redundancy_share


# ---- Sec. 3.4: zero-redundancy dispatch (one copy of a token per destination device) ----

def dedup_dispatch(topk_idx, E, dev_of_expert, n_dev):
    """Returns (send_counts[n_dev], send_offsets[n_dev+1], send_token[n_send], send_row[T*K])."""
    idx = _i32(topk_idx)
    T, K = idx.shape
    dev = _i32(dev_of_expert)
    counts = np.empty(n_dev, dtype=np.int32)
    offsets = np.empty(n_dev + 1, dtype=np.int32)
    tok = np.empty(T * K, dtype=np.int32)
    row = np.empty(T * K, dtype=np.int32)
    lib().orc_dedup_dispatch.restype = C.c_int64
    n = lib().orc_dedup_dispatch(_p(idx), C.c_int64(T), K, E, _p(dev), n_dev, _p(counts), _p(offsets), _p(tok), _p(row))
    return counts, offsets, tok[:n].copy(), row


def combine_partial(y_perm, gates, inv_perm, send_row, T, K, n_send):
    yp = np.ascontiguousarray(y_perm, dtype=np.float64)
    d = yp.shape[1]
    g = np.ascontiguousarray(gates, dtype=np.float64)
    out = np.empty((n_send, d), dtype=np.float64)
    lib().orc_combine_partial(_p(yp), _p(g), _p(_i32(inv_perm)), _p(_i32(send_row)), C.c_int64(T), d, K,
                              C.c_int64(n_send), _p(out))
    return out


def combine_copies(y_part, send_row, T, K, y_shared=None):
    yp = np.ascontiguousarray(y_part, dtype=np.float64)
    d = yp.shape[1]
    ys = None if y_shared is None else np.ascontiguousarray(y_shared, dtype=np.float64)
    y = np.empty((T, d), dtype=np.float64)
    lib().orc_combine_copies(_p(yp), _p(_i32(send_row)), C.c_int64(T), d, K, _p(ys), _p(y))
    return y


def place_experts(Cm, n_dev):
    """Greedy co-location of collaborating experts (Sec. 3.4).  Returns int32[E] expert -> device."""
    Cm = np.ascontiguousarray(Cm, dtype=np.int64)
    E = Cm.shape[0]
    out = np.empty(E, dtype=np.int32)
    lib().orc_place_experts(_p(Cm), E, n_dev, _p(out))
    return out
