"""Seeded synthetic inputs for the C2R MoE layer (shapes of Sec. 4.1 of the paper).

This module only draws random numbers and rounds them to the storage dtype.  It
holds none of the method's arithmetic (no routing, no counting, no expert
compute) so that the CPU oracle and the HIP path can both be fed from it without
sharing any code of the method itself.  Everything is generated on the host with
numpy; nothing here touches a GPU.

The five workloads ("C1".."C5") stand in for the paper's WikiText / LongBench
token streams and fine-tuned LLaMA-MoE / Qwen1.5-MoE weights, none of which are
available offline:

* hidden states  x ~ N(0, 1)
* router weight  W_g[k, e] ~ N(0, 0.02) plus a planted group direction
  u_{grp(e)} ~ N(0, I/d) shared by the experts of a contiguous block, so that
  experts of one block co-activate more often (the structure Sec. 3.2 profiles)
* optional Zipf(s=1.1) per-expert logit offsets to skew the expert load
* expert weights ~ N(0, 0.02)
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

SEED_BASE = 20250401


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    T: int                  # tokens in the timed / checked batch
    d: int                  # model width
    E: int                  # experts per layer (the paper's N)
    F: int                  # expert intermediate width (0: routing-only workload)
    K: int                  # experts per token
    Tc: int                 # collaborator-list length (the paper's T)
    dtype: str              # "f32" | "bf16": activations and expert weights
    groups: int             # planted co-activation blocks in the router
    zipf: bool = False      # Zipf(1.1) per-expert logit offsets
    F_shared: int = 0       # always-on shared expert width (Qwen), 0 = none
    E_local: int = 0        # experts held by this device (0 = all)
    T_profile: int = 0      # separate profiling tokens (0 = profile on the batch)
    cfg_id: int = 0

    @property
    def n_local(self) -> int:
        return self.E_local if self.E_local else self.E


WORKLOADS = {
    "C1": Workload("C1", T=512, d=256, E=8, F=512, K=2, Tc=4, dtype="f32", groups=2, cfg_id=1),
    "C2": Workload("C2", T=4096, d=4096, E=16, F=688, K=4, Tc=8, dtype="bf16", groups=4,
                   T_profile=65536, cfg_id=2),
    "C3": Workload("C3", T=8192, d=2048, E=60, F=1408, K=4, Tc=16, dtype="bf16", groups=6,
                   zipf=True, F_shared=5632, T_profile=65536, cfg_id=3),
    "C4": Workload("C4", T=1048576, d=2048, E=60, F=0, K=4, Tc=16, dtype="f32", groups=6, cfg_id=4),
    "C5": Workload("C5", T=32768, d=2048, E=60, F=1408, K=4, Tc=16, dtype="bf16", groups=6,
                   zipf=True, E_local=15, T_profile=65536, cfg_id=5),
    # the paper's own LLaMA-MoE setting (Sec. 4.1: 8 experts, top-2, intermediate width 1376,
    # collaborator lists of 5), as a second shape for the list-length sweep of Fig. 3
    "L1": Workload("L1", T=2048, d=4096, E=8, F=1376, K=2, Tc=5, dtype="bf16", groups=2,
                   T_profile=8192, cfg_id=6),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some sizes replaced (reduced-size parity cases)."""
    return dataclasses.replace(w, **kw)


def _rng(w: Workload, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng(SEED_BASE + 1000 * w.cfg_id + tensor_id)


def round_bf16_reference(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32 (bit twiddling)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Same rounding through torch's multi-threaded CPU cast (finite inputs)."""
    import torch
    a = np.ascontiguousarray(a, dtype=np.float32)
    return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values that are already bf16-representable."""
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a = a.astype(np.float32, copy=False)
    return round_bf16(a) if dtype == "bf16" else a


def _normal(rng, shape, scale=1.0):
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        out *= np.float32(scale)
    return out


def hidden(w: Workload, n: Optional[int] = None, stream: int = 0) -> np.ndarray:
    """x[n, d] ~ N(0,1) in the workload's storage dtype (returned as fp32 values)."""
    n = w.T if n is None else n
    return _store(_normal(_rng(w, 10 + stream), (n, w.d)), w.dtype)


def router(w: Workload):
    """(W_g[d, E] fp32, bias[E] fp32 or None): the layout of x . W_g in Eq. 1."""
    Wg = _normal(_rng(w, 1), (w.d, w.E), 0.02)
    if w.groups > 0:
        u = _normal(_rng(w, 2), (w.groups, w.d), 1.0 / np.sqrt(w.d))
        per = -(-w.E // w.groups)
        for e in range(w.E):
            Wg[:, e] += u[min(e // per, w.groups - 1)]
    bias = None
    if w.zipf:
        ranks = _rng(w, 3).permutation(w.E) + 1
        lp = -1.1 * np.log(ranks.astype(np.float64))
        bias = (lp - lp.mean()).astype(np.float32)
    return np.ascontiguousarray(Wg), bias


def expert_weights(w: Workload, n_experts: Optional[int] = None, F: Optional[int] = None,
                   stream: int = 0):
    """(w_gate[E,F,d], w_up[E,F,d], w_down[E,d,F]) ~ N(0, 0.02) in the storage dtype."""
    n = w.n_local if n_experts is None else n_experts
    F = w.F if F is None else F
    rng = _rng(w, 20 + stream)
    wg = _store(_normal(rng, (n, F, w.d), 0.02), w.dtype)
    wu = _store(_normal(rng, (n, F, w.d), 0.02), w.dtype)
    wd = _store(_normal(rng, (n, w.d, F), 0.02), w.dtype)
    return wg, wu, wd


def shared_expert_weights(w: Workload):
    assert w.F_shared > 0
    return expert_weights(w, n_experts=1, F=w.F_shared, stream=5)


def local_slot(w: Workload) -> Optional[np.ndarray]:
    """int32[E]: position of expert e among this device's experts, or -1.

    A fixed contiguous expert-to-device map (device 0 holds experts 0..E_local-1)."""
    if not w.E_local:
        return None
    ls = np.full(w.E, -1, dtype=np.int32)
    ls[: w.E_local] = np.arange(w.E_local, dtype=np.int32)
    return ls


def device_map(E: int, ep: int) -> np.ndarray:
    """int32[E]: contiguous expert-to-device map for an expert-parallel degree ep."""
    per = -(-E // ep)
    return (np.arange(E) // per).astype(np.int32)


def direct_logits(w: Workload, n: Optional[int] = None, chunk: int = 65536) -> np.ndarray:
    """fp32 logits[n, E] with the same joint law as x . W_g of `router(w)` for
    Gaussian x, drawn directly: a shared N(0,1) term per planted block plus
    N(0, 0.02^2 d) private noise per expert.  Used by the profiling-only workload
    whose 2^20 x 2048 hidden states would be wasteful to materialise."""
    n = w.T if n is None else n
    rng = _rng(w, 30)
    per = -(-w.E // w.groups)
    grp = np.minimum(np.arange(w.E) // per, w.groups - 1)
    sigma = np.float32(0.02 * np.sqrt(w.d))
    out = np.empty((n, w.E), dtype=np.float32)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        z = rng.standard_normal(size=(m, w.groups), dtype=np.float32)
        noise = rng.standard_normal(size=(m, w.E), dtype=np.float32)
        out[s:s + m] = z[:, grp] + sigma * noise
    return out


def exact_arithmetic_router(T: int, d: int, E: int, seed: int = 7):
    """Tie-stress inputs on which fp32 dot products are exact in any summation
    order: x integer in [-4, 4] (exact in bf16), W_g multiples of 1/8 in [-1, 1].
    Every partial sum is a multiple of 1/8 below 2^14 for d <= 4096, so it fits
    fp32's 24-bit significand; equal logits are frequent by construction."""
    assert d <= 4096
    rng = np.random.default_rng(SEED_BASE + 900000 + seed)
    x = rng.integers(-4, 5, size=(T, d)).astype(np.float32)
    Wg = (rng.integers(-8, 9, size=(d, E)).astype(np.float32)) / np.float32(8.0)
    return x, Wg
