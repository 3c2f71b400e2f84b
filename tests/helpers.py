"""Shared plumbing of the GPU parity tests: host<->device copies and the
oracle-side pipeline.  No arithmetic of the method lives here."""
import numpy as np
import torch

from paper_2504_01337_amd import workloads as wl


def dev(a, dtype="f32"):
    """numpy -> cuda tensor in the given storage dtype (values already representable)."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32 and dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda()


def host(t):
    if t is None:
        return None
    t = t.detach()
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.cpu().numpy()


def max_rel_err(got, ref):
    """max |got - ref| / max |ref| : the error measure of the layer-output bar."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


TOL = {"f32": 1e-5, "bf16": 1e-2}


class OracleLayer:
    """The oracle's view of one workload: profiling -> lists -> routing -> dispatch."""

    def __init__(self, orc, w, x=None, x_prof=None):
        self.w = w
        self.Wg, self.bias = wl.router(w)
        self.x = wl.hidden(w) if x is None else x
        if w.T_profile:
            self.x_prof = wl.hidden(w, w.T_profile, stream=1) if x_prof is None else x_prof
        else:
            self.x_prof = self.x
        lp = orc.logits_canon_f32(self.x_prof, self.Wg, self.bias)
        self.idx_prof, _ = orc.route(lp, w.K)
        self.C = orc.coactivation(self.idx_prof, w.E)
        self.collab = orc.collaborators(self.C, w.Tc)
        self.logits = lp if self.x_prof is self.x else orc.logits_canon_f32(self.x, self.Wg, self.bias)
        self.idx, self.gates = orc.route(self.logits, w.K, self.collab)
        self.local_slot = wl.local_slot(w)
        self.counts, self.offsets, self.perm, self.inv_perm = orc.permute(
            self.idx, w.E, self.local_slot, w.n_local)
