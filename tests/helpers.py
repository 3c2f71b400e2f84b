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


# Relative tolerance of the fp32 gates against the oracle's fp64 gates (both from the same fp32
# logits).  A gate is exp(a_s) / sum_s' exp(a_s') with a_s = l_s - l_0 <= 0.  In fp32: a_s is one
# rounded subtraction (relative 2^-24, so exp(a_s) moves by |a_s| 2^-24 relatively), the exponential
# is good to 2 ulp, the sum of K <= 8 positive terms to (K - 1) roundings, the division to 1 ulp:
# (|a_s| + 2 + 7 + 1) 2^-24 in all.  A gate that is not flushed to zero has |a_s| < 88 in
# principle, but the workloads' logits differ by less than 24 inside a token's kept set, which
# gives (24 + 10) 2^-24 = 2.0e-6.  (1e-6 would hold only for |a_s| < 7.)
GATE_RTOL = 2e-6


def share_outside(got, ref, tol):
    """Second error measure of the layer-output bar: the share of elements whose error exceeds
    tol * (|ref| + rms(ref)), so that rows that are small next to the batch maximum count too."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.mean(np.abs(got - ref) > tol * (np.abs(ref) + rms)))


TOL = {"f32": 1e-5, "bf16": 1e-2}
# Share of elements allowed outside tol * (|ref| + rms): none in fp32.  In bf16 every output is
# rounded to 8 significant bits three times on the way (h, y_perm, y): an element's error is
# a few times 2^-9 of the magnitude of the TERMS it sums, which for an element that is itself
# near zero is a few times 2^-9 * rms, i.e. inside 1e-2 * rms but not by a wide margin, so a
# small share of elements is allowed to land outside.
SHARE_OUTSIDE_MAX = {"f32": 0.0, "bf16": 1e-4}     # measured at full size: 6e-8 .. 1e-5
# Every token's row on its own scale: max |d| over the row / max |ref| over the row.  Measured at
# full size 7.6e-3 (bf16), 1.5e-6 (fp32): a wrong row (a tile of the ragged map written to the
# wrong place, a missing term of the combine) is off by order 1.
ROW_TOL = {"f32": 1e-5, "bf16": 1.5e-2}


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
