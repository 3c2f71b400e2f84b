"""GPU parity of the whole layer at the five workloads, in the launch
configuration the benchmark times: profiling -> collaborator lists -> route ->
permute -> expert FFN -> combine, each compared with the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2504_01337_amd import workloads as wl
from helpers import GATE_RTOL, OracleLayer, ROW_TOL, SHARE_OUTSIDE_MAX, TOL, dev, host, max_rel_err, share_outside

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c2r():
    from paper_2504_01337_amd import c2r as m
    m.lib()
    return m


def _run_layer(c2r, orc, w, n_sample):
    print(f"[layer] {w.name} T={w.T} d={w.d} E={w.E} F={w.F} K={w.K} Tc={w.Tc} {w.dtype}", flush=True)
    o = OracleLayer(orc, w)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    Wg, bias = dev(o.Wg), dev(o.bias)
    # --- profiling on the GPU: conventional top-K -> Eq. 2 -> Eq. 4 ---
    idx_p, _, _ = c2r.route(dev(o.x_prof, w.dtype), Wg, bias, w.K, None)
    assert np.array_equal(host(idx_p), o.idx_prof)
    Cm = c2r.build_coactivation(idx_p, w.E)
    assert np.array_equal(host(Cm).astype(np.int64), o.C)
    collab, _ = c2r.collaborators(Cm, w.Tc)
    assert np.array_equal(host(collab), o.collab)
    # --- the layer ---
    wg, wu, wd = wl.expert_weights(w)
    shared = wl.shared_expert_weights(w) if w.F_shared else None
    layer = c2r.C2RLayer(w.T, w.d, w.E, w.K, w.F, tdt, Wg, bias, collab,
                         dev(wg, w.dtype), dev(wu, w.dtype), dev(wd, w.dtype),
                         local_slot=dev(o.local_slot), E_local=w.n_local,
                         shared=None if shared is None else tuple(dev(a, w.dtype) for a in shared))
    x = dev(o.x, w.dtype)
    y = layer.forward(x)
    y = layer.forward(x)            # twice: buffers are reused, the result must not depend on it
    torch.cuda.synchronize()
    if layer.fuse_gather or layer.gather_both:
        # the same layer through c2r_permute's x_perm and c2r_expert_ffn, and with the shared
        # expert (if any) on a second stream: identical bits
        plain = c2r.C2RLayer(w.T, w.d, w.E, w.K, w.F, tdt, Wg, bias, collab, *layer.w,
                             local_slot=layer.local_slot, E_local=w.n_local, shared=layer.shared,
                             fuse_gather=False, overlap=True)
        y_plain = plain.forward(x)
        torch.cuda.synchronize()
        assert torch.equal(y_plain, y)
        assert torch.equal(plain.perm[: int(o.offsets[-1])], layer.perm[: int(o.offsets[-1])])
        x_perm_dev = plain.x_perm
    else:
        x_perm_dev = layer.x_perm
    assert np.array_equal(host(layer.idx), o.idx)
    np.testing.assert_allclose(host(layer.gates), o.gates, rtol=GATE_RTOL, atol=1e-7)
    assert np.array_equal(host(layer.counts), o.counts)
    assert np.array_equal(host(layer.offsets), o.offsets)
    n = int(o.offsets[-1])
    assert np.array_equal(host(layer.perm)[:n], o.perm)
    assert np.array_equal(host(layer.inv_perm), o.inv_perm)
    assert np.array_equal(host(x_perm_dev)[:n], o.x[o.perm // w.K])
    # --- outputs: every token of the batch (n_sample None) or sampled tokens, which the oracle
    #     computes one by one; two measures: max |d| / max |ref| and the share of elements
    #     with |d| > tol * (|ref| + rms(ref)) ---
    if n_sample is None or n_sample >= w.T:
        toks = np.arange(w.T)
    else:
        toks = np.sort(np.random.default_rng(w.cfg_id).permutation(w.T)[:n_sample])
    ref = orc.layer_tokens(o.x, toks, o.idx, o.gates, wg, wu, wd, w.E, o.local_slot, shared)
    got = host(y)[toks]
    err = max_rel_err(got, ref)
    share = share_outside(got, ref, TOL[w.dtype])
    # the worst token (row) by its own scale, for the report
    row_err = np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-30)
    print(f"[layer] {w.name} {len(toks)} tokens: max rel err {err:.3e} (bar {TOL[w.dtype]}); share of elements "
          f"outside tol*(|ref|+rms) {share:.2e} (bar {SHARE_OUTSIDE_MAX[w.dtype]}); worst row by its own "
          f"max {np.nanmax(row_err):.3e}", flush=True)
    assert err <= TOL[w.dtype]
    assert share <= SHARE_OUTSIDE_MAX[w.dtype]
    assert np.nanmax(row_err) <= ROW_TOL[w.dtype]
    assert torch.isfinite(y.float()).all()
    layer.Cm = Cm
    return layer, o


def test_layer_c1_full(c2r, orc):
    w = wl.WORKLOADS["C1"]
    _run_layer(c2r, orc, w, n_sample=w.T)


@pytest.mark.parametrize("name,T,Tp", [("C2", 1500, 4096), ("C3", 1111, 4096), ("C5", 2047, 4096)])
def test_layer_reduced(c2r, orc, name, T, Tp):
    _run_layer(c2r, orc, wl.scaled(wl.WORKLOADS[name], T=T, T_profile=Tp), n_sample=96)


@pytest.mark.parametrize("name", ["C2", "C3", "C5"])
def test_layer_full_size(c2r, orc, name):
    w = wl.WORKLOADS[name]
    layer, o = _run_layer(c2r, orc, w, n_sample=None)    # every token of the batch
    if name in ("C3", "C5"):
        # Sec. 3.4 at full size: the zero-redundancy send list under a fixed 4-way contiguous map
        # (bit exact), its copy count against the host-side count of distinct devices, and the
        # two-level combine against the layer's own output
        dm = wl.device_map(w.E, 4)
        Cm = layer.Cm
        counts, offsets, tok, row = c2r.dedup_dispatch(layer.idx, w.E, dev(dm), 4)
        rc, ro, rt, rr = orc.dedup_dispatch(o.idx, w.E, dm, 4)
        n = int(ro[-1])
        assert np.array_equal(host(offsets), ro) and np.array_equal(host(tok)[:n], rt) and np.array_equal(host(row), rr)
        dd = orc.distinct_devices(o.idx, dm)
        assert n == int(dd.sum())
        idx_topk, _ = orc.route(o.logits, w.K)
        print("[layer] %s copies sent per token (4 devices): C2R %.3f, top-K %.3f; redundancy %.3f vs %.3f" % (
            name, dd.mean(), orc.distinct_devices(idx_topk, dm).mean(), orc.redundancy(dd, w.K),
            orc.redundancy(orc.distinct_devices(idx_topk, dm), w.K)), flush=True)
        # the same with experts co-located by their profiled co-activation (Sec. 3.4)
        placed = c2r.place_experts(Cm, 4)
        pm = orc.place_experts(o.C, 4)
        assert np.array_equal(host(placed), pm)
        _, poff, _, _ = c2r.dedup_dispatch(layer.idx, w.E, placed, 4)
        pd, pdk = orc.distinct_devices(o.idx, pm), orc.distinct_devices(idx_topk, pm)
        assert int(poff[-1].item()) == int(pd.sum())
        print("[layer] %s with co-located experts: C2R %.3f copies/token (redundancy %.3f), top-K %.3f (%.3f)" % (
            name, pd.mean(), orc.redundancy(pd, w.K), pdk.mean(), orc.redundancy(pdk, w.K)), flush=True)
        part = c2r.combine_partial(layer.y_perm, layer.gates, layer.inv_perm, tok, row, offsets)
        y2 = c2r.combine_copies(part, row, w.T, w.K, layer.y_shared)
        torch.cuda.synchronize()
        ref = host(layer.y)
        assert np.abs(host(y2) - ref).max() <= 2.0 ** -7 * np.abs(ref).max()   # one more rounding than c2r_combine


def test_layer_llama_moe_shape_and_list_length_sweep(c2r, orc):
    """The paper's LLaMA-MoE setting (Sec. 4.1) end to end, then Fig. 3's axes on the same
    kernels: collaborator lists of every length 1..E-1 (E-1 = conventional top-K) and the
    random-list variant, routing compared bit for bit."""
    w = wl.WORKLOADS["L1"]
    layer, o = _run_layer(c2r, orc, w, n_sample=64)
    x, Wg, bias = dev(o.x, w.dtype), dev(o.Wg), dev(o.bias)
    topk, gk = orc.route(o.logits, w.K)
    rng = np.random.default_rng(61)
    for Tc in range(1, w.E):
        lists = orc.collaborators(o.C, Tc)
        rand = np.stack([rng.permutation([j for j in range(w.E) if j != i])[:Tc] for i in range(w.E)]).astype(np.int32)
        for ci in (lists, rand):
            idx, g, _ = c2r.route(x, Wg, bias, w.K, dev(ci))
            ri, rg = orc.route(o.logits, w.K, ci)
            assert np.array_equal(host(idx), ri), Tc
            np.testing.assert_allclose(host(g), rg, rtol=GATE_RTOL, atol=1e-7)
            if Tc == 1:                                    # Fig. 3, T = 1: the partner is the list entry
                assert np.array_equal(ri[:, 1], ci[ri[:, 0], 0])
            if Tc == w.E - 1:                              # Fig. 3 caption: degenerates to top-K
                assert np.array_equal(ri, topk)


def test_profiling_c4_full_size(c2r, orc):
    # 2^20 tokens: stored fp32 logits -> top-4 -> co-activation counts -> top-16 lists
    w = wl.WORKLOADS["C4"]
    logits = wl.direct_logits(w)
    lg = dev(logits)
    idx, gates = c2r.route_from_logits(lg, w.K, None)
    Cm = c2r.build_coactivation(idx, w.E)
    collab, _ = c2r.collaborators(Cm, w.Tc)
    torch.cuda.synchronize()
    idx_ref, g_ref = orc.route(logits, w.K)
    assert np.array_equal(host(idx), idx_ref)
    C_ref = orc.coactivation(idx_ref, w.E)
    assert np.array_equal(host(Cm).astype(np.int64), C_ref)
    assert np.array_equal(host(collab), orc.collaborators(C_ref, w.Tc))
    sel = np.random.default_rng(4).permutation(w.T)[:4096]
    np.testing.assert_allclose(host(gates)[sel], g_ref[sel], rtol=GATE_RTOL, atol=1e-7)
    # the one-launch form (selection and counts; the selections not written), as bench.py times it,
    # then once more with the selections written, adding to the same matrix
    Cf = torch.zeros_like(Cm)
    c2r.profile_from_logits(lg, w.K, Cf)
    assert np.array_equal(host(Cf).astype(np.int64), C_ref)
    _, idx2, gates2 = c2r.profile_from_logits(lg, w.K, Cf, want_selection=True)
    assert np.array_equal(host(Cf).astype(np.int64), 2 * C_ref)
    assert torch.equal(idx2, idx) and torch.equal(gates2, gates)


def test_layer_forward_in_a_captured_graph(c2r, orc):
    """The library allocates nothing, synchronises nothing and records no memset: a forward
    captured in a graph replays to the eager result, every time, with eager work in between."""
    w = wl.scaled(wl.WORKLOADS["C3"], T=1024, T_profile=2048)
    o = OracleLayer(orc, w)
    wg, wu, wd = wl.expert_weights(w)
    shared = wl.shared_expert_weights(w)
    layer = c2r.C2RLayer(w.T, w.d, w.E, w.K, w.F, torch.bfloat16, dev(o.Wg), dev(o.bias), dev(o.collab),
                         dev(wg, "bf16"), dev(wu, "bf16"), dev(wd, "bf16"), local_slot=dev(o.local_slot),
                         E_local=w.n_local, shared=tuple(dev(a, "bf16") for a in shared))
    x = dev(o.x, "bf16")
    y_eager = layer.forward(x).clone()
    idx_eager = layer.idx.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer.forward(x)                                   # warm-up on the capture stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            layer.forward(x)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for i in range(4):
        layer.y.zero_()
        layer.idx.fill_(-7)
        layer.h.fill_(float("nan"))                       # stale scratch must not leak into a replay
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(layer.idx, idx_eager), i
        assert torch.equal(layer.y, y_eager), i
        y2 = layer.forward(x)                              # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(y2, y_eager)
