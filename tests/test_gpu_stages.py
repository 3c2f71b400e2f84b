"""GPU parity, stage by stage: every entry point of the C ABI against the CPU
oracle on the same seeded inputs.  Integer results are compared bit for bit."""
import numpy as np
import pytest
import torch

from paper_2504_01337_amd import workloads as wl
from helpers import GATE_RTOL, dev, host, max_rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c2r():
    from paper_2504_01337_amd import c2r as m
    m.lib()
    assert torch.cuda.is_available()
    return m


def _collab(E, Tc, seed):
    rng = np.random.default_rng(seed)
    out = np.empty((E, Tc), dtype=np.int32)
    for i in range(E):
        others = np.array([j for j in range(E) if j != i])
        out[i] = rng.permutation(others)[:Tc]
    return out


def _check_route(c2r, orc, x, Wg, bias, K, collab, dtype, bit_exact_logits=True):
    idx, gates, logits = c2r.route(dev(x, dtype), dev(Wg), dev(bias), K,
                                   None if collab is None else dev(collab), want_logits=True)
    torch.cuda.synchronize()
    l_ref = orc.logits_canon_f32(x, Wg, bias)
    l_gpu = host(logits)
    if bit_exact_logits:
        assert np.array_equal(l_gpu.view(np.uint32), l_ref.view(np.uint32)), \
            f"logit bits differ in {(l_gpu != l_ref).sum()} places"
    idx_ref, g_ref = orc.route(l_gpu, K, collab)          # stage-wise: the GPU's own logits
    assert np.array_equal(host(idx), idx_ref)
    np.testing.assert_allclose(host(gates), g_ref, rtol=GATE_RTOL, atol=1e-7)
    l64 = orc.logits_f64(x, Wg, bias)
    assert np.abs(l_gpu - l64).max() <= 1e-5 * max(np.abs(l64).max(), 1.0)
    return host(idx)


@pytest.mark.parametrize("name,T", [("C1", 512), ("C2", 700), ("C3", 1000), ("C5", 333)])
def test_route_workload_shapes(c2r, orc, name, T):
    w = wl.scaled(wl.WORKLOADS[name], T=T)
    x = wl.hidden(w)
    Wg, bias = wl.router(w)
    collab = _collab(w.E, w.Tc, 1)
    _check_route(c2r, orc, x, Wg, bias, w.K, collab, w.dtype)
    _check_route(c2r, orc, x, Wg, bias, w.K, None, w.dtype)            # conventional top-K


@pytest.mark.parametrize("E,K,Tc,d,T,dtype", [
    (8, 2, 4, 256, 512, "f32"), (60, 4, 16, 2048, 777, "bf16"), (64, 8, 20, 512, 130, "bf16"),
    (5, 2, 3, 64, 65, "f32"), (13, 13, 12, 136, 1, "bf16"), (7, 1, 0, 264, 63, "bf16"),
    (33, 3, 2, 1000, 257, "f32")])
def test_route_exact_arithmetic_ties(c2r, orc, E, K, Tc, d, T, dtype):
    # integer / dyadic inputs: logits exact in any order, ties frequent -> tie rule and masks
    x, Wg = wl.exact_arithmetic_router(T, d, E, seed=E + K)
    collab = _collab(E, Tc, 2) if Tc > 0 else None
    idx = _check_route(c2r, orc, x, Wg, None, K, collab, dtype)
    exact = (x.astype(np.int64) @ np.round(Wg * 8).astype(np.int64)).astype(np.float64) / 8.0
    l_ref = orc.logits_canon_f32(x, Wg)
    assert np.array_equal(l_ref.astype(np.float64), exact)
    if collab is not None:
        for t in range(T):
            assert set(idx[t, 1:]) <= set(collab[idx[t, 0]])


def test_route_full_list_is_topk(c2r, orc):
    # Fig. 3 caption: a list of all other experts removes the constraint
    w = wl.scaled(wl.WORKLOADS["C1"], T=300)
    x = wl.hidden(w)
    Wg, _ = wl.router(w)
    full = np.array([[j for j in range(w.E) if j != i] for i in range(w.E)], dtype=np.int32)
    a = c2r.route(dev(x), dev(Wg), None, w.K, dev(full))
    b = c2r.route(dev(x), dev(Wg), None, w.K, None)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_route_short_or_bad_list_entries(c2r, orc):
    # duplicate / self / out-of-range entries are ignored; an unfillable slot gets -1 and gate 0
    E, K = 8, 3
    x, Wg = wl.exact_arithmetic_router(100, 64, E, seed=3)
    collab = np.array([[i, (i + 1) % E, (i + 1) % E, 99] for i in range(E)], dtype=np.int32)
    idx, gates, _ = c2r.route(dev(x), dev(Wg), None, K, dev(collab))
    idx, gates = host(idx), host(gates)
    l = orc.logits_canon_f32(x, Wg)
    assert np.array_equal(idx[:, 0], np.argmax(l, axis=1))
    assert np.array_equal(idx[:, 1], (idx[:, 0] + 1) % E)
    assert np.all(idx[:, 2] == -1) and np.all(gates[:, 2] == 0)
    np.testing.assert_allclose(gates.sum(1), 1.0, rtol=1e-6)


@pytest.mark.parametrize("E,K,Tc,T", [(60, 4, 16, 5000), (7, 2, 3, 63), (64, 4, 8, 257), (16, 4, 8, 1),
                                     (16, 6, 9, 300), (24, 10, 12, 129), (30, 4, 5, 200)])
def test_route_from_logits(c2r, orc, E, K, Tc, T):
    rng = np.random.default_rng(E)
    logits = rng.integers(-5, 6, size=(T, E)).astype(np.float32)       # many ties
    logits[::7] += rng.standard_normal((len(logits[::7]), E)).astype(np.float32)
    collab = _collab(E, Tc, 3)
    for ci in (collab, None):
        idx, gates = c2r.route_from_logits(dev(logits), K, None if ci is None else dev(ci))
        idx_ref, g_ref = orc.route(logits, K, ci)
        assert np.array_equal(host(idx), idx_ref)
        np.testing.assert_allclose(host(gates), g_ref, rtol=GATE_RTOL, atol=1e-7)


@pytest.mark.parametrize("E,K,Tc,T", [(4, 1, 0, 100), (4, 4, 3, 777), (20, 2, 5, 1000), (36, 3, 35, 641),
                                     (52, 3, 2, 300), (60, 4, 16, 4 * 64 * 513 + 5), (8, 4, 7, 140001)])
def test_route_from_logits_special_values_signed_zeros_and_short_lists(c2r, orc, E, K, Tc, T):
    # E a multiple of 4 and K <= 4: the quad-per-token kernel.  Values with many ties, signed zeros
    # (equal as floats: the lower index stands), -inf / +inf / NaN in some rows (those take the literal
    # scan), lists with duplicates, self and out-of-range entries (fewer usable entries than K - 1),
    # and enough tokens that a workgroup walks more than one group of 64.
    rng = np.random.default_rng(E * 100 + K)
    logits = rng.integers(-3, 4, size=(T, E)).astype(np.float32)
    logits[rng.random((T, E)) < 0.2] = -0.0
    logits[1::9] += rng.standard_normal((len(logits[1::9]), E)).astype(np.float32)
    logits[3::50, rng.integers(0, E)] = -np.inf
    logits[7::61, rng.integers(0, E)] = np.inf
    logits[11::73, rng.integers(0, E)] = np.nan
    logits[13::97] = -np.inf
    if T > 200:
        logits[150] = np.nan
    # (list handed to the library, the same list as the oracle takes it: the oracle's lists hold valid
    # expert numbers only, so an out-of-range entry - which the library ignores - is given to it as a
    # repeat of another entry)
    lists = [(None, None)]
    if Tc > 0:
        collab = _collab(E, Tc, 7)
        lists.append((collab, collab))
        if Tc - 3 >= K - 1:
            bad = collab.copy()
            bad[:, 0] = np.arange(E)          # the expert itself
            bad[:, 1] = bad[:, 2]             # a duplicate
            clean = bad.copy()
            bad[::2, Tc - 1] = E + 5          # out of range
            bad[1::2, Tc - 1] = -2
            clean[:, Tc - 1] = clean[:, 2]
            lists.append((bad, clean))
    for ci, ci_ref in lists:
        idx, gates = c2r.route_from_logits(dev(logits), K, None if ci is None else dev(ci))
        idx_ref, g_ref = orc.route(logits, K, ci_ref)
        assert np.array_equal(host(idx), idx_ref)
        np.testing.assert_allclose(host(gates), g_ref, rtol=GATE_RTOL, atol=1e-7, equal_nan=True)


@pytest.mark.parametrize("E,K,Tc,T", [(60, 4, 16, 70001), (60, 4, 0, 4 * 64 * 513 + 9), (16, 2, 5, 1000), (8, 4, 7, 64),
                                     (30, 3, 6, 500), (24, 6, 8, 300)])
def test_profile_from_logits_equals_route_then_count(c2r, orc, E, K, Tc, T):
    # one launch (selection + Eq. 2 counts) against the oracle's route -> coactivation, with and without
    # the selections written, accumulating over two batches; shapes outside the fused kernel
    # (E not a multiple of 4, K > 4) run the two kernels and must give the same
    rng = np.random.default_rng(E + K + T)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[:, : E // 3] += 1.0
    logits[::13] = np.round(logits[::13])                              # ties
    logits[5::101, 0] = np.nan
    ci = _collab(E, Tc, 11) if Tc else None
    idx_ref, g_ref = orc.route(logits, K, ci)
    C_ref = orc.coactivation(idx_ref, E)
    fused_shape = E % 4 == 0 and K <= 4
    Cm = torch.zeros((E, E), dtype=torch.int32, device="cuda")
    _, idx, gates = c2r.profile_from_logits(dev(logits), K, Cm, None if ci is None else dev(ci), want_selection=True)
    assert np.array_equal(host(idx), idx_ref)
    np.testing.assert_allclose(host(gates), g_ref, rtol=GATE_RTOL, atol=1e-7, equal_nan=True)
    assert np.array_equal(host(Cm).astype(np.int64), C_ref)
    if fused_shape:                                                     # counts alone, added to what is there
        c2r.profile_from_logits(dev(logits[: T // 2]), K, Cm, None if ci is None else dev(ci))
        assert np.array_equal(host(Cm).astype(np.int64), orc.coactivation(idx_ref[: T // 2], E, C_ref))
    else:
        with pytest.raises(RuntimeError):
            c2r.profile_from_logits(dev(logits), K, Cm, None if ci is None else dev(ci))


def test_route_from_logits_single_expert(c2r, orc):
    # E = 1: every token selects expert 0; its gate is exp(l - l) / sum = 1 for a finite logit and
    # NaN for an infinite or NaN one (the stated gate rule)
    logits = np.random.default_rng(1).standard_normal((333, 1)).astype(np.float32)
    logits[5, 0], logits[17, 0], logits[40, 0] = np.nan, np.inf, -np.inf
    idx, gates = c2r.route_from_logits(dev(logits), 1, None)
    idx_ref, g_ref = orc.route(logits, 1, None)
    assert np.array_equal(host(idx), idx_ref) and not host(idx).any()
    g = host(gates)
    assert np.array_equal(np.isnan(g), np.isnan(g_ref)) and np.isnan(g[[5, 17, 40], 0]).all()
    assert np.array_equal(g[~np.isnan(g)], np.ones(330, dtype=np.float32))


def test_route_nan_logits_follow_the_stated_rule(c2r, orc):
    E, K = 12, 3
    logits = np.random.default_rng(5).standard_normal((200, E)).astype(np.float32)
    logits[::3, 0] = np.nan
    logits[1::5, 7] = np.nan
    logits[10] = np.nan
    idx, _ = c2r.route_from_logits(dev(logits), K, None)
    idx_ref, _ = orc.route(logits, K, None)
    assert np.array_equal(host(idx), idx_ref)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_route_nan_and_inf_logits_through_the_router(c2r, orc, dtype):
    # infinite router weights meet zero (-> NaN) and non-zero (-> +-inf) activations; one token is all NaN
    w = wl.scaled(wl.WORKLOADS["C3"], T=300)
    x = wl.hidden(w).copy()
    Wg, bias = wl.router(w)
    Wg = Wg.copy()
    Wg[5, 0], Wg[7, 9], Wg[300, 59] = np.inf, -np.inf, np.inf
    x[::3, 5] = 0.0
    x[1::4, 7] = 0.0
    x[2::7, 300] = 0.0
    x[10] = np.nan
    collab = _collab(w.E, w.Tc, 3)
    for cl in (collab, None):
        idx, gates, logits = c2r.route(dev(x, dtype), dev(Wg), dev(bias), w.K,
                                       None if cl is None else dev(cl), want_logits=True)
        torch.cuda.synchronize()
        l_gpu, l_ref = host(logits), orc.logits_canon_f32(x, Wg, bias)
        assert np.isnan(l_gpu).sum() > 200 and np.isinf(l_gpu).sum() > 200
        assert np.array_equal(np.isnan(l_gpu), np.isnan(l_ref))
        ok = ~np.isnan(l_ref)
        assert np.array_equal(l_gpu[ok].view(np.uint32), l_ref[ok].view(np.uint32))
        idx_ref, g_ref = orc.route(l_gpu, w.K, cl)
        assert np.array_equal(host(idx), idx_ref)
        np.testing.assert_allclose(host(gates), g_ref, rtol=GATE_RTOL, atol=1e-7, equal_nan=True)


@pytest.mark.parametrize("E,K,T", [(8, 2, 512), (16, 4, 1000), (60, 4, 70001), (64, 6, 129), (33, 3, 64)])
def test_coactivation(c2r, orc, E, K, T):
    rng = np.random.default_rng(E + T)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[:, : E // 3] += 1.5                                          # skewed load
    idx, _ = orc.route(logits, K)
    idx[::11, K - 1] = -1                                               # padded slots are ignored
    Cg = c2r.build_coactivation(dev(idx), E)
    assert np.array_equal(host(Cg).astype(np.int64), orc.coactivation(idx, E))
    # accumulate a second batch into the same matrix
    c2r.build_coactivation(dev(idx[: T // 2]), E, Cg)
    assert np.array_equal(host(Cg).astype(np.int64),
                          orc.coactivation(idx[: T // 2], E, orc.coactivation(idx, E)))
    M = host(Cg)
    assert np.array_equal(M, M.T)


@pytest.mark.parametrize("E", [2, 8, 60, 64])
def test_collaborators(c2r, orc, E):
    rng = np.random.default_rng(E)
    Cm = rng.integers(0, 4, size=(E, E))
    Cm = Cm + Cm.T
    if E > 4:
        Cm[3, :] = 0
        Cm[:, 3] = 0
    np.fill_diagonal(Cm, 10 ** 6)
    for Tc in sorted({1, min(4, E - 1), E - 1, E + 3}):
        ci, mask = c2r.collaborators(dev(Cm.astype(np.int32)), Tc)
        ref = orc.collaborators(Cm, Tc)
        assert np.array_equal(host(ci), ref)
        m = host(mask).astype(np.uint64)
        for i in range(E):
            assert int(m[i]) == sum(1 << int(j) for j in ref[i])


@pytest.mark.parametrize("E,K,T,d,dtype,local", [
    (8, 2, 512, 256, "f32", None), (60, 4, 3001, 64, "bf16", None), (60, 4, 5000, 128, "bf16", 15),
    (16, 4, 1, 64, "bf16", None), (64, 1, 1025, 72, "f32", 7), (5, 5, 300, 8, "f32", None),
    # more than 49152 assignments: the histogram / scan / rank launches instead of the one-launch sweep;
    # 49152 and 49153: either side of the switch; 2^15 + 1: the one-launch sweep's second register pass
    (60, 4, 70001, 8, "bf16", None), (16, 4, 65536, 8, "bf16", 5), (16, 4, 65537, 8, "bf16", None),
    (60, 3, 16384, 8, "bf16", None), (16, 1, 49153, 8, "bf16", 5), (33, 1, 32769, 8, "bf16", None)])
def test_permute(c2r, orc, E, K, T, d, dtype, local):
    rng = np.random.default_rng(E * 7 + T)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[:, 0] += 2.0
    idx, _ = orc.route(logits, K)
    x = rng.standard_normal((T, d)).astype(np.float32)
    if dtype == "bf16":
        x = wl.round_bf16(x)
    ls, E_local = None, E
    if local:
        ls = np.full(E, -1, dtype=np.int32)
        chosen = np.sort(rng.permutation(E)[:local])
        ls[chosen] = rng.permutation(local).astype(np.int32)            # arbitrary renumbering
        E_local = local
    counts, offsets, perm, inv, x_perm = c2r.permute(dev(x, dtype), dev(idx), E, dev(ls), E_local)
    rc, ro, rp, ri = orc.permute(idx, E, ls, E_local)
    assert np.array_equal(host(counts), rc) and np.array_equal(host(offsets), ro)
    n = int(ro[-1])
    assert np.array_equal(host(perm)[:n], rp) and np.all(host(perm)[n:] == -1)
    assert np.array_equal(host(inv), ri)
    assert np.array_equal(host(x_perm)[:n], x[rp // K])                 # pure copy: bit exact


@pytest.mark.parametrize("dtype,d,F,sizes", [
    ("f32", 64, 96, [5, 0, 70, 1, 130]), ("f32", 256, 512, [100, 300, 0, 3]),
    ("bf16", 128, 256, [300, 0, 1, 64, 257, 5]), ("bf16", 64, 88, [33, 700]),
    ("bf16", 256, 688, [12, 0, 0, 513]), ("bf16", 2048, 128, [40, 260]),
    # tile-map edges: group sizes around the 128-row short-tile and 256-row tile limits, groups of
    # more than one 4-tile chunk, many small groups next to a large one, 64 groups
    ("bf16", 64, 64, [128, 129, 127, 256, 255, 257, 0, 1]), ("bf16", 64, 128, [1100, 3, 0, 0, 2100, 64]),
    ("bf16", 128, 64, [7] * 30 + [1500] + [0] * 20 + [130] * 13),
    # around the 64-row tile class and the 16-row fragment granularity; then a Zipf-like mix of 48 groups
    ("bf16", 64, 64, [63, 65, 15, 16, 17, 191, 192, 193, 320, 321, 48, 49]),
    ("bf16", 64, 128, [int(2600 / (i + 1) ** 1.1) for i in range(48)])])
def test_expert_ffn_ragged_groups(c2r, orc, dtype, d, F, sizes):
    rng = np.random.default_rng(d + F)
    E = len(sizes)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    n = int(offsets[-1])
    cap = n + 37                                                         # capacity beyond the used rows
    store = wl.round_bf16 if dtype == "bf16" else (lambda a: a)
    x = store(rng.standard_normal((cap, d)).astype(np.float32))
    wg = store((rng.standard_normal((E, F, d)) * 0.05).astype(np.float32))
    wu = store((rng.standard_normal((E, F, d)) * 0.05).astype(np.float32))
    wd = store((rng.standard_normal((E, d, F)) * 0.05).astype(np.float32))
    sentinel = 123.0
    y = torch.full((cap, d), sentinel, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    c2r.expert_ffn(dev(x, dtype), dev(offsets), dev(wg, dtype), dev(wu, dtype), dev(wd, dtype), out=y)
    torch.cuda.synchronize()
    yh = host(y)
    eor = np.repeat(np.arange(E), sizes).astype(np.int32)
    ref = orc.expert_ffn_rows(x[:n], eor, wg, wu, wd)
    assert max_rel_err(yh[:n], ref) <= (1e-2 if dtype == "bf16" else 1e-5)
    assert np.all(yh[n:] == sentinel)                                   # rows past the last group untouched


@pytest.mark.parametrize("E,K,T,d,F,local", [(8, 2, 700, 128, 256, None), (60, 4, 1500, 2048, 128, 7),
                                              (4, 1, 129, 64, 64, None), (16, 3, 300, 256, 192, 5)])
def test_gate_up_gather_equals_gate_up_on_x_perm(c2r, E, K, T, d, F, local):
    """The first FFN pass reading x through perm (the dispatch gather folded into its loads)
    gives, bit for bit, what it gives on the x_perm that c2r_permute writes; dropped
    assignments (perm = -1 beyond the last group) are never read."""
    rng = np.random.default_rng(E + T)
    idx = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    x = dev(wl.round_bf16(rng.standard_normal((T, d)).astype(np.float32)), "bf16")
    ls, E_local = None, E
    if local:
        ls = np.full(E, -1, dtype=np.int32)
        ls[np.sort(rng.permutation(E)[:local])] = rng.permutation(local).astype(np.int32)
        E_local = local
    counts, offsets, perm, inv, x_perm = c2r.permute(x, dev(idx), E, dev(ls), E_local)
    wg = dev(wl.round_bf16((rng.standard_normal((E_local, F, d)) * 0.05).astype(np.float32)), "bf16")
    wu = dev(wl.round_bf16((rng.standard_normal((E_local, F, d)) * 0.05).astype(np.float32)), "bf16")
    assert c2r.gather_fusable(torch.bfloat16, d, F)
    h0 = torch.full((T * K, F), 7.0, dtype=torch.bfloat16, device="cuda")
    h1 = h0.clone()
    c2r.expert_ffn_gate_up(x_perm, offsets, wg, wu, h0)
    c2r.expert_ffn_gate_up_gather(x, perm, K, offsets, wg, wu, h1)
    torch.cuda.synchronize()
    assert torch.equal(h0, h1)
    n = int(offsets[-1])
    assert n > 0 and torch.all(h1[n:] == 7.0)


@pytest.mark.parametrize("E,K,T,d,F,local", [(16, 4, 600, 256, 688, None), (8, 2, 513, 128, 1376, None),
                                              (12, 3, 300, 64, 88, 5), (8, 2, 700, 128, 256, None)])
def test_ffn_gather_equals_ffn_on_x_perm(c2r, E, K, T, d, F, local):
    """Both passes with the gather folded in, for any F the library takes (h padded inside the
    workspace): bit for bit what c2r_expert_ffn gives on the x_perm of c2r_permute."""
    rng = np.random.default_rng(E + T + F)
    idx = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    x = dev(wl.round_bf16(rng.standard_normal((T, d)).astype(np.float32)), "bf16")
    ls, E_local = None, E
    if local:
        ls = np.full(E, -1, dtype=np.int32)
        ls[np.sort(rng.permutation(E)[:local])] = rng.permutation(local).astype(np.int32)
        E_local = local
    counts, offsets, perm, inv, x_perm = c2r.permute(x, dev(idx), E, dev(ls), E_local)
    w = [dev(wl.round_bf16((rng.standard_normal(shape) * 0.05).astype(np.float32)), "bf16")
         for shape in ((E_local, F, d), (E_local, F, d), (E_local, d, F))]
    y0 = torch.full((T * K, d), 7.0, dtype=torch.bfloat16, device="cuda")
    y1 = y0.clone()
    c2r.expert_ffn(x_perm, offsets, *w, out=y0)
    c2r.expert_ffn_gather(x, perm, K, offsets, *w, out=y1)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    n = int(offsets[-1])
    assert n > 0 and torch.all(y1[n:] == 7.0) and not torch.all(y1[:n] == 7.0)


@pytest.mark.parametrize("E,K,T,d,F,Fs,local", [(60, 4, 700, 128, 192, 448, False), (7, 2, 300, 64, 64, 64, False),
                                                   (16, 4, 1500, 256, 128, 640, True), (5, 1, 64, 64, 128, 192, False)])
def test_ffn_with_shared_equals_separate_launches(c2r, E, K, T, d, F, Fs, local):
    # routed groups + always-on shared expert in one launch per pass: the same bits as the
    # separate launches (gather-fused routed passes; shared expert with E_local = 1 on x)
    rng = np.random.default_rng(E * 1000 + T)
    idx = rng.integers(0, E, size=(T, K)).astype(np.int32)
    idx[::9, 0] = -1
    if local:
        ls = np.full(E, -1, dtype=np.int32)
        keep = np.sort(rng.permutation(E)[: E // 2])
        ls[keep] = np.arange(len(keep), dtype=np.int32)
        El = len(keep)
    else:
        ls, El = None, E
    x = dev(rng.standard_normal((T, d)).astype(np.float32), "bf16")
    w = lambda *sh: dev((rng.standard_normal(sh) * 0.05).astype(np.float32), "bf16")
    wg, wu, wd = w(El, F, d), w(El, F, d), w(El, d, F)
    sg, su, sd = w(1, Fs, d), w(1, Fs, d), w(1, d, Fs)
    counts, offsets, perm, inv, _ = c2r.permute(x, dev(idx), E, dev(ls), El, rows=False)
    A = T * K
    bf = dict(dtype=torch.bfloat16, device="cuda")
    h1, hs1 = torch.zeros(A, F, **bf), torch.zeros(T, Fs, **bf)
    y1, ys1 = torch.zeros(A, d, **bf), torch.zeros(T, d, **bf)
    h2, hs2, y2, ys2 = (torch.zeros_like(t) for t in (h1, hs1, y1, ys1))
    off_s = torch.tensor([0, T], dtype=torch.int32, device="cuda")
    c2r.expert_ffn_gate_up_gather(x, perm, K, offsets, wg, wu, h1)
    c2r.expert_ffn_gate_up(x, off_s, sg, su, hs1)
    c2r.expert_ffn_down(h1, offsets, wd, y1)
    c2r.expert_ffn_down(hs1, off_s, sd, ys1)
    c2r.expert_ffn_gate_up_with_shared(x, perm, K, offsets, wg, wu, h2, sg, su, hs2)
    c2r.expert_ffn_down_with_shared(h2, offsets, wd, y2, hs2, sd, ys2)
    torch.cuda.synchronize()
    n = int(offsets[-1])
    assert n > 0
    assert torch.equal(h1[:n], h2[:n]) and torch.equal(hs1, hs2)
    assert torch.equal(y1[:n], y2[:n]) and torch.equal(ys1, ys2)
    assert not y2[n:].any() and not h2[n:].any()          # rows past the groups are untouched


def test_gate_up_gather_rejects_other_shapes(c2r):
    x = torch.zeros((8, 72), dtype=torch.float32, device="cuda")
    perm = torch.zeros((8,), dtype=torch.int32, device="cuda")
    off = torch.tensor([0, 8], dtype=torch.int32, device="cuda")
    w = torch.zeros((1, 64, 72), dtype=torch.float32, device="cuda")
    h = torch.zeros((8, 64), dtype=torch.float32, device="cuda")
    assert not c2r.gather_fusable(torch.float32, 72, 64)
    with pytest.raises(RuntimeError):
        c2r.expert_ffn_gate_up_gather(x, perm, 1, off, w, w, h)


@pytest.mark.parametrize("dtype,T,K,d", [("f32", 100, 2, 64), ("bf16", 1000, 4, 2048), ("bf16", 3, 1, 8)])
def test_combine(c2r, orc, dtype, T, K, d):
    rng = np.random.default_rng(T)
    store = wl.round_bf16 if dtype == "bf16" else (lambda a: a)
    E = 9
    idx, g = orc.route(rng.standard_normal((T, E)).astype(np.float32), K)
    ls = np.arange(E, dtype=np.int32)
    ls[4] = -1
    ls[5:] -= 1
    _, _, perm, inv = orc.permute(idx, E, ls, E - 1)
    yp = store(rng.standard_normal((T * K, d)).astype(np.float32))
    ys = store(rng.standard_normal((T, d)).astype(np.float32))
    g32 = g.astype(np.float32)
    for shared in (None, ys):
        y = c2r.combine(dev(yp, dtype), dev(g32), dev(inv), None if shared is None else dev(shared, dtype))
        ref = orc.combine(yp, g32, inv, T, K, shared)
        tol = 2.0 ** -8 if dtype == "bf16" else 1e-6                    # one rounding of the result
        assert np.abs(host(y) - ref).max() <= tol * max(np.abs(ref).max(), 1.0)


@pytest.mark.parametrize("E,K,T,n_dev,holes", [(12, 4, 300, 4, True), (60, 4, 5000, 4, False), (64, 8, 1025, 64, True),
                                               (8, 2, 1, 2, False), (60, 4, 8192, 6, False), (16, 1, 4100, 3, True),
                                               # K > 8: the devices of a token no longer fit one packed register
                                               (24, 9, 700, 5, True), (64, 16, 1030, 8, False)])
def test_dedup_dispatch(c2r, orc, E, K, T, n_dev, holes):
    """Sec. 3.4: send list (device-major, tokens ascending) and copy row per assignment, bit exact."""
    rng = np.random.default_rng(E * 13 + T)
    idx, _ = orc.route(rng.standard_normal((T, E)).astype(np.float32), K)
    devmap = (np.arange(E) * n_dev // E).astype(np.int32)
    if holes:
        idx = idx.copy()
        idx[rng.integers(0, T, size=max(1, T // 7)), rng.integers(0, K, size=max(1, T // 7))] = -1   # empty slots
        devmap[rng.integers(0, E)] = -1                                                               # expert without a device
    counts, offsets, tok, row = c2r.dedup_dispatch(dev(idx), E, dev(devmap), n_dev)
    rc, ro, rt, rr = orc.dedup_dispatch(idx, E, devmap, n_dev)
    assert np.array_equal(host(counts), rc) and np.array_equal(host(offsets), ro)
    n = int(ro[-1])
    assert np.array_equal(host(tok)[:n], rt) and np.all(host(tok)[n:] == -1)
    assert np.array_equal(host(row), rr)
    if not holes:
        assert n == int(orc.distinct_devices(idx, devmap).sum())


@pytest.mark.parametrize("dtype,T,K,d,n_dev", [("f32", 300, 3, 64, 3), ("bf16", 2000, 4, 512, 4), ("bf16", 5, 2, 8, 2)])
def test_two_level_combine(c2r, orc, dtype, T, K, d, n_dev):
    rng = np.random.default_rng(T + d)
    store = wl.round_bf16 if dtype == "bf16" else (lambda a: a)
    E = 12
    idx, g = orc.route(rng.standard_normal((T, E)).astype(np.float32), K)
    ls = np.arange(E, dtype=np.int32)
    ls[7] = -1
    ls[8:] -= 1                                                          # expert 7 is not computed here
    _, _, perm, inv = orc.permute(idx, E, ls, E - 1)
    devmap = (np.arange(E) * n_dev // E).astype(np.int32)
    yp = store(rng.standard_normal((T * K, d)).astype(np.float32))
    ys = store(rng.standard_normal((T, d)).astype(np.float32))
    g32 = g.astype(np.float32)
    _, offsets, tok, row = c2r.dedup_dispatch(dev(idx), E, dev(devmap), n_dev)
    _, ro, rt, rr = orc.dedup_dispatch(idx, E, devmap, n_dev)
    part = c2r.combine_partial(dev(yp, dtype), dev(g32), dev(inv), tok, row, offsets)
    n = int(ro[-1])
    ref_part = orc.combine_partial(yp, g32, inv, rr, T, K, n)
    tol = 2.0 ** -8 if dtype == "bf16" else 1e-6                         # one rounding per level
    assert np.abs(host(part)[:n] - ref_part).max() <= tol * max(np.abs(ref_part).max(), 1.0)
    for shared in (None, ys):
        y = c2r.combine_copies(part, row, T, K, None if shared is None else dev(shared, dtype))
        ref = orc.combine(yp, g32, inv, T, K, shared)                    # the same sum, grouped differently
        assert np.abs(host(y) - ref).max() <= 2 * tol * max(np.abs(ref).max(), 1.0)
        # and exactly the second level applied to the first level's (rounded) rows
        ref2 = orc.combine_copies(host(part)[:n], rr, T, K, shared)
        assert np.abs(host(y) - ref2).max() <= tol * max(np.abs(ref2).max(), 1.0)


@pytest.mark.parametrize("E,n_dev,kind", [(12, 4, "blocks"), (60, 4, "random"), (64, 8, "random"), (10, 4, "ties"),
                                          (7, 7, "random"), (60, 6, "profile")])
def test_place_experts(c2r, orc, E, n_dev, kind):
    rng = np.random.default_rng(E + n_dev)
    if kind == "blocks":
        label = rng.permutation(np.repeat(np.arange(n_dev), E // n_dev))
        Cm = (label[:, None] == label[None, :]).astype(np.int64) * 100 + rng.integers(0, 10, size=(E, E))
        Cm = Cm + Cm.T
    elif kind == "ties":
        Cm = np.ones((E, E), dtype=np.int64)
    elif kind == "profile":
        w = wl.WORKLOADS["C3"]
        Wg, b = wl.router(w)
        idx, _ = orc.route(orc.logits_canon_f32(wl.hidden(w, 4096, stream=1), Wg, b), w.K)
        Cm = orc.coactivation(idx, w.E)
    else:
        Cm = rng.integers(0, 1000, size=(E, E))
        Cm = Cm + Cm.T
    got = c2r.place_experts(dev(Cm.astype(np.int32)), n_dev)
    assert np.array_equal(host(got), orc.place_experts(Cm, n_dev))


@pytest.mark.parametrize("E,kind", [(8, "random"), (60, "profile"), (64, "random"), (16, "sparse"), (1, "random")])
def test_collaboration_degree(c2r, orc, E, kind):
    # Eq. 3 in fp64 on the device against the numpy definition; the bar is rounding order only
    rng = np.random.default_rng(100 + E)
    if kind == "profile":
        w = wl.WORKLOADS["C3"]
        Wg, b = wl.router(w)
        idx, _ = orc.route(orc.logits_canon_f32(wl.hidden(w, 4096, stream=1), Wg, b), w.K)
        Cm = orc.coactivation(idx, w.E)
    else:
        Cm = rng.integers(0, 1 << 20, size=(E, E))
        Cm = Cm + Cm.T
        if kind == "sparse":
            Cm[rng.random((E, E)) < 0.6] = 0
            Cm[3, :] = 0          # an expert that is never co-activated: degree 0
            Cm[3, 3] = 77         # the diagonal takes no part
    got = host(c2r.collaboration_degree(dev(Cm.astype(np.int32))))
    ref = orc.collaboration_degree(Cm)
    assert got.dtype == np.float64 and got.shape == (E,)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-15)
    if kind == "sparse":
        assert got[3] == 0.0


@pytest.mark.parametrize("T,K,E,eps", [(1000, 4, 60, (2, 3, 4, 5, 6)), (4097, 2, 8, (2, 4, 8)), (1, 4, 64, (64,)),
                                       (70000, 4, 60, (1, 2, 3, 4, 5, 6, 10, 12)), (0, 4, 60, (2,))])
def test_distinct_devices(c2r, orc, T, K, E, eps):
    # per-token counts and totals for several expert-parallel degrees in one pass; exact
    rng = np.random.default_rng(T + K + E)
    idx = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32) if T else np.zeros((0, K), np.int32)
    n_dev = max(eps)
    maps = np.stack([rng.permutation(wl.device_map(E, ep) if E % ep == 0 else np.arange(E) % ep) for ep in eps])
    tot, pt = c2r.distinct_devices(dev(idx), E, dev(maps.astype(np.int32)), n_dev, per_token=True)
    tot, pt = host(tot), host(pt)
    for m in range(len(eps)):
        ref = orc.distinct_devices(idx, maps[m]) if T else np.zeros(0, np.int32)
        assert np.array_equal(pt[m], ref), eps[m]
        assert tot[m] == int(ref.sum())
    if T:
        # the totals are the copies the zero-redundancy send list holds for the same map
        n_send = int(host(c2r.dedup_dispatch(dev(idx), E, dev(maps[0].astype(np.int32)), n_dev)[1])[-1])
        assert n_send == tot[0]
        # experts without a device and empty slots are skipped
        idx2, map2 = idx.copy(), maps[0].astype(np.int32).copy()
        idx2[::3, 0] = -1
        map2[::5] = -1
        ref = np.array([len({map2[e] for e in row if e >= 0 and map2[e] >= 0}) for row in idx2])
        tot2, pt2 = c2r.distinct_devices(dev(idx2), E, dev(map2), n_dev, per_token=True)
        assert np.array_equal(host(pt2)[0], ref) and int(host(tot2)[0]) == int(ref.sum())
