"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each one is chosen so that a
plausible slip in oracle/c2r_oracle.c (dropped term, wrong sign or index,
transposed operand, wrong tie rule) fails it.
"""
import itertools
import math
import os

import numpy as np
import pytest

from paper_2504_01337_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _small_logits(T, E, seed, ties=False):
    rng = np.random.default_rng(seed)
    if ties:
        return rng.integers(-3, 4, size=(T, E)).astype(np.float32)
    return rng.standard_normal((T, E)).astype(np.float32)


def _random_collab(E, Tc, seed):
    rng = np.random.default_rng(seed)
    out = np.empty((E, Tc), dtype=np.int32)
    for i in range(E):
        others = np.array([j for j in range(E) if j != i])
        out[i] = rng.permutation(others)[:Tc]
    return out


# ---------------- Eq. 1: logits ----------------

def test_logits_f64_matches_library_matmul(orc):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((37, 50)).astype(np.float32)
    Wg = rng.standard_normal((50, 11)).astype(np.float32)
    b = rng.standard_normal(11).astype(np.float32)
    ref = x.astype(np.float64) @ Wg.astype(np.float64) + b.astype(np.float64)
    np.testing.assert_allclose(orc.logits_f64(x, Wg, b), ref, rtol=1e-13, atol=1e-13)
    # a transposed W_g would not even have this shape; a non-square case pins the layout
    np.testing.assert_allclose(orc.logits_f64(x, Wg), x.astype(np.float64) @ Wg.astype(np.float64),
                               rtol=1e-13, atol=1e-13)


def test_logits_exact_arithmetic_any_order(orc):
    # P12: integer / dyadic inputs: fp32 result is the exact integer-arithmetic value
    x, Wg = wl.exact_arithmetic_router(64, 1024, 12)
    exact = (x.astype(np.int64) @ np.round(Wg * 8).astype(np.int64)).astype(np.float64) / 8.0
    for chunk in (1, 7, 256, 4096):
        got = orc.logits_canon_f32(x, Wg, chunk=chunk)
        assert got.dtype == np.float32
        assert np.array_equal(got.astype(np.float64), exact)
    assert np.array_equal(orc.logits_f64(x, Wg), exact)


def test_logits_canon_order_hand_cases(orc):
    with open(os.path.join(GOLDEN, "canon_order_cases.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for r in rows:
        chunk, expected = int(r[0]), float(r[1])
        x = np.array([[float(v) for v in r[2:]]], dtype=np.float32)
        Wg = np.ones((x.shape[1], 1), dtype=np.float32)
        assert orc.logits_canon_f32(x, Wg, chunk=chunk)[0, 0] == np.float32(expected), r


def test_logits_canon_is_fused(orc):
    # (1+2^-12)^2 - (1+2^-11) = 2^-24 exactly; an unfused multiply rounds the product
    # to 1+2^-11 (tie to even) and returns 0.
    a = np.float32(1.0 + 2.0 ** -12)
    x = np.array([[-1.0 - 2.0 ** -11, a]], dtype=np.float32)
    Wg = np.array([[1.0], [a]], dtype=np.float32)
    assert orc.logits_canon_f32(x, Wg, chunk=256)[0, 0] == np.float32(2.0 ** -24)


def test_logits_canon_bias_added_last_and_close_to_f64(orc):
    w = wl.scaled(wl.WORKLOADS["C3"], T=48)
    x = wl.hidden(w)
    Wg, b = wl.router(w)
    l32 = orc.logits_canon_f32(x, Wg, b)
    l32_nb = orc.logits_canon_f32(x, Wg, None)
    assert np.array_equal(l32, l32_nb + b[None, :])      # one fp32 add, after the sum
    l64 = orc.logits_f64(x, Wg, b)
    assert np.abs(l32 - l64).max() <= 1e-5 * np.abs(l64).max()


# ---------------- Sec. 3.3: selection ----------------

@pytest.mark.parametrize("ties", [False, True])
def test_plain_topk_matches_stable_sort(orc, ties):
    l = _small_logits(300, 13, 1, ties)
    idx, _ = orc.route(l, 4)
    ref = np.argsort(-l.astype(np.float64), axis=1, kind="stable")[:, :4]   # ties -> lower index
    assert np.array_equal(idx, ref)


@pytest.mark.parametrize("E,K", [(8, 2), (13, 4), (60, 4)])
def test_full_list_degenerates_to_topk(orc, E, K):
    # Fig. 3 caption: with N-1 collaborators the method is conventional top-K (P1)
    l = _small_logits(400, E, 2, ties=True)
    full = np.array([[j for j in range(E) if j != i] for i in range(E)], dtype=np.int32)
    i0, g0 = orc.route(l, K)
    i1, g1 = orc.route(l, K, full[:, ::-1].copy())        # list order must not matter
    assert np.array_equal(i0, i1) and np.array_equal(g0, g1)


@pytest.mark.parametrize("ties", [False, True])
def test_c2r_selection_invariants(orc, ties):
    E, K, Tc = 16, 4, 6
    l = _small_logits(500, E, 3, ties)
    ci = _random_collab(E, Tc, 4)
    idx, g = orc.route(l, K, ci)
    assert np.array_equal(idx[:, 0], np.argmax(l, axis=1))            # slot 0: global arg max
    for t in range(l.shape[0]):
        e0 = idx[t, 0]
        assert len(set(idx[t])) == K
        assert set(idx[t, 1:]) <= set(ci[e0])                          # P2
        v = l[t, idx[t]]
        assert np.all(np.diff(v[1:]) <= 0) and v[0] >= v.max()
    # P6
    np.testing.assert_allclose(g.sum(1), 1.0, rtol=1e-14)
    assert np.all(g > 0) and np.all(g[:, 0] >= 1.0 / K - 1e-15)
    assert np.all(np.diff(g[:, 1:], axis=1) <= 1e-18)


def test_c2r_brute_force(orc):
    # P7: all K-subsets {arg max} + (K-1 of the list), best = lexicographically largest
    # sorted (logit desc, index asc) sequence
    E, K, Tc = 8, 3, 4
    l = _small_logits(200, E, 5, ties=True)
    ci = _random_collab(E, Tc, 6)
    idx, _ = orc.route(l, K, ci)
    for t in range(l.shape[0]):
        e0 = min(range(E), key=lambda e: (-l[t, e], e))
        best = None
        for sub in itertools.combinations(sorted(ci[e0]), K - 1):
            order = sorted(sub, key=lambda e: (-l[t, e], e))
            key = [(-l[t, e], e) for e in order]
            if best is None or key < best[0]:
                best = (key, order)
        assert list(idx[t]) == [e0] + best[1]


def test_single_collaborator_ignores_scores(orc):
    # P11: K=2 with a one-entry list: the partner is that entry whatever its logit
    E = 8
    l = _small_logits(100, E, 7)
    ci = _random_collab(E, 1, 8)
    idx, _ = orc.route(l, 2, ci)
    assert np.array_equal(idx[:, 1], ci[idx[:, 0], 0])


def test_short_list_is_an_error(orc):
    l = _small_logits(4, 8, 9)
    with pytest.raises(ValueError):
        orc.route(l, 4, _random_collab(8, 2, 1))


def test_gates_are_softmax_of_kept_logits(orc):
    from scipy.special import softmax
    l = _small_logits(200, 16, 10) * 3
    ci = _random_collab(16, 5, 11)
    idx, g = orc.route(l, 4, ci)
    kept = np.take_along_axis(l.astype(np.float64), idx, axis=1)
    np.testing.assert_allclose(g, softmax(kept, axis=1), rtol=1e-13)
    # and equal to the full softmax restricted to the kept experts, renormalised
    full = softmax(l.astype(np.float64), axis=1)
    sel = np.take_along_axis(full, idx, axis=1)
    np.testing.assert_allclose(g, sel / sel.sum(1, keepdims=True), rtol=1e-12)


def test_non_finite_logits(orc):
    # The scan "first allowed expert stands unless a later one is strictly larger", walked here
    # expert by expert in plain Python: a NaN is selected only where it is the first allowed one.
    # Gates: the library softmax of the kept logits, which is NaN for a row whose largest kept
    # logit is +inf or a NaN (inf - inf), and one-hot never.
    from scipy.special import softmax
    E, K, Tc = 10, 3, 5
    l = _small_logits(300, E, 21, ties=True)
    l[::3, 0] = np.nan
    l[1::4, 6] = np.nan
    l[2::5, 3] = np.inf
    l[5::7, 8] = -np.inf
    l[11] = np.nan
    l[12] = -np.inf
    ci = _random_collab(E, Tc, 22)

    def scan(row, allowed):
        best = None
        for e in allowed:
            if best is None or row[e] > row[best]:
                best = e
        return best

    for lists in (ci, None):
        idx, g = orc.route(l, K, lists)
        for t in range(l.shape[0]):
            e0 = scan(l[t], range(E))
            left = sorted(int(v) for v in (lists[e0] if lists is not None else range(E)) if v != e0)
            want = [e0]
            for _ in range(K - 1):
                e = scan(l[t], left)
                want.append(e)
                left.remove(e)
            assert list(idx[t]) == want, (t, list(idx[t]), want)
        kept = np.take_along_axis(l.astype(np.float64), idx, axis=1)
        with np.errstate(invalid="ignore"):
            ref = softmax(kept, axis=1)
        assert np.array_equal(np.isnan(g), np.isnan(ref))
        ok = ~np.isnan(ref)
        np.testing.assert_allclose(g[ok], ref[ok], rtol=1e-13)
        assert np.isnan(g[np.isposinf(kept[:, 0])]).all() and np.isnan(g[11]).all() and np.isnan(g[12]).all()


# ---------------- Eq. 2 / Eq. 4: profiling ----------------

def test_coactivation_is_MtM(orc):
    E, K = 20, 4
    l = _small_logits(3000, E, 12)
    idx, _ = orc.route(l, K)
    Cm = orc.coactivation(idx, E)
    M = np.zeros((l.shape[0], E), dtype=np.int64)
    np.put_along_axis(M, idx, 1, axis=1)
    assert np.array_equal(Cm, M.T @ M)                                 # P4
    assert np.array_equal(Cm, Cm.T)                                    # P3
    counts, _, _, _ = orc.permute(idx, E)
    assert np.array_equal(np.diag(Cm), counts)
    assert np.array_equal(Cm.sum(1) - np.diag(Cm), (K - 1) * np.diag(Cm))
    assert Cm.sum() == l.shape[0] * K * K
    # accumulation over batches
    C2 = orc.coactivation(idx[:1000], E)
    C2 = orc.coactivation(idx[1000:], E, C2)
    assert np.array_equal(C2, Cm)


def test_collaborators_sorted_self_excluded(orc):
    rng = np.random.default_rng(13)
    E = 12
    Cm = rng.integers(0, 5, size=(E, E))
    Cm = Cm + Cm.T
    Cm[3, :] = 0
    Cm[:, 3] = 0                                                       # an expert never used
    np.fill_diagonal(Cm, 1000)                                         # diagonal is the row maximum
    for Tc in (1, 4, E - 1, E + 5):
        ci = orc.collaborators(Cm, Tc)
        n = min(Tc, E - 1)
        assert ci.shape == (E, n)
        for i in range(E):
            ref = sorted((j for j in range(E) if j != i), key=lambda j: (-Cm[i, j], j))[:n]
            assert list(ci[i]) == ref
    ci = orc.collaborators(Cm, 4)
    assert list(ci[3]) == [0, 1, 2, 4]                                 # all-zero row: index order


def test_reprofile_under_c2r_support(orc):
    # Fig. 2(b): under C2R a pair (i, j) can only co-occur if some expert's
    # {itself} + list contains both (P5); with short lists most entries are 0.
    E, K, Tc = 16, 3, 3
    l = _small_logits(5000, E, 14)
    idx0, _ = orc.route(l, K)
    ci = orc.collaborators(orc.coactivation(idx0, E), Tc)
    idx1, _ = orc.route(l, K, ci)
    C1 = orc.coactivation(idx1, E)
    allowed = np.zeros((E, E), dtype=bool)
    for e0 in range(E):
        grp = [e0] + list(ci[e0])
        for i in grp:
            for j in grp:
                allowed[i, j] = True
    assert not np.any((C1 > 0) & ~allowed)
    assert (C1 == 0).sum() > (orc.coactivation(idx0, E) == 0).sum()


# ---------------- dispatch / combine ----------------

def test_permute_is_stable_sort(orc):
    E, K = 10, 3
    l = _small_logits(700, E, 15)
    idx, _ = orc.route(l, K)
    counts, offsets, perm, inv = orc.permute(idx, E)
    flat = idx.reshape(-1)
    assert np.array_equal(perm, np.argsort(flat, kind="stable"))       # library stable sort
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(inv[perm], np.arange(perm.size))             # P8
    # local subset: experts 2..5 local, renumbered
    ls = np.full(E, -1, dtype=np.int32)
    ls[2:6] = np.arange(4)
    counts, offsets, perm, inv = orc.permute(idx, E, ls, 4)
    keep = np.flatnonzero((flat >= 2) & (flat < 6))
    assert np.array_equal(perm, keep[np.argsort(flat[keep], kind="stable")])
    assert np.all(inv[np.setdiff1d(np.arange(flat.size), keep)] == -1)
    assert np.array_equal(inv[perm], np.arange(perm.size))


def test_combine_definition(orc):
    rng = np.random.default_rng(16)
    T, K, d, E = 50, 3, 7, 6
    idx, g = orc.route(_small_logits(T, E, 17), K)
    _, _, perm, inv = orc.permute(idx, E)
    yp = rng.standard_normal((T * K, d))
    ys = rng.standard_normal((T, d))
    ref = np.einsum("tk,tkd->td", g, yp[inv.reshape(T, K)]) + ys
    np.testing.assert_allclose(orc.combine(yp, g, inv, T, K, ys), ref, rtol=1e-13, atol=1e-14)
    # identity experts, K = 1: combine(permute(x)) == x exactly
    idx1, g1 = orc.route(_small_logits(T, E, 18), 1)
    _, _, perm1, inv1 = orc.permute(idx1, E)
    x = rng.standard_normal((T, d))
    assert np.array_equal(orc.combine(x[perm1], g1, inv1, T, 1), x)
    # non-local slots (-1) contribute nothing
    inv2 = inv.copy()
    inv2[::2] = -1
    m = (inv2.reshape(T, K) >= 0)
    ref2 = np.einsum("tk,tkd->td", g * m, yp[np.maximum(inv2, 0).reshape(T, K)])
    np.testing.assert_allclose(orc.combine(yp, g, inv2, T, K), ref2, rtol=1e-13, atol=1e-14)


# ---------------- expert FFN ----------------

def _dense_swiglu(x, wg, wu, wd):
    x = x.astype(np.float64)
    a = x @ wg.astype(np.float64).T
    u = x @ wu.astype(np.float64).T
    return (a / (1.0 + np.exp(-a)) * u) @ wd.astype(np.float64).T


def test_expert_ffn_dense_special_case(orc):
    # P9: one expert, every row -> a dense SwiGLU MLP via library fp64 matmuls.
    rng = np.random.default_rng(19)
    n, d, F = 33, 24, 40                       # d != F: a transposed weight fails
    x = rng.standard_normal((n, d)).astype(np.float32)
    wg = rng.standard_normal((1, F, d)).astype(np.float32) * 0.3
    wu = rng.standard_normal((1, F, d)).astype(np.float32) * 0.3
    wd = rng.standard_normal((1, d, F)).astype(np.float32) * 0.3
    y = orc.expert_ffn_rows(x, np.zeros(n, np.int32), wg, wu, wd)
    np.testing.assert_allclose(y, _dense_swiglu(x, wg[0], wu[0], wd[0]), rtol=1e-12, atol=1e-13)
    # gate and up are not interchangeable: silu is applied to the gate branch
    y_sw = orc.expert_ffn_rows(x, np.zeros(n, np.int32), wu, wg, wd)
    assert np.abs(y_sw - y).max() > 1e-3


def test_expert_ffn_block_structure_and_layer(orc):
    rng = np.random.default_rng(20)
    T, d, F, E, K = 40, 16, 24, 5, 2
    x = rng.standard_normal((T, d)).astype(np.float32)
    wg = rng.standard_normal((E, F, d)).astype(np.float32) * 0.3
    wu = rng.standard_normal((E, F, d)).astype(np.float32) * 0.3
    wd = rng.standard_normal((E, d, F)).astype(np.float32) * 0.3
    idx, g = orc.route(_small_logits(T, E, 21), K)
    counts, offsets, perm, inv = orc.permute(idx, E)
    x_perm = x[perm // K]
    eor = idx.reshape(-1)[perm]
    y_perm = orc.expert_ffn_rows(x_perm, eor, wg, wu, wd)
    for e in range(E):
        sl = slice(offsets[e], offsets[e + 1])
        np.testing.assert_allclose(y_perm[sl], _dense_swiglu(x_perm[sl], wg[e], wu[e], wd[e]),
                                   rtol=1e-12, atol=1e-13)
    sh = tuple(rng.standard_normal(s).astype(np.float32) * 0.3 for s in ((1, 30, d), (1, 30, d), (1, d, 30)))
    y_sh = _dense_swiglu(x, sh[0][0], sh[1][0], sh[2][0])
    y = orc.combine(y_perm, g, inv, T, K, y_sh)
    toks = np.arange(T)
    y2 = orc.layer_tokens(x, toks, idx, g, wg, wu, wd, E, shared=sh)
    np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-13)
    # token subset + local experts only
    ls = np.array([-1, 0, 1, -1, 2], dtype=np.int32)
    sub = np.array([3, 17, 39])
    y3 = orc.layer_tokens(x, sub, idx, g, wg[[1, 2, 4]], wu[[1, 2, 4]], wd[[1, 2, 4]], E, local_slot=ls)
    ref = np.zeros((3, d))
    for i, t in enumerate(sub):
        for s in range(K):
            e = idx[t, s]
            if ls[e] >= 0:
                ref[i] += g[t, s] * _dense_swiglu(x[t:t + 1], wg[e], wu[e], wd[e])[0]
    np.testing.assert_allclose(y3, ref, rtol=1e-12, atol=1e-13)


# ---------------- Sec. 3.4 / Sec. 4.1 host-side counts ----------------

def test_distinct_devices_and_redundancy(orc):
    E, K = 12, 4
    idx, _ = orc.route(_small_logits(500, E, 22), K)
    dev = wl.device_map(E, 4)
    dd = orc.distinct_devices(idx, dev)
    assert list(dd) == [len({int(dev[e]) for e in row}) for row in idx]
    assert orc.redundancy(np.full(10, 1), 4) == 0.75       # all four copies on one device
    assert orc.redundancy(np.full(10, 4), 4) == 0.0


def test_dedup_dispatch_properties(orc):
    # Sec. 3.4: one copy of a token per device that hosts one of its experts.  Pinned by the
    # definition written out with Python sets, by the copy count = sum of distinct devices
    # (pinned above), and by three closed forms.
    E, K, n_dev = 12, 4, 4
    idx, _ = orc.route(_small_logits(300, E, 23), K)
    idx[5, 2] = -1                                           # an empty slot sends nothing
    dev = wl.device_map(E, n_dev)
    counts, offsets, tok, row = orc.dedup_dispatch(idx, E, dev, n_dev)
    pairs = sorted({(int(dev[e]), t) for t in range(idx.shape[0]) for e in idx[t] if e >= 0})
    assert [(g, t) for g in range(n_dev) for t in tok[offsets[g]:offsets[g + 1]]] == pairs
    assert list(counts) == [sum(1 for g, _ in pairs if g == q) for q in range(n_dev)]
    assert offsets[0] == 0 and offsets[-1] == len(pairs) and np.all(np.diff(offsets) == counts)
    row = row.reshape(idx.shape)
    for t in range(idx.shape[0]):
        for s in range(K):
            e = idx[t, s]
            if e < 0:
                assert row[t, s] == -1
            else:                                            # the copy slot s uses is (device of e, t)
                assert tok[row[t, s]] == t and offsets[dev[e]] <= row[t, s] < offsets[dev[e] + 1]
    idx[5, 2] = 0
    _, offsets, tok, _ = orc.dedup_dispatch(idx, E, dev, n_dev)
    assert len(tok) == orc.distinct_devices(idx, dev).sum()
    # closed forms: one device -> every token once; one expert per device -> nothing saved;
    # K = 1 -> the send list is the tokens sorted by their expert's device
    _, _, tok1, row1 = orc.dedup_dispatch(idx, E, np.zeros(E, dtype=np.int32), 1)
    assert list(tok1) == list(range(idx.shape[0])) and np.all(row1.reshape(idx.shape) == np.arange(idx.shape[0])[:, None])
    _, _, tokE, _ = orc.dedup_dispatch(idx, E, np.arange(E, dtype=np.int32), E)
    assert len(tokE) == idx.size
    one = idx[:, :1].copy()
    _, _, tokK, _ = orc.dedup_dispatch(one, E, dev, n_dev)
    assert list(tokK) == sorted(range(one.shape[0]), key=lambda t: (dev[one[t, 0]], t))


def test_two_level_combine_equals_combine(orc):
    # adding a token's expert outputs per device first and the per-device partial rows second
    # is the same sum: exact on integer-valued inputs, whatever the grouping
    rng = np.random.default_rng(24)
    T, E, K, d, n_dev = 200, 10, 3, 6, 5
    idx, _ = orc.route(_small_logits(T, E, 25), K)
    g = rng.integers(1, 5, size=(T, K)).astype(np.float64)
    ls = np.arange(E, dtype=np.int32)
    ls[3] = -1
    ls[4:] -= 1                                              # expert 3 is not computed here
    _, _, perm, inv = orc.permute(idx, E, ls, E - 1)
    yp = rng.integers(-8, 9, size=(len(perm), d)).astype(np.float64)
    ys = rng.integers(-8, 9, size=(T, d)).astype(np.float64)
    dev = wl.device_map(E, n_dev)
    _, _, tok, row = orc.dedup_dispatch(idx, E, dev, n_dev)
    part = orc.combine_partial(yp, g, inv, row, T, K, len(tok))
    for shared in (None, ys):
        assert np.array_equal(orc.combine_copies(part, row, T, K, shared), orc.combine(yp, g, inv, T, K, shared))
    # a copy's partial row holds exactly the terms of the experts on its device
    r = row.reshape(T, K)
    t, s = 17, 1
    same = [q for q in range(K) if r[t, q] == r[t, s] and inv[t * K + q] >= 0]
    assert np.array_equal(part[r[t, s]], sum(g[t, q] * yp[inv[t * K + q]] for q in same))


def test_place_experts_recovers_planted_groups(orc):
    # Sec. 3.4 co-location (greedy reading).  Pins: a block-structured C gives back its blocks;
    # every expert is placed once and devices are filled in order up to ceil(E/n_dev); on small
    # clear-cut inputs the greedy partition keeps as much co-activation inside devices as the
    # best balanced partition found by enumeration.
    rng = np.random.default_rng(31)
    for E, n_dev in ((12, 4), (60, 4), (15, 5)):
        cap = E // n_dev
        label = rng.permutation(np.repeat(np.arange(n_dev), cap))
        Cm = (label[:, None] == label[None, :]).astype(np.int64) * 100 + rng.integers(0, 10, size=(E, E))
        Cm = Cm + Cm.T
        dev = orc.place_experts(Cm, n_dev)
        assert sorted(np.bincount(dev, minlength=n_dev)) == [cap] * n_dev
        for g in range(n_dev):                               # a device holds exactly one planted group
            assert len(set(label[dev == g])) == 1
    dev = orc.place_experts(np.ones((10, 10), dtype=np.int64), 4)   # all ties: index order, 3+3+3+1
    assert list(dev) == [0, 0, 0, 1, 1, 1, 2, 2, 2, 3]
    E = 8
    label = np.array([0, 1, 0, 1, 1, 0, 0, 1])
    Cm = (label[:, None] == label[None, :]).astype(np.int64) * 20 + rng.integers(0, 4, size=(E, E))
    Cm = Cm + Cm.T
    inside = lambda d: sum(Cm[i, j] for i in range(E) for j in range(E) if i != j and d[i] == d[j])
    best = max(inside(np.isin(np.arange(E), c).astype(int)) for c in itertools.combinations(range(E), 4))
    assert inside(orc.place_experts(Cm, 2)) == best
    # the first expert of device 0 is the one that collaborates most overall (lower index on ties)
    Cm = rng.integers(0, 50, size=(9, 9)); Cm = Cm + Cm.T
    off = Cm.sum(1) - np.diag(Cm)
    assert orc.place_experts(Cm, 3)[int(np.argmax(off))] == 0


def test_table3_speedup_product(orc):
    # P10: the printed speed-ups are the products of the printed shares (inputs are rounded,
    # so agree to 0.1 point)
    with open(os.path.join(GOLDEN, "table3_ep_scaling.txt")) as f:
        rows = [[float(v) for v in l.split()] for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for ep, red, a2a, sp in rows:
        assert abs(100 * orc.estimated_speedup(a2a / 100, red / 100) - sp) <= 0.1, ep


def test_collaboration_degree_closed_forms(orc):
    N = 9
    Cm = np.ones((N, N)) * 7
    np.fill_diagonal(Cm, 1e6)                   # diagonal must not enter
    np.testing.assert_allclose(orc.collaboration_degree(Cm), np.log(N - 1), rtol=1e-14)
    Cm = np.zeros((N, N))
    for i in range(N):
        Cm[i, (i + 1) % N] = 5                  # one collaborator each: fully specialised
    assert np.all(orc.collaboration_degree(Cm) == 0)


def test_collaboration_degree_hand_worked_rows(orc):
    # Eq. 3 on rows that are neither uniform nor one-hot, worked by hand.  Expert 0 meets the
    # others 2, 1 and 1 times: p = 1/2, 1/4, 1/4 and
    #   P = (1/2) ln 2 + 2 (1/4) ln 4 = (3/2) ln 2.
    # Expert 1 meets only expert 0: P = 0.  Experts 2 and 3 meet others 1 and 3 times:
    #   p = 1/4, 3/4 and P = (1/4) ln 4 + (3/4) ln (4/3) = ln 4 - (3/4) ln 3.
    # The large diagonal (an expert's own token count) must enter neither sum.
    Cm = np.array([[100, 2, 1, 1],
                   [2, 50, 0, 0],
                   [1, 0, 7, 3],
                   [1, 0, 3, 9]])
    want = [1.5 * math.log(2.0), 0.0, math.log(4.0) - 0.75 * math.log(3.0), math.log(4.0) - 0.75 * math.log(3.0)]
    np.testing.assert_allclose(orc.collaboration_degree(Cm), want, rtol=1e-15, atol=0)
    # a mistake that keeps the diagonal in the normalisation gives a different, smaller number
    assert abs(want[0] - 1.0397207708399179) < 1e-15


def test_place_experts_hand_worked_pick_sequence(orc):
    # Sec. 3.4 co-location (greedy reading) on a generic symmetric matrix, picks worked by hand.
    # Off-diagonal row sums: 15, 13, 12, 13, 8, 13.  The diagonal (50 for expert 1) is ignored.
    Cm = np.array([[1, 5, 1, 0, 2, 7],
                   [5, 50, 3, 4, 0, 1],
                   [1, 3, 1, 6, 2, 0],
                   [0, 4, 6, 1, 1, 2],
                   [2, 0, 2, 1, 1, 3],
                   [7, 1, 0, 2, 3, 1]], dtype=np.int64)
    assert np.array_equal(Cm, Cm.T)
    # three devices of two: device 0 starts with expert 0 (row sum 15) and takes expert 5 (7 with 0);
    # device 1 starts with expert 1 (row sums over ALL other experts: 13 ties with expert 3's 13,
    # lower index wins) and takes expert 3 (4 with 1, against 3 for expert 2); experts 2, 4 remain.
    assert list(orc.place_experts(Cm, 3)) == [0, 1, 2, 1, 2, 0]
    # two devices of three: {0, 5} then the largest TOTAL with both: expert 1 (5 + 1 = 6) against
    # expert 4 (2 + 3 = 5), expert 3 (0 + 2) and expert 2 (1 + 0)
    assert list(orc.place_experts(Cm, 2)) == [0, 0, 1, 1, 1, 0]
    # six devices of one: descending row sum, ties to the lower index: 0, then 1, 3, 5 (13 each), 2, 4
    assert list(orc.place_experts(Cm, 6)) == [0, 1, 4, 2, 5, 3]
