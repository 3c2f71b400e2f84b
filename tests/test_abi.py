"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    from paper_2504_01337_amd import c2r
    if not os.path.exists(c2r.LIB_PATH):
        pytest.fail("libc2r_hip.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    return c2r


def test_header_symbols_exported():
    c2r = _lib()
    with open(os.path.join(ROOT, "include", "c2r.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(c2r_[a-z0-9_]+)\s*\(", text)))
    assert declared == sorted(c2r.EXPORTS)
    L = c2r.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert c2r.version() >= 100
    assert c2r.route_chunk() == 256


def test_every_entry_point_is_documented_with_its_passage():
    # the comment in front of each declaration cites the passage of the paper that defines the operation
    # (a section, an equation or a table) - or, for the calls no passage defines, says what they are for
    with open(os.path.join(ROOT, "include", "c2r.h")) as f:
        text = f.read()
    no_passage = {"c2r_version": "version", "c2r_route_chunk": "order", "c2r_workspace_bytes": "scratch",
                  "c2r_permute_noalloc": "cannot allocate"}
    for m in re.finditer(r"/\*(.*?)\*/\s*(?:int|size_t)\s+(c2r_[a-z0-9_]+)\s*\(", text, flags=re.S):
        comment, name = m.group(1), m.group(2)
        comment = comment.split("/*")[-1]
        if name in no_passage:
            assert no_passage[name] in comment, name
        else:
            assert re.search(r"Sec\. \d|Eq\. \d|Table \d", comment), name
        assert len(comment.strip()) > (40 if name in no_passage else 80), name


def test_workspace_query_is_host_only():
    c2r = _lib()
    assert c2r.workspace_bytes(c2r.STAGE_COACTIVATION, 1000, 64, 8, 2, 0, c2r.F32) == 0
    # route scratch: one fp32 per (chunk, expert, token padded to 64)
    assert c2r.workspace_bytes(c2r.STAGE_ROUTE, 8192, 2048, 60, 4, 0, c2r.BF16) == 8 * 60 * 8192 * 4
    # (+ a zero-padded copy of W_g when E is not a multiple of 4)
    assert c2r.workspace_bytes(c2r.STAGE_ROUTE, 64, 256, 7, 2, 0, c2r.F32) == 1 * 8 * 64 * 4 + 256 * 8 * 4
    assert c2r.workspace_bytes(c2r.STAGE_ROUTE, 100, 256, 8, 2, 0, c2r.F32) == 1 * 8 * 128 * 4
    assert c2r.workspace_bytes(c2r.STAGE_EXPERT_FFN, 32768, 2048, 60, 1, 1408, c2r.BF16) == 32768 * 1408 * 2
    assert c2r.workspace_bytes(c2r.STAGE_EXPERT_FFN, 100, 4096, 16, 1, 688, c2r.BF16) == 100 * 704 * 2 + 0 * 256
    assert c2r.workspace_bytes(c2r.STAGE_EXPERT_FFN, 64, 256, 8, 1, 520, c2r.F32) == 64 * 520 * 4
    assert c2r.workspace_bytes(c2r.STAGE_PERMUTE, 8192, 2048, 60, 4, 0, c2r.BF16) > 0


def test_argument_errors_before_launch():
    # every call below is rejected on the host: nothing is enqueued, no GPU is needed
    c2r = _lib()
    L = c2r.lib()
    p = ctypes.c_void_p(0x1000)      # never dereferenced by the host checks
    null = ctypes.c_void_p(0)
    assert L.c2r_route(p, 1, p, null, 16, 64, 8, 9, null, 0, p, p, null, p, 1 << 20, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_route(p, 1, p, null, 16, 64, 8, 4, p, 2, p, p, null, p, 1 << 20, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_route(p, 1, p, null, 16, 64, 65, 4, null, 0, p, p, null, p, 1 << 20, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_route(p, 1, p, null, 16, 60, 8, 2, null, 0, p, p, null, p, 1 << 20, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_route(p, 1, p, null, 16, 64, 8, 2, null, 0, p, p, null, null, 0, null) == c2r.ERR_WORKSPACE
    assert L.c2r_route(null, 1, p, null, 16, 64, 8, 2, null, 0, p, p, null, p, 1 << 20, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_build_coactivation(p, 16, 2, 65, p, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_build_coactivation(null, 16, 2, 8, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_collaborators(null, 8, 4, p, null, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_permute(p, 1, p, 16, 64, 8, 2, null, 4, p, p, p, p, p, p, 1 << 20, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_expert_ffn(p, 1, p, 4, 64, 64, 60, p, p, p, p, p, 1 << 20, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_expert_ffn(p, 1, p, 4, 64, 64, 64, p, p, p, p, null, 0, null) == c2r.ERR_WORKSPACE
    assert L.c2r_combine(p, 1, p, p, 16, 60, 2, null, p, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_combine(null, 1, p, p, 16, 64, 2, null, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_expert_ffn_gate_up_gather(p, 0, p, 16, 2, p, 4, 32, 64, 64, p, p, p, null) == c2r.ERR_UNSUPPORTED  # fp32
    assert L.c2r_expert_ffn_gate_up_gather(p, 1, null, 16, 2, p, 4, 32, 64, 64, p, p, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_expert_ffn_gather(p, 0, p, 16, 2, p, 4, 32, 64, 64, p, p, p, p, p, 1 << 20, null) == c2r.ERR_UNSUPPORTED  # fp32
    assert L.c2r_expert_ffn_gather(p, 1, p, 16, 2, p, 4, 32, 72, 64, p, p, p, p, p, 1 << 20, null) == c2r.ERR_UNSUPPORTED  # d % 64
    assert L.c2r_expert_ffn_gather(p, 1, null, 16, 2, p, 4, 32, 64, 88, p, p, p, p, p, 1 << 20, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_expert_ffn_gather(p, 1, p, 16, 2, p, 4, 32, 64, 88, p, p, p, p, null, 0, null) == c2r.ERR_WORKSPACE
    assert L.c2r_place_experts(p, 65, 4, p, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_place_experts(null, 8, 4, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_place_experts(p, 8, 0, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_dedup_dispatch(p, 16, 2, 8, p, 65, p, p, p, p, p, 1 << 20, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_dedup_dispatch(p, 16, 2, 8, null, 4, p, p, p, p, p, 1 << 20, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_dedup_dispatch(p, 16, 2, 8, p, 4, p, p, p, p, null, 0, null) == c2r.ERR_WORKSPACE
    assert L.c2r_combine_partial(p, 1, p, p, p, p, p, 16, 32, 60, 2, p, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_combine_partial(p, 1, p, p, p, p, null, 16, 32, 64, 2, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_combine_copies(p, 1, null, 16, 32, 64, 2, null, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_collaboration_degree(p, 65, p, null) == c2r.ERR_UNSUPPORTED
    assert L.c2r_collaboration_degree(p, 8, null, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_distinct_devices(p, 16, 2, 8, p, 9, 4, null, p, null) == c2r.ERR_UNSUPPORTED   # more than 8 maps
    assert L.c2r_distinct_devices(p, 16, 2, 8, p, 2, 4, null, null, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_distinct_devices(p, 16, 2, 8, p, 2, 4, null, ctypes.c_void_p(0x1004), null) == c2r.ERR_INVALID_ARG
    assert c2r.workspace_bytes(c2r.STAGE_DEDUP_DISPATCH, 5000, 0, 4, 4, 0, c2r.F32) == 256
    assert L.c2r_expert_ffn_gate_up_with_shared(p, 0, p, 16, 2, p, 4, 32, 64, 64, p, p, p, 64, p, p, p, null) == c2r.ERR_UNSUPPORTED  # fp32
    assert L.c2r_expert_ffn_gate_up_with_shared(p, 1, p, 16, 2, p, 4, 32, 64, 64, p, p, p, 72, p, p, p, null) == c2r.ERR_UNSUPPORTED  # F_shared % 64
    assert L.c2r_expert_ffn_gate_up_with_shared(p, 1, p, 16, 2, p, 4, 32, 64, 64, p, p, p, 64, null, p, p, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_expert_ffn_down_with_shared(p, 1, p, 4, 32, 64, 64, p, p, 16, 64, p, p, null, null) == c2r.ERR_INVALID_ARG
    assert L.c2r_expert_ffn_down_with_shared(p, 1, p, 4, 32, 64, 88, p, p, 16, 64, p, p, p, null) == c2r.ERR_UNSUPPORTED  # F % 64
    assert L.c2r_profile_from_logits(p, 16, 8, 2, null, 0, null, null, null, null) == c2r.ERR_INVALID_ARG      # no C
    assert L.c2r_profile_from_logits(p, 16, 6, 2, null, 0, null, null, p, null) == c2r.ERR_UNSUPPORTED         # E % 4 without outputs
    assert L.c2r_profile_from_logits(p, 16, 8, 5, null, 0, null, null, p, null) == c2r.ERR_UNSUPPORTED         # K > 4 without outputs
    assert L.c2r_profile_from_logits(p, 16, 8, 9, null, 0, p, p, p, null) == c2r.ERR_INVALID_ARG               # K > E
    # the allocation-free dispatch rejects what its static array cannot hold
    assert L.c2r_permute_noalloc(p, 1, p, (1 << 20) + 1, 64, 8, 4, null, 8, p, p, p, p, p, null) == c2r.ERR_UNSUPPORTED
    # empty batches are fine and launch nothing
    assert L.c2r_route(null, 1, null, null, 0, 64, 8, 2, null, 0, null, null, null, null, 0, null) == c2r.OK
    assert L.c2r_combine(null, 1, null, null, 0, 64, 2, null, null, null) == c2r.OK


def test_workload_rounding_and_shapes():
    import numpy as np
    from paper_2504_01337_amd import workloads as wl
    a = np.random.default_rng(0).standard_normal(1 << 16, dtype=np.float32)
    r = wl.round_bf16(a)
    assert np.array_equal(r, wl.round_bf16_reference(a))
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    w = wl.scaled(wl.WORKLOADS["C3"], T=64)
    Wg, b = wl.router(w)
    assert Wg.shape == (2048, 60) and b.shape == (60,) and abs(float(b.mean())) < 1e-6
    assert wl.hidden(w).shape == (64, 2048)
    assert list(wl.local_slot(wl.WORKLOADS["C5"])[13:17]) == [13, 14, -1, -1]
    x, W = wl.exact_arithmetic_router(8, 64, 5)
    assert np.all(x == np.round(x)) and np.all(W * 8 == np.round(W * 8))
