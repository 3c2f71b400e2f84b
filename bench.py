#!/usr/bin/env python3
"""Benchmark of the C2R MoE layer hot path on one MI355X.

A step is one pass of the whole path (route -> permute -> grouped SwiGLU expert
FFN (+ shared expert) -> combine) over one batch of seeded synthetic tokens that
is already resident in HBM.  Prints ONE JSON line: layer tokens/s, the roofline
of the dominant kernel (the gate/up MFMA pass of the expert FFN) measured live
with events on the launch stream, per-stage times, and the CPU oracle timed on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm_GBps": 8000.0, "mfma_bf16_TFLOPs": 2500.0, "valu_f32_TFLOPs": 157.3}


def _benchaid():
    """The benchmark's own probe library (not part of the C2R ABI): a pure bf16 MFMA loop."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_2504_01337_amd", "bench_aids", "libc2r_benchaid.so")
    if not os.path.exists(path):
        return None
    L = C.CDLL(path)
    L.benchaid_probe_mfma_bf16.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double),
                                           C.c_void_p, C.c_void_p]
    L.benchaid_probe_mfma_bf16.restype = C.c_int
    return L


def measured_ceilings(torch):
    """Ceilings of this box: the matrix pipe on zero / random operands (with the shader clock the
    loop ran at) and a plain device copy."""
    import ctypes as C
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    res = {}
    aid = _benchaid()
    if aid is not None:
        out_p = torch.empty(1024 * 512, dtype=torch.float32, device="cuda")
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        g = torch.Generator(device="cpu").manual_seed(7)

        def probe(ops, iters, clk):
            fl = C.c_double(0.0)
            rc = aid.benchaid_probe_mfma_bf16(C.c_void_p(ops.data_ptr()), iters, 1024, C.c_void_p(out_p.data_ptr()),
                                              C.byref(fl), C.c_void_p(clk.data_ptr()) if clk is not None else None, st)
            assert rc == 0, rc
            return fl.value

        for name, ops in (("mfma_bf16_zero_operands_TFLOPs", torch.zeros(1024 * 8, dtype=torch.bfloat16)),
                          ("mfma_bf16_random_operands_TFLOPs",
                           (torch.rand(1024 * 8, generator=g) * 2 - 1).to(torch.bfloat16))):
            ops = ops.cuda()
            clk = torch.zeros(2, dtype=torch.int64, device="cuda")
            probe(ops, 2000, None)
            e0.record()
            fl = probe(ops, 20000, clk)
            e1.record()
            torch.cuda.synchronize()
            res[name] = fl / e0.elapsed_time(e1) / 1e9
            cyc, ticks = clk.tolist()   # shader cycles / 100 MHz ticks of the loop: the clock under this load
            res[name.replace("_TFLOPs", "_shader_clock_GHz")] = cyc / (ticks / 1e8) / 1e9 if ticks else None
    src = torch.full(((512 << 20) // 4,), 1.0, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    res["copy_read_plus_write_GBps"] = 5 * 2 * (512 << 20) / e0.elapsed_time(e1) / 1e6
    return res


class ColdTimer:
    """Times one launch from cold memory.  Two protocols, because they differ by a factor of two on
    this chip: "after_write" = a 512 MiB fill before the launch (the memory-side cache is then full
    of dirty lines whose write-back competes with the launch's own traffic: even a plain device copy
    runs at 3.7 instead of 5.4 TB/s behind it); "after_read" = that fill followed by a 1 GiB read
    (the caches then hold clean lines of an unrelated buffer).  A plain device-to-device copy is
    timed the same way as the yardstick of each protocol."""

    def __init__(self, torch):
        self.torch = torch
        self.w = torch.empty((512 << 20) // 4, dtype=torch.float32, device="cuda")
        self.r = torch.ones((1024 << 20) // 4, dtype=torch.float32, device="cuda")
        self.cs = torch.ones((96 << 20) // 4, dtype=torch.float32, device="cuda")
        self.cd = torch.empty_like(self.cs)

    def flush(self, mode):
        self.w.fill_(1.0)
        if mode == "after_read":
            self.r.sum()

    def time(self, prepare, launch, n_it, mode):
        """median microseconds of launch() behind prepare() (re-creates the launch's inputs) + flush"""
        torch = self.torch
        ts = []
        for _ in range(n_it):
            prepare()
            self.flush(mode)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            launch()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3)
        ts.sort()
        return ts[len(ts) // 2]

    def copy_yardstick(self, n_it):
        out = {}
        for mode in ("after_write", "after_read"):
            us = self.time(lambda: None, lambda: self.cd.copy_(self.cs), n_it, mode)
            out[mode] = {"us": us, "GBps": 2 * self.cs.numel() * 4 / us / 1e3}
        return out


def bench_profiling(args, w, torch, np, c2r, wl):
    """Workload C4: the offline profiling of Sec. 3.2 / Sec. 3.3 step 1 on a stored logit stream.
    A step = C zeroed -> conventional top-K of every token and its pair counts (Eq. 2) in one launch
    (c2r_profile_from_logits; the selections themselves are not written) -> collaborator lists (Eq. 4,
    c2r_collaborators).  --separate-count runs c2r_route_from_logits and c2r_build_coactivation instead."""
    t_gen = time.time()
    lg_h = wl.direct_logits(w)
    lg = torch.from_numpy(lg_h).cuda()
    T, E, K, Tc = w.T, w.E, w.K, w.Tc
    idx = torch.empty((T, K), dtype=torch.int32, device="cuda")
    gates = torch.empty((T, K), dtype=torch.float32, device="cuda")
    Cm = torch.zeros((E, E), dtype=torch.int32, device="cuda")
    lists = (torch.empty((E, min(Tc, E - 1)), dtype=torch.int32, device="cuda"),
             torch.empty((E,), dtype=torch.int64, device="cuda"))
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen
    mk = lambda: torch.cuda.Event(enable_timing=True)
    fused = not args.separate_count
    names = ("zero_C", "select_and_count", "collaborators") if fused else ("select", "zero_C", "coactivation", "collaborators")
    dom = "select_and_count" if fused else "select"

    def step(tr=None):
        def run(name, fn):
            if tr is not None and name in tr:
                tr[name][0].record()
            fn()
            if tr is not None and name in tr:
                tr[name][1].record()
        if fused:   # one launch selects and counts; the selections themselves are not written
            run("zero_C", lambda: Cm.zero_())
            run("select_and_count", lambda: c2r.profile_from_logits(lg, K, Cm))
        else:
            run("select", lambda: c2r.route_from_logits(lg, K, None, out=(idx, gates)))
            run("zero_C", lambda: Cm.zero_())
            run("coactivation", lambda: c2r.build_coactivation(idx, E, Cm))
        run("collaborators", lambda: c2r.collaborators(Cm, Tc, out=lists))

    t_ramp, ramp_steps = time.perf_counter(), 0
    while (time.perf_counter() - t_ramp) * 1e3 < args.ramp_ms:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
        ramp_steps += 8
    for _ in range(args.warmup):
        step()
    ev_every = 4 if args.steps >= 8 else 1
    ev_dom = [{dom: (mk(), mk())} if i % ev_every == 0 else None for i in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(ev_dom[i])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    dom_ms = float(np.mean([e[dom][0].elapsed_time(e[dom][1]) for e in ev_dom if e is not None]))
    ev = [{n: (mk(), mk()) for n in names} for _ in range(args.steps)]
    for i in range(args.steps):
        step(ev[i])
    torch.cuda.synchronize()
    st_ms = {n: float(np.mean([e[n][0].elapsed_time(e[n][1]) for e in ev])) for n in names}
    # algorithmic bytes.  Separate calls: the logits are read once, indices and gates written, the
    # indices read again by the counting kernel.  Fused: the logits are read once, nothing else moves.
    sel_bytes = T * (E * 4 + K * 8)
    co_bytes = T * K * 4
    fused_bytes = T * E * 4
    # the calls of the other form, timed back to back outside the step, for the table
    def loop_ms(fn, n=10):
        a, b = mk(), mk()
        fn()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n
    if fused:
        dom_bytes, dom_kernel = fused_bytes, "route_select_rows_kernel<4, false, true>"
        stages = {"zero_C": {"ms": st_ms["zero_C"]},
                  "select_and_count": {"ms": st_ms[dom], "GBps": fused_bytes / st_ms[dom] / 1e6,
                                       "frac_hbm": fused_bytes / st_ms[dom] / 1e6 / PEAK["hbm_GBps"], "bytes": fused_bytes,
                                       "increments_per_token": K * (K + 1) // 2, "kernel": dom_kernel},
                  "collaborators": {"ms": st_ms["collaborators"], "bound": "latency (60 x 60 integers)"}}
        sel_ms = loop_ms(lambda: c2r.route_from_logits(lg, K, None, out=(idx, gates)))
        co_ms = loop_ms(lambda: c2r.build_coactivation(idx, E, Cm))
        stages["separate_calls_outside_the_step"] = {
            "select": {"ms": sel_ms, "bytes": sel_bytes, "GBps": sel_bytes / sel_ms / 1e6,
                       "frac_hbm": sel_bytes / sel_ms / 1e6 / PEAK["hbm_GBps"], "kernel": "route_select_rows_kernel<4, false, false>"},
            "coactivation": {"ms": co_ms, "bytes": co_bytes, "GBps": co_bytes / co_ms / 1e6,
                             "frac_hbm": co_bytes / co_ms / 1e6 / PEAK["hbm_GBps"], "kernel": "coactivation_kernel<16>"}}
    else:
        dom_bytes, dom_kernel = sel_bytes, "route_select_rows_kernel<4, false, false>"
        stages = {"select": {"ms": st_ms["select"], "GBps": sel_bytes / st_ms["select"] / 1e6,
                             "frac_hbm": sel_bytes / st_ms["select"] / 1e6 / PEAK["hbm_GBps"],
                             "bytes": sel_bytes, "kernel": dom_kernel},
                  "zero_C": {"ms": st_ms["zero_C"]},
                  "coactivation": {"ms": st_ms["coactivation"], "GBps": co_bytes / st_ms["coactivation"] / 1e6,
                                   "frac_hbm": co_bytes / st_ms["coactivation"] / 1e6 / PEAK["hbm_GBps"],
                                   "bytes": co_bytes, "increments_per_token": K * (K + 1) // 2, "kernel": "coactivation_kernel<16>"},
                  "collaborators": {"ms": st_ms["collaborators"], "bound": "latency (60 x 60 integers)"}}
    isolated = None
    if args.isolate:
        cold = ColdTimer(torch)
        n_it = max(3, min(args.steps, 8))
        isolated = {"device_copy_192MB": cold.copy_yardstick(n_it)}
        for name, fn, nbytes in (("select_and_count", lambda: c2r.profile_from_logits(lg, K, Cm), fused_bytes),
                                 ("select", lambda: c2r.route_from_logits(lg, K, None, out=(idx, gates)), sel_bytes),
                                 ("coactivation", lambda: c2r.build_coactivation(idx, E, Cm), co_bytes)):
            isolated[name] = {}
            for mode in ("after_write", "after_read"):
                us = cold.time(lambda: None, fn, n_it, mode)
                isolated[name][mode + "_us"] = us
                isolated[name][mode + "_GBps"] = nbytes / us / 1e3
                isolated[name][mode + "_frac_hbm"] = nbytes / us / 1e3 / PEAK["hbm_GBps"]
                isolated[name][mode + "_frac_of_copy"] = (nbytes / us / 1e3) / isolated["device_copy_192MB"][mode]["GBps"]
        step()
        torch.cuda.synchronize()
    roofline = {"kernel": dom_kernel + (" (top-K of stored logits and Eq. 2 counts in one launch)" if fused
                                        else " (top-K of stored logits)"), "bound": "hbm",
                "achieved": dom_bytes / dom_ms / 1e6, "peak": PEAK["hbm_GBps"], "unit": "GB/s",
                "frac": dom_bytes / dom_ms / 1e6 / PEAK["hbm_GBps"], "traffic": None,
                "avg_launch_ms": dom_ms, "launches_per_step": 1,
                "launches_timed": sum(1 for e in ev_dom if e is not None),
                "algorithmic_bytes_per_launch": dom_bytes,
                "note": "the 252 MB logit stream fits the 256 MB memory-side cache, so back-to-back steps read part "
                        "of it from there; stages_from_cold_memory has the same launch from cold memory",
                "timed_by": "event pairs on the launch stream around every fourth step's launch"}
    cpu = None
    if args.cpu_sample > 0:
        from oracle import c2r_oracle as orc
        n = T   # the whole stream: the oracle's selection and counting take well under a minute
        tc = time.perf_counter()
        idx_o, _ = orc.route(lg_h[:n], K)
        C_o = orc.coactivation(idx_o, E)
        lists_o = orc.collaborators(C_o, Tc)
        tc = time.perf_counter() - tc
        # the GPU on the same sample, compared bit for bit
        ig, _ = c2r.route_from_logits(lg[:n].contiguous(), K, None)
        Cg = c2r.build_coactivation(ig, E)
        lg_lists, _ = c2r.collaborators(Cg, Tc)
        # ... and the one-launch form on the same stream
        Cf, _, _ = c2r.profile_from_logits(lg[:n].contiguous(), K, torch.zeros_like(Cg))
        cpu = {"value": n / tc, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"first {n} tokens of the logit stream through top-K, Eq. 2 and Eq. 4, {tc:.1f} s",
               "indices_bit_exact": bool(np.array_equal(ig.cpu().numpy(), idx_o)),
               "C_bit_exact": bool(np.array_equal(Cg.cpu().numpy().astype(np.int64), np.asarray(C_o, dtype=np.int64))),
               "C_of_the_one_launch_form_bit_exact": bool(np.array_equal(Cf.cpu().numpy().astype(np.int64),
                                                                         np.asarray(C_o, dtype=np.int64))),
               "lists_bit_exact": bool(np.array_equal(lg_lists.cpu().numpy(), lists_o))}
    out = {"metric": "C2R profiling tokens/sec (stored logits -> top-K -> co-activation -> collaborator lists)",
           "value": T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "clock_ramp_steps_before_warmup": ramp_steps, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
           "config": {"workload": f"{w.name}: T={T} tokens of fp32 logits over E={E}, K={K}, lists of {Tc}; "
                                  f"planted {w.groups}-group logit law"},
           "roofline": roofline, "cpu_baseline": cpu, "stages": stages, "setup_s": t_gen}
    if isolated is not None:
        out["stages_from_cold_memory"] = isolated
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--ramp-ms", type=float, default=300.0,
                    help="run the step for this long before the warm-up steps: from idle the chip takes ~50 ms "
                         "under load to settle its clocks, and steps inside that ramp run 5-15 %% slower")
    ap.add_argument("--separate-count", action="store_true",
                    help="C4: selection and co-activation counting as two calls (selections written and read back)")
    ap.add_argument("--workload", default="C3",
                    help="C1|C2|C3|C5 (C3 = Qwen1.5-MoE-A2.7B-shaped layer) or C4 (profiling only: stored "
                         "logits -> top-K -> co-activation matrix -> collaborator lists)")
    ap.add_argument("--cpu-sample", type=int, default=8192, help="tokens the CPU oracle is timed on (0: skip)")
    ap.add_argument("--separate-shared", action="store_true",
                    help="launch the shared expert's FFN passes on their own (four FFN launches per step instead of two)")
    ap.add_argument("--overlap", action="store_true",
                    help="run the shared expert on a second stream (stage spans then overlap)")
    ap.add_argument("--no-isolate", dest="isolate", action="store_false",
                    help="skip the cold pass: every stage timed on its own behind a cache flush (the 256 MB "
                         "memory-side cache otherwise serves back-to-back stages), once after a 512 MiB "
                         "write and once after that write plus a 1 GiB read")
    ap.add_argument("--hash-inputs", action="store_true", help="add the SHA-256 of every generated host array")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain device-to-device copies of known size (to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2504_01337_amd import c2r, workloads as wl

    c2r.lib()  # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        nbytes = 512 << 20
        src = torch.full((nbytes // 4,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_copy": nbytes, "bytes_written_per_copy": nbytes,
                          "copies": 10}))
        return
    w = wl.WORKLOADS[args.workload]
    if w.F == 0:
        return bench_profiling(args, w, torch, np, c2r, wl)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    sz = 2 if w.dtype == "bf16" else 4

    def dev(a, dtype="f32"):
        if a is None:
            return None
        t = torch.from_numpy(np.ascontiguousarray(a))
        if t.dtype == torch.float32 and dtype == "bf16":
            t = t.to(torch.bfloat16)
        return t.cuda()

    t_gen = time.time()
    x_h = wl.hidden(w)
    Wg_h, bias_h = wl.router(w)
    wg_h, wu_h, wd_h = wl.expert_weights(w)
    shared_h = wl.shared_expert_weights(w) if w.F_shared else None
    x_prof_h = wl.hidden(w, w.T_profile, stream=1) if w.T_profile else x_h
    x, Wg, bias = dev(x_h, w.dtype), dev(Wg_h), dev(bias_h)
    wgt = tuple(dev(a, w.dtype) for a in (wg_h, wu_h, wd_h))
    shared = None if shared_h is None else tuple(dev(a, w.dtype) for a in shared_h)
    ls_h = wl.local_slot(w)

    # offline profiling (Sec. 3.2 / Eq. 4) on the GPU: conventional top-K -> C -> lists
    idx_p, _, _ = c2r.route(dev(x_prof_h, w.dtype), Wg, bias, w.K, None)
    Cm = c2r.build_coactivation(idx_p, w.E)
    collab, _ = c2r.collaborators(Cm, w.Tc)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    L = c2r.C2RLayer(w.T, w.d, w.E, w.K, w.F, tdt, Wg, bias, collab, *wgt,
                     local_slot=dev(ls_h), E_local=w.n_local, shared=shared, overlap=args.overlap,
                     fuse_shared=False if args.separate_shared else None)
    # One step = one forward of the layer as the product enqueues it (C2RLayer.forward).
    # Each stage's start/end events are recorded on the stream the stage runs on; with
    # --overlap the spans of stages that run side by side overlap.
    stages = list(L.stage_names())
    sep_shared = bool(shared) and not L.fuse_shared      # the shared expert has launches of its own
    dom_stages = [s for s in ("ffn_gate_up", "shared_gate_up") if s in stages]   # launches of the dominant kernel
    mk = lambda: torch.cuda.Event(enable_timing=True)
    # timed region: only the dominant kernel's launches carry events, and only on every fourth
    # step (an event record holds the stream for 5.6 us: fourteen per step were 3 % of the step,
    # the four around the two gate/up launches still 1.9 %)
    ev_every = 4 if args.steps >= 8 else 1
    ev_dom = [{s: (mk(), mk()) for s in dom_stages} if i % ev_every == 0 else None for i in range(args.steps)]
    ev = [{s: (mk(), mk()) for s in stages} for _ in range(args.steps)]

    # clock ramp (not a measurement): from idle, the first ~50 ms of kernels run at lower clocks
    t_ramp = time.perf_counter()
    ramp_steps = 0
    while (time.perf_counter() - t_ramp) * 1e3 < args.ramp_ms:
        for _ in range(8):
            L.forward(x)
        torch.cuda.synchronize()
        ramp_steps += 8
    for _ in range(args.warmup):
        L.forward(x)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        L.forward(x, trace=ev_dom[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.T / (ms_per_step * 1e-3)
    dom_ms_live = {s: float(np.mean([e[s][0].elapsed_time(e[s][1]) for e in ev_dom if e is not None]))
                   for s in dom_stages}
    dom_launches_timed = sum(len(dom_stages) for e in ev_dom if e is not None)

    # stage breakdown: the same steps again, every stage bracketed by events (not part of `value`)
    for i in range(args.steps):
        L.forward(x, trace=ev[i])
    torch.cuda.synchronize()
    st_ms = {s: float(np.mean([ev[i][s][0].elapsed_time(ev[i][s][1]) for i in range(args.steps)])) for s in stages}
    # all four FFN launches: from the first one's start to the last one's end
    first = "shared_gate_up" if sep_shared else "ffn_gate_up"
    ffn_span_ms = float(np.mean([max(ev[i][first][0].elapsed_time(ev[i]["ffn_down"][1]),
                                     ev[i][first][0].elapsed_time(ev[i]["shared_down"][1]) if sep_shared else 0.0)
                                 for i in range(args.steps)]))

    # the ABI's stand-alone dispatch (index sort + row gather into x_perm), timed outside the step
    x_perm_sa = torch.empty((w.T * w.K, w.d), dtype=tdt, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for it in range(args.warmup + args.steps):
        if it == args.warmup:
            e0.record()
        c2r.permute(x, L.idx, L.E, L.local_slot, L.E_local, ws=L.ws_perm,
                    out=(L.counts, L.offsets, L.perm, L.inv_perm, x_perm_sa))
    e1.record()
    torch.cuda.synchronize()
    permute_rows_ms = e0.elapsed_time(e1) / args.steps
    # ... and the same call without the row scatter: the difference is the row-scatter kernel alone
    for it in range(args.warmup + args.steps):
        if it == args.warmup:
            e0.record()
        c2r.permute(x, L.idx, L.E, L.local_slot, L.E_local, ws=L.ws_perm,
                    out=(L.counts, L.offsets, L.perm, L.inv_perm, None), rows=False)
    e1.record()
    torch.cuda.synchronize()
    permute_index_ms = e0.elapsed_time(e1) / args.steps

    # Sec. 3.4 on one GPU (outside the step): the zero-redundancy send list for a fixed contiguous
    # 4-device map and the two-level combine that goes with it
    n_dev = 4
    dm = dev(wl.device_map(w.E, n_dev))
    zr = {}
    ws_dd = torch.empty(max(256, c2r.workspace_bytes(c2r.STAGE_DEDUP_DISPATCH, w.T, 0, n_dev, w.K, 0, c2r.F32)),
                        dtype=torch.uint8, device="cuda")
    y_part = torch.empty((w.T * w.K, w.d), dtype=tdt, device="cuda")
    y_zr = torch.empty((w.T, w.d), dtype=tdt, device="cuda")
    for _ in range(args.warmup):
        _, zoff, ztok, zrow = c2r.dedup_dispatch(L.idx, w.E, dm, n_dev, ws=ws_dd)
        c2r.combine_partial(L.y_perm, L.gates, L.inv_perm, ztok, zrow, zoff, y_part=y_part)
        c2r.combine_copies(y_part, zrow, w.T, w.K, L.y_shared, out=y_zr)
    ez = [mk() for _ in range(4)]
    ez[0].record()
    for _ in range(args.steps):
        _, zoff, ztok, zrow = c2r.dedup_dispatch(L.idx, w.E, dm, n_dev, ws=ws_dd)
    ez[1].record()
    for it in range(args.steps):
        c2r.combine_partial(L.y_perm, L.gates, L.inv_perm, ztok, zrow, zoff, y_part=y_part)
    ez[2].record()
    for it in range(args.steps):
        c2r.combine_copies(y_part, zrow, w.T, w.K, L.y_shared, out=y_zr)
    ez[3].record()
    torch.cuda.synchronize()
    n_send = int(zoff[-1].item())
    zr_ms = [ez[i].elapsed_time(ez[i + 1]) / args.steps for i in range(3)]
    part_bytes = (int(L.offsets[-1].item()) + n_send) * w.d * sz
    copies_bytes = (n_send + (2 if shared else 1) * w.T) * w.d * sz
    # the same count with experts co-located by their profiled co-activation (c2r_place_experts),
    # for this routing and for plain top-K of the same router
    placed = c2r.place_experts(Cm, n_dev)
    n_placed = int(c2r.dedup_dispatch(L.idx, w.E, placed, n_dev)[1][-1].item())
    idx_topk, _, _ = c2r.route(x, Wg, bias, w.K, None)
    n_placed_topk = int(c2r.dedup_dispatch(idx_topk, w.E, placed, n_dev)[1][-1].item())
    n_topk = int(c2r.dedup_dispatch(idx_topk, w.E, dm, n_dev)[1][-1].item())
    red = lambda n: 1.0 - n / (w.T * w.K)
    zr = {"devices": n_dev, "copies_sent": n_send, "copies_per_token": n_send / w.T,
          "redundancy": 1.0 - n_send / (w.T * w.K),
          "redundancy_by_map_and_routing": {"contiguous_map": {"c2r": red(n_send), "top_k": red(n_topk)},
                                            "co_located_map": {"c2r": red(n_placed), "top_k": red(n_placed_topk)}},
          "dedup_dispatch_ms": zr_ms[0],
          "combine_partial": {"ms": zr_ms[1], "GBps": part_bytes / zr_ms[1] / 1e6,
                              "frac_hbm": part_bytes / zr_ms[1] / 1e6 / PEAK["hbm_GBps"]},
          "combine_copies": {"ms": zr_ms[2], "GBps": copies_bytes / zr_ms[2] / 1e6,
                             "frac_hbm": copies_bytes / zr_ms[2] / 1e6 / PEAK["hbm_GBps"]}}

    # Sec. 4.1 / Table 3: token redundancy for expert-parallel degrees 2..6 in one pass per routing
    # (c2r_distinct_devices), for contiguous maps and for maps co-located from the profile, and
    # the estimator "all-to-all share x redundancy" fed with the shares Table 3 prints for the
    # paper's own testbed (context only: another machine, real tokens).  Eq. 3 on the profile too.
    eps = [ep for ep in (2, 3, 4, 5, 6) if ep <= w.E]
    a2a_share = {2: 0.301, 3: 0.407, 4: 0.619, 5: 0.763, 6: 0.772}
    maps_c = dev(np.stack([wl.device_map(w.E, ep) for ep in eps]))
    maps_p = torch.stack([c2r.place_experts(Cm, ep) for ep in eps])
    sweep = {}
    for mname, maps in (("contiguous_map", maps_c), ("co_located_map", maps_p)):
        tot_c2r = c2r.distinct_devices(L.idx, w.E, maps, max(eps)).tolist()
        tot_topk = c2r.distinct_devices(idx_topk, w.E, maps, max(eps)).tolist()
        sweep[mname] = {str(ep): {"c2r": red(tot_c2r[i]), "top_k": red(tot_topk[i]),
                                  "est_speedup_c2r": a2a_share[ep] * red(tot_c2r[i]),
                                  "est_speedup_top_k": a2a_share[ep] * red(tot_topk[i])}
                        for i, ep in enumerate(eps)}
    zr["redundancy_by_ep"] = sweep
    zr["redundancy_by_ep_note"] = ("est_speedup = Table 3's all-to-all time share of the paper's testbed x the "
                                   "redundancy measured here on synthetic tokens")
    P_deg = c2r.collaboration_degree(Cm)
    zr["collaboration_degree_eq3"] = {"mean": float(P_deg.mean()), "min": float(P_deg.min()),
                                      "max": float(P_deg.max()), "uniform_limit_ln_E_minus_1": float(np.log(max(w.E - 1, 1)))}

    # ---- algorithmic work per stage ----
    n_local = int(L.offsets[-1].item())          # rows the local experts process
    A = w.T * w.K
    stage_info = {}
    route_flops = 2.0 * w.T * w.d * w.E
    route_bytes = w.T * w.d * sz + w.T * w.K * 8 + w.d * w.E * 4
    stage_info["route"] = {"ms": st_ms["route"], "bytes": route_bytes, "flops": route_flops,
                           "GBps": route_bytes / st_ms["route"] / 1e6,
                           "TFLOPs": route_flops / st_ms["route"] / 1e9,
                           "frac_hbm": route_bytes / st_ms["route"] / 1e6 / PEAK["hbm_GBps"],
                           "frac_valu_f32": route_flops / st_ms["route"] / 1e9 / PEAK["valu_f32_TFLOPs"]}
    perm_bytes = w.T * w.d * sz + n_local * w.d * sz + A * 12
    stage_info["permute"] = {"ms": st_ms["permute"], "gather_fused_into_gate_up": bool(L.fuse_gather or L.gather_both)}
    if not (L.fuse_gather or L.gather_both):
        stage_info["permute"].update({"GBps": perm_bytes / st_ms["permute"] / 1e6,
                                      "frac_hbm": perm_bytes / st_ms["permute"] / 1e6 / PEAK["hbm_GBps"]})
    stage_info["permute_standalone_with_rows"] = {
        "ms": permute_rows_ms, "bytes": perm_bytes, "GBps": perm_bytes / permute_rows_ms / 1e6,
        "frac_hbm": perm_bytes / permute_rows_ms / 1e6 / PEAK["hbm_GBps"], "in_step": not (L.fuse_gather or L.gather_both)}
    rows_bytes = w.T * w.d * sz + n_local * w.d * sz + A * 4
    rows_ms = max(permute_rows_ms - permute_index_ms, 1e-6)
    stage_info["permute_standalone_with_rows"]["row_scatter_kernel"] = {
        "ms": rows_ms, "how": "the call with the row scatter minus the same call without it (%.4f ms)" % permute_index_ms,
        "bytes": rows_bytes, "GBps": rows_bytes / rows_ms / 1e6, "frac_hbm": rows_bytes / rows_ms / 1e6 / PEAK["hbm_GBps"]}
    comb_bytes = n_local * w.d * sz + w.T * w.d * sz * (2 if shared else 1) + A * 8
    stage_info["combine"] = {"ms": st_ms["combine"], "bytes": comb_bytes, "GBps": comb_bytes / st_ms["combine"] / 1e6,
                             "frac_hbm": comb_bytes / st_ms["combine"] / 1e6 / PEAK["hbm_GBps"]}
    fl_gu = 4.0 * n_local * w.d * w.F
    fl_dn = 2.0 * n_local * w.d * w.F
    fl_sgu = 4.0 * w.T * w.d * w.F_shared
    fl_sdn = 2.0 * w.T * w.d * w.F_shared
    if shared and L.fuse_shared:     # one launch per pass carries the routed groups and the shared expert
        fl_gu, fl_dn, fl_sgu, fl_sdn = fl_gu + fl_sgu, fl_dn + fl_sdn, 0.0, 0.0
    # a layer that cannot fold the gather into the first pass (or split the shared expert) runs both
    # passes of that FFN in one call, inside the span of its "gate_up" stage: report them as one
    both = {"ffn_gate_up": not L.fuse_gather, "shared_gate_up": sep_shared and not L.split_shared}
    for name, fl, fl2, second in (("ffn_gate_up", fl_gu, fl_dn, "ffn_down"), ("shared_gate_up", fl_sgu, fl_sdn, "shared_down")):
        if fl <= 0:
            continue
        if both[name]:
            ms = st_ms[name] + st_ms.get(second, 0.0)
            tf = (fl + fl2) / ms / 1e9
            stage_info[name.replace("gate_up", "both_passes")] = {"ms": ms, "TFLOPs": tf, "frac_mfma": tf / PEAK["mfma_bf16_TFLOPs"]}
        else:
            for nm, f in ((name, fl), (second, fl2)):
                tf = f / st_ms[nm] / 1e9
                stage_info[nm] = {"ms": st_ms[nm], "TFLOPs": tf, "frac_mfma": tf / PEAK["mfma_bf16_TFLOPs"]}
    if not L.overlap:
        ffn_span_ms = sum(st_ms.get(k, 0.0) for k in ("ffn_gate_up", "ffn_down", "shared_gate_up", "shared_down"))
    # Group-wise roof of the routed passes: an expert with few rows is bound by streaming its
    # weights, not by the matrix pipe, so the launch's floor is the sum over experts of
    # max(flops / MFMA peak, bytes / HBM peak) with each group given the whole chip.
    cnts = L.counts.cpu().numpy().astype(np.float64)
    peak_fl = (PEAK["mfma_bf16_TFLOPs"] if w.dtype == "bf16" else PEAK["valu_f32_TFLOPs"]) * 1e12
    hbm = PEAK["hbm_GBps"] * 1e9
    nz = cnts > 0
    t_gu = np.maximum(4.0 * cnts * w.d * w.F / peak_fl, (2.0 * w.F * w.d + cnts * (w.d + w.F)) * sz / hbm)[nz].sum()
    t_dn = np.maximum(2.0 * cnts * w.d * w.F / peak_fl, (1.0 * w.F * w.d + cnts * (w.d + w.F)) * sz / hbm)[nz].sum()
    if shared and L.fuse_shared:     # the shared expert is one more group of the same launch
        t_gu += max(4.0 * w.T * w.d * w.F_shared / peak_fl, (2.0 * w.F_shared * w.d + w.T * (w.d + w.F_shared)) * sz / hbm)
        t_dn += max(2.0 * w.T * w.d * w.F_shared / peak_fl, (1.0 * w.F_shared * w.d + w.T * (w.d + w.F_shared)) * sz / hbm)
    for name, t in (("ffn_gate_up", t_gu), ("ffn_down", t_dn)):
        if name in stage_info:
            stage_info[name]["groupwise_roof_ms"] = t * 1e3
            stage_info[name]["frac_groupwise_roof"] = t * 1e3 / st_ms[name]
            stage_info[name]["groups_weight_bound"] = int((nz & (4.0 * cnts * w.d * w.F / peak_fl <
                                                                 (2.0 * w.F * w.d + cnts * (w.d + w.F)) * sz / hbm)).sum())
    # algorithmic HBM bytes of the FFN launches: every non-empty expert's weights once, activations
    # read once (x: every token row once, also for the shared expert of the same launch) and
    # written once
    n_ne = int(nz.sum())
    by_gu = n_ne * 2 * w.F * w.d * sz + w.T * w.d * sz + n_local * 4 + n_local * w.F * sz
    by_dn = n_ne * w.F * w.d * sz + n_local * w.F * sz + n_local * w.d * sz
    by_sgu = (2 * w.F_shared * w.d * sz + w.T * w.F_shared * sz) if shared else 0
    by_sdn = (w.F_shared * w.d * sz + w.T * w.F_shared * sz + w.T * w.d * sz) if shared else 0
    if shared and L.fuse_shared:
        by_gu, by_dn = by_gu + by_sgu, by_dn + by_sdn
    elif shared:
        by_sgu += w.T * w.d * sz
    for name, nb in (("ffn_gate_up", by_gu), ("ffn_down", by_dn), ("shared_gate_up", by_sgu), ("shared_down", by_sdn)):
        if name in stage_info:
            stage_info[name]["bytes"] = nb
    if "ffn_both_passes" in stage_info:
        stage_info["ffn_both_passes"]["bytes"] = by_gu + by_dn
    ffn_tf = (fl_gu + fl_dn + fl_sgu + fl_sdn) / ffn_span_ms / 1e9
    stage_info["expert_ffn_all"] = {"ms": ffn_span_ms, "TFLOPs": ffn_tf, "frac_mfma": ffn_tf / PEAK["mfma_bf16_TFLOPs"],
                                    "note": "first FFN launch's start to last one's end; route and permute run inside it"
                                            if L.overlap else "sum of the FFN launches"}

    # HBM traffic of the dominant kernel per launch, from the committed rocprofv3 --pmc summary (if any)
    traffic, traffic_src = None, None
    tfile = os.path.join(ROOT, "profiles", f"ffn_gate_up_{w.name}_hbm_traffic.txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
            if line.startswith("measured_at_commit:"):
                traffic_src = f"profiles/{os.path.basename(tfile)} (counters of a separate rocprofv3 --pmc run, " \
                              f"library at commit {line.split(':')[1].strip()})"
    # dominant kernel: the gate/up pass (launched for the routed groups and, if any, the shared expert)
    n_launch = 2 if sep_shared else 1
    dom_ms = sum(dom_ms_live.values()) / n_launch   # from the timed region
    dom_fl = (fl_gu + fl_sgu) / n_launch
    both = ""
    # where the intermediate width is not a multiple of 64 the layer calls c2r_expert_ffn, whose
    # two passes are not bracketed separately: the events then span both kernels of a call
    if not L.fuse_gather:
        dom_fl += fl_dn / n_launch
    if sep_shared and not L.split_shared:
        dom_fl += fl_sdn / n_launch
    if not L.fuse_gather:
        both = " and <1> (both passes of c2r_expert_ffn)"
        for k_gu, k_dn in (("ffn_gate_up", "ffn_down"), ("shared_gate_up", "shared_down")):
            if k_gu in stage_info and k_dn in stage_info:
                stage_info[k_gu]["note"] = "both passes (c2r_expert_ffn); flops of gate/up only in TFLOPs"
    if w.dtype == "bf16":
        roofline = {"kernel": "ffn_bf16_dma_kernel<0>" + both + " (gate/up + SwiGLU" +
                              ("; routed groups and shared expert in one launch)" if shared and L.fuse_shared else ")"),
                    "bound": "mfma",
                    "achieved": dom_fl / dom_ms / 1e9, "peak": PEAK["mfma_bf16_TFLOPs"], "unit": "TFLOP/s",
                    "frac": dom_fl / dom_ms / 1e9 / PEAK["mfma_bf16_TFLOPs"], "traffic": traffic,
                    "traffic_source": traffic_src,
                    "avg_launch_ms": dom_ms, "launches_per_step": n_launch, "launches_timed": dom_launches_timed,
                    "timed_by": "event pairs on the launch stream around every fourth step's launches, inside the "
                                "timed region (a pair brackets the marker latency too: a few per cent more than "
                                "the kernel's own duration in the rocprofv3 trace)"}
    else:
        roofline = {"kernel": "ffn_f32_kernel<0>" + both + " (gate/up + SwiGLU)", "bound": "alu",
                    "achieved": dom_fl / dom_ms / 1e9, "peak": PEAK["valu_f32_TFLOPs"], "unit": "TFLOP/s",
                    "frac": dom_fl / dom_ms / 1e9 / PEAK["valu_f32_TFLOPs"], "traffic": None,
                    "avg_launch_ms": dom_ms, "launches_per_step": n_launch, "launches_timed": dom_launches_timed}

    ceilings = measured_ceilings(torch)

    # ---- every stage on its own from cold memory (see ColdTimer) ----
    isolated = None
    if args.isolate:
        cold = ColdTimer(torch)
        n_it = max(3, min(args.steps, 8))
        isolated = {"protocols": ColdTimer.__doc__.split("Two protocols, because")[0].strip() +
                                 " after_write: 512 MiB fill before the launch; after_read: that fill, then a 1 GiB read.",
                    "device_copy_192MB": cold.copy_yardstick(n_it)}
        for s_name in stages:
            isolated[s_name] = {}
            for mode in ("after_write", "after_read"):
                pair = {}

                def launch():
                    pair["p"] = (mk(), mk())
                    L.forward(x, trace={s_name: pair["p"]}, only=s_name)
                # prepare: a real step leaves the stage's inputs in place
                us = cold.time(lambda: L.forward(x), launch, n_it, mode)
                isolated[s_name][mode + "_us"] = us
        for s_name, nbytes in (("route", route_bytes), ("combine", comb_bytes)):
            for mode in ("after_write", "after_read"):
                us = isolated[s_name][mode + "_us"]
                isolated[s_name][mode + "_GBps"] = nbytes / us / 1e3
                isolated[s_name][mode + "_frac_hbm"] = nbytes / us / 1e3 / PEAK["hbm_GBps"]
                isolated[s_name][mode + "_frac_of_copy"] = (nbytes / us / 1e3) / isolated["device_copy_192MB"][mode]["GBps"]
        # the ABI's stand-alone dispatch with the row scatter
        for mode in ("after_write", "after_read"):
            us = cold.time(lambda: None, lambda: c2r.permute(x, L.idx, L.E, L.local_slot, L.E_local, ws=L.ws_perm,
                           out=(L.counts, L.offsets, L.perm, L.inv_perm, x_perm_sa)), n_it, mode)
            isolated.setdefault("permute_standalone_with_rows", {})[mode + "_us"] = us
            isolated["permute_standalone_with_rows"][mode + "_GBps"] = perm_bytes / us / 1e3
            isolated["permute_standalone_with_rows"][mode + "_frac_hbm"] = perm_bytes / us / 1e3 / PEAK["hbm_GBps"]
            isolated["permute_standalone_with_rows"][mode + "_frac_of_copy"] = \
                (perm_bytes / us / 1e3) / isolated["device_copy_192MB"][mode]["GBps"]
            us_idx = cold.time(lambda: None, lambda: c2r.permute(x, L.idx, L.E, L.local_slot, L.E_local, ws=L.ws_perm,
                               out=(L.counts, L.offsets, L.perm, L.inv_perm, None), rows=False), n_it, mode)
            us_rows = max(us - us_idx, 1e-3)
            isolated["permute_standalone_with_rows"][mode + "_row_scatter_kernel_us"] = us_rows
            isolated["permute_standalone_with_rows"][mode + "_row_scatter_kernel_frac_hbm"] = \
                rows_bytes / us_rows / 1e3 / PEAK["hbm_GBps"]
            isolated["permute_standalone_with_rows"][mode + "_row_scatter_kernel_frac_of_copy"] = \
                (rows_bytes / us_rows / 1e3) / isolated["device_copy_192MB"][mode]["GBps"]

    input_hashes = None
    if args.hash_inputs:
        import hashlib
        arrs = {"x": x_h, "W_g": Wg_h, "bias": bias_h, "w_gate": wg_h, "w_up": wu_h, "w_down": wd_h,
                "x_profile": x_prof_h}
        if shared_h is not None:
            arrs.update({"shared_w_gate": shared_h[0], "shared_w_up": shared_h[1], "shared_w_down": shared_h[2]})
        input_hashes = {k: {"shape": list(np.shape(v)), "sha256": hashlib.sha256(np.ascontiguousarray(v).tobytes()).hexdigest()}
                        for k, v in arrs.items() if v is not None}

    # ---- CPU oracle on a bounded sample of the same workload (rank 0, N = 1) ----
    cpu = None
    if args.cpu_sample > 0:
        from oracle import c2r_oracle as orc
        n = min(args.cpu_sample, w.T)
        collab_h = collab.cpu().numpy()
        tc = time.perf_counter()
        lg = orc.logits_canon_f32(x_h[:n], Wg_h, bias_h)
        idx_o, g_o = orc.route(lg, w.K, collab_h)
        orc.permute(idx_o, w.E, ls_h, w.n_local)
        y_o = orc.layer_tokens(x_h, np.arange(n), idx_o, g_o, wg_h, wu_h, wd_h, w.E, ls_h, shared_h)
        tc = time.perf_counter() - tc
        y_g = L.y[:n].float().cpu().numpy()
        cpu = {"value": n / tc, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"first {n} tokens of the batch through route+permute+FFN+combine (fp64), {tc:.1f} s",
               "gpu_vs_oracle_max_rel_err": float(np.abs(y_g - y_o).max() / np.abs(y_o).max()),
               "routing_bit_exact": bool(np.array_equal(L.idx[:n].cpu().numpy(), idx_o))}

    out = {
        "metric": "C2R MoE layer tokens/sec (Qwen-MoE shape)", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_ramp_steps_before_warmup": ramp_steps,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype if w.dtype != "f32" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: T={w.T} d={w.d} E={w.E} (local {w.n_local}) F={w.F} "
                               f"F_shared={w.F_shared} K={w.K} Tc={w.Tc}, planted {w.groups}-group router"
                               f"{' + Zipf(1.1) offsets' if w.zipf else ''}, profiled on {w.T_profile or w.T} tokens",
                   "rows_routed_local": n_local, "router": "fp32, canonical chunk order"},
        "roofline": roofline, "cpu_baseline": cpu, "stages": stage_info,
        "measured_ceilings": ceilings, "zero_redundancy_dispatch": zr,
        "schedule": ("two streams: shared gate/up beside route+permute, routed gate/up alone, the two down passes "
                     "side by side; stage times are spans on their own stream and overlap") if L.overlap
                    else "one stream, stages back to back" + ("; each FFN pass is one launch over the routed groups and "
                                                              "the shared expert" if shared and L.fuse_shared else ""),
        "setup_s": t_gen,
    }
    if isolated is not None:
        out["stages_from_cold_memory"] = isolated
    if input_hashes is not None:
        out["inputs"] = {"seed_base": wl.SEED_BASE if hasattr(wl, "SEED_BASE") else None, "arrays": input_hashes}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
