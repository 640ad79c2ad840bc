#!/usr/bin/env python3
"""Benchmark of the InfiniGen rehearsal + sparse-attention hot path on one MI355X.

A step is one decode step: for each of the model's L layers, the rehearsal (ig_speculate), the
prefetch of the selected rows and the attention over them, on that layer's own slab / KV pool
(distinct memory per layer, so the 256 MB last-level cache cannot serve the scan).  `value` is
microseconds per layer per decode step of the fastest launch sequence with all inputs resident in
HBM (host-pool workloads: the KV pool in pinned host memory by definition of the workload, the
two-stream pipeline).  The `roofline` object prices the partial-K scan kernel against the HBM peak
from its algorithmic bytes 2*B*H*N*r and its average duration, taken from HIP events attached to
each launch; `roofline_value_path` does the same for the dominant kernel of the sequence `value`
was measured on.  `cpu_baseline` is the CPU oracle timed on the host.

Without --workload the headline is the largest workload (cfg 5: long context, host KV pool) and
the same figures for cfg 2, 3 and 4 are carried in `workloads`; every workload runs in a child
process of its own (`bench.py --workload N`), so memory is returned in between and one failing
workload cannot take the others' figures with it.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
METRIC = "rehearsal+sparse-attn us/layer/decode step; partial-K scan GB/s vs HBM peak"
HEADLINE, OTHERS = 5, (2, 3, 4)


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def scan_traffic_from_profile(cfg: int):
    """HBM bytes per scan launch as the committed rocprofv3 counter summary of this workload states
    them (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size); None if there is none."""
    path = os.path.join(ROOT, "profiles", f"cfg{cfg}_hbm_traffic_counters.txt")
    try:
        m = re.search(r"=\s*([0-9.]+) MB of HBM traffic per launch", open(path).read())
    except OSError:
        return None, None
    return (float(m.group(1)) * 1e6, os.path.relpath(path, ROOT)) if m else (None, None)


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def scan_only(args, R, ctx, timed) -> dict:
    """The rehearsal kernels alone (projection + partial key cache scan of every layer, back to
    back) and plain reads of the same slabs: the short run the profiler summaries of the scan
    kernel are taken from."""
    import torch
    import paper_2406_19707_amd as ig
    L, K = R.L, args.steps

    def spec():
        for l in range(L):
            R.speculate(l)

    def read_slabs():
        n = R.slab[0].numel()
        for l in range(L):
            ctx.ig_read_bytes(R.slab[l], n - n % 16)

    for _ in range(args.warmup):
        spec()
        read_slabs()
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == ig.IG_OK
    loop_ms = timed(spec, K)
    ctx.ig_profile_begin()
    for _ in range(K):
        spec()
        read_slabs()
    torch.cuda.synchronize()
    ctx.ig_profile_end()
    out = {}
    for kid, name in ((ig.IG_K_PROJECT, "project"), (ig.IG_K_FINALIZE, "finalize"), (ig.IG_K_SCAN, "scan"),
                      (ig.IG_K_SELECT, "select"), (ig.IG_K_READ, "read")):
        ms, n = ctx.ig_profile_read(kid)
        if n:
            out[name] = {"avg_us": ms * 1e3 / n, "launches": n}
    if args.copy_reference:
        a_ = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
        b_ = torch.empty_like(a_)
        for _ in range(3):
            ctx.ig_copy_bytes(a_, b_, 1 << 28)
        torch.cuda.synchronize()
    sb = R.scan_bytes()
    return {"workload": R.w.name, "mode": "rehearsal kernels only", "layers": L, "steps": K,
            "kernels_by_hip_events": out, "speculate_loop_us_per_layer": loop_ms * 1e3 / L,
            "scan_algorithmic_bytes": sb,
            "scan_GBps": sb / (out["scan"]["avg_us"] * 1e-6) / 1e9,
            "scan_frac_of_hbm_peak": sb / (out["scan"]["avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "plain_read_GBps": R.slab[0].numel() / (out["read"]["avg_us"] * 1e-6) / 1e9}


def run_workload(args) -> dict:
    import numpy as np
    import torch
    import ig_workloads as wl
    import paper_2406_19707_amd as ig
    from paper_2406_19707_amd.pipeline import Rehearsal

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[args.workload]
    ctx = ig.Context(0)
    t0 = time.time()
    R = Rehearsal(ctx, w, gain=args.gain or None, layers=args.layers or None,
                  log=lambda *a: log(*a, f"({time.time() - t0:.1f}s)"))
    L = R.L
    K, W = args.steps, args.warmup
    brief = args.brief

    def timed(fn, steps):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / steps

    if args.scan_only:
        return scan_only(args, R, ctx, timed)

    # ---- eager ----
    pcie = None
    one_stream_ms = None
    if R.host_pool:
        # host pool: PCIe ceiling from a plain pinned -> device copy, then the side-stream pipeline
        src = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
        dst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst.copy_(src, non_blocking=True)
        h2d_ms = timed(lambda: dst.copy_(src, non_blocking=True), 5)
        h2d_gbs = (1 << 30) / (h2d_ms * 1e-3) / 1e9
        del src, dst
        log(f"pinned->device copy: {h2d_gbs:.1f} GB/s")
        for _ in range(W):
            R.step_overlapped()
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_OK
        eager_ms = timed(R.step_overlapped, K)
        # the same pipeline issued by the library in one call (events and buffer rotation in C++)
        for _ in range(W):
            R.step_overlapped_native()
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_OK
        native_ms = timed(R.step_overlapped_native, K)
        python_ms = eager_ms
        native_pipeline = native_ms < eager_ms
        eager_ms = min(eager_ms, native_ms)
        main_ms = timed(R.step_without_gather, K)
        R.collect_lists()
        with torch.cuda.stream(R.side):
            R.step_gather_only()
            torch.cuda.synchronize()
            gather_ms = timed(R.step_gather_only, K)
        rows = sum(int(c.sum().item()) for _, c in R.layer_lists)
        gbytes = rows * 2 * w.d * 2 / L                      # K and V rows per layer
        g_gbs = gbytes / (gather_ms * 1e-3 / L) / 1e9
        shorter = min(main_ms, gather_ms)
        pcie = {"h2d_memcpy_GBps": h2d_gbs, "gather_GBps": g_gbs, "frac_of_memcpy": g_gbs / h2d_gbs,
                "gathered_MB_per_layer": gbytes / 1e6, "gather_alone_us_per_layer": gather_ms * 1e3 / L,
                "main_alone_us_per_layer": main_ms * 1e3 / L, "overlapped_us_per_layer": eager_ms * 1e3 / L,
                "overlapped_issued_by": "ig_decode_step_overlapped (one library call per step)" if native_pipeline
                else "pipeline.py (three calls and three events per layer)",
                "overlapped_us_per_layer_library_call": native_ms * 1e3 / L,
                "overlapped_us_per_layer_python_calls": python_ms * 1e3 / L,
                # 1.0 = the whole step costs what the PCIe-bound prefetch costs alone
                "pipelined_over_gather_alone": eager_ms / gather_ms,
                # share of the main stream's work that ran under the prefetch
                "main_stream_hidden_fraction": (main_ms + gather_ms - eager_ms) / shorter}
        # the same step on one stream (rehearsal, prefetch, attention of a layer in sequence): the
        # PCIe link idles while the main-stream kernels run, but nothing runs against the prefetch
        R._use(0)
        for _ in range(W):
            R.step()
        torch.cuda.synchronize()
        one_stream_ms = timed(R.step, K)
        pcie["one_stream_us_per_layer"] = one_stream_ms * 1e3 / L
        log("pcie", pcie)
    else:
        for _ in range(W):
            R.step()
        assert ctx.ig_check_status() == ig.IG_OK
        eager_ms = timed(R.step, K)
    log(f"eager {eager_ms:.3f} ms/step = {eager_ms * 1e3 / L:.2f} us/layer")

    # ---- HIP graphs of the whole step (HBM pools): the four calls in sequence; prefetch and
    # attention in one pass; and that with the rehearsal of the next layer on a side stream ----
    variants = {}
    launch = "eager, two streams" if R.host_pool else "eager"
    value_path = "overlapped" if R.host_pool else "step"
    ms_per_step = eager_ms
    if R.host_pool and one_stream_ms < ms_per_step:
        ms_per_step, launch, value_path = one_stream_ms, "eager, one stream", "step"

    if not args.no_graph and not R.host_pool:
        def graphed(fn):
            g = torch.cuda.CUDAGraph()
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                fn()
            torch.cuda.current_stream().wait_stream(s)
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=s):
                fn()
            return g
        R._use(0)
        R.step()
        torch.cuda.synchronize()
        out_ref = R.out.clone()
        for name, fn, path in (("speculate, gather, attention", R.step, "step"),
                               ("speculate, gather+attention in one pass", R.step_one_pass, "one_pass"),
                               ("rehearsal of the next layer on a side stream, gather+attention in one pass",
                                R.step_two_stream, "one_pass"),
                               ("projection, then the next layer's scan and this layer's gather+attention in one launch",
                                R.step_joint, "joint")):
            try:
                g = graphed(fn)
                for _ in range(W):
                    g.replay()
                ms = timed(g.replay, K)
                # replays interleaved with eager work and synchronisation, each checked
                for _ in range(2):
                    R._use(0)
                    R.speculate(0)
                    torch.cuda.synchronize()
                    g.replay()
                    torch.cuda.synchronize()
                    assert torch.equal(R.out, out_ref), "graph replay changed the attention output"
                variants[name] = ms * 1e3 / L
                log(f"graph [{name}] {ms:.3f} ms/step = {ms * 1e3 / L:.2f} us/layer")
                if ms < ms_per_step:
                    ms_per_step, launch, value_path = ms, "hip graph replay: " + name, path
            except Exception as e:   # noqa: BLE001 -- report and keep the eager number
                log(f"graph [{name}] unavailable:", repr(e))

    # ---- fused-attention variant (no K_sel / V_sel copy), eager ----
    fused_ms = None
    if not R.host_pool and not brief:
        for _ in range(W):
            R.step_fused_attention()
        fused_ms = timed(R.step_fused_attention, K)

    # ---- per-kernel durations from HIP events attached to the launches ----
    names = {ig.IG_K_PROJECT: "project", ig.IG_K_FINALIZE: "finalize", ig.IG_K_SCAN: "scan",
             ig.IG_K_SELECT: "select", ig.IG_K_GATHER: "gather", ig.IG_K_ATTENTION: "attention"}

    def profiled(fns, steps):
        ctxs = [ctx] + ([R.side_ctx] if R.host_pool else [])
        for c in ctxs:
            c.ig_profile_begin()
        for _ in range(steps):
            for fn in fns:
                fn()
                torch.cuda.synchronize()   # one stream's work at a time
        for c in ctxs:
            c.ig_profile_end()
        out = {}
        for kid, name in names.items():
            ms, n = 0.0, 0
            for c in ctxs:
                m_, n_ = c.ig_profile_read(kid)
                ms, n = ms + m_, n + n_
            if n:
                out[name] = {"avg_us": ms * 1e3 / n, "launches": n}
        return out

    kernels_overlapped = None
    pk = max(1, min(K, 8))
    if R.host_pool:
        # each stream's kernels on their own (the roofline figures), then the overlapped pipeline
        def gather_only():
            with torch.cuda.stream(R.side):
                R.step_gather_only()
        kernels = profiled([R.step_without_gather, gather_only], max(1, pk // 2))
        kernels_overlapped = profiled([R.step_overlapped], max(1, pk // 2))
    else:
        kernels = profiled([R.step], pk)
        one = profiled([R.step_one_pass], pk)
        kernels["gather+attention in one pass"] = one["attention"]
        names[ig.IG_K_LAYER] = "joint"
        joint = profiled([R.step_joint], pk)
        if "joint" in joint:
            kernels["next layer's scan + this layer's gather+attention in one launch"] = joint["joint"]
        del names[ig.IG_K_LAYER]
    # streaming-read rate of this GPU on buffers of the slab's size (the slabs themselves, rotated)
    names[ig.IG_K_READ] = "read"
    slab_bytes = R.slab[0].numel()

    def read_slabs():
        for l in range(L):
            ctx.ig_read_bytes(R.slab[l], slab_bytes - slab_bytes % 16)
    read_slabs()
    read_us = profiled([read_slabs], 4)["read"]["avg_us"]
    read_gbs = slab_bytes / (read_us * 1e-6) / 1e9
    scan_us = kernels["scan"]["avg_us"]
    scan_bytes = R.scan_bytes()
    achieved = scan_bytes / (scan_us * 1e-6) / 1e9

    if args.copy_reference:
        a_ = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
        b_ = torch.empty_like(a_)
        for _ in range(3):
            ctx.ig_copy_bytes(a_, b_, 1 << 28)
        torch.cuda.synchronize()
        del a_, b_

    # ---- selected fraction over all layers ----
    fr = []
    for l in range(L):
        R._use(0)
        R.speculate(l)
        fr.append(R.sel_cnt.float().mean().item() / w.N)
    torch.cuda.synchronize()

    # ---- head-equalised variant (every head of a sequence fetches the mean count, 20 % cap) ----
    equalized = None
    if not R.host_pool and not brief:
        R._use(0)
        for _ in range(2):
            R.step_equalized()
        eq_ms = timed(R.step_equalized, max(2, K // 2))
        eq_launch = "eager"
        eq_graph_us = None
        eq_eager_us = eq_ms * 1e3 / L
        if not args.no_graph:
            try:
                g = torch.cuda.CUDAGraph()
                gs = torch.cuda.Stream()
                gs.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(gs):
                    R.step_equalized()
                torch.cuda.current_stream().wait_stream(gs)
                torch.cuda.synchronize()
                ref_cnt = R.sel_cnt.clone()
                with torch.cuda.graph(g, stream=gs):
                    R.step_equalized()
                for _ in range(2):
                    g.replay()
                g_ms = timed(g.replay, max(2, K // 2))
                R.sel_cnt.zero_()
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                assert torch.equal(R.sel_cnt, ref_cnt), "graph replay changed the equalised lists"
                eq_graph_us = g_ms * 1e3 / L
                if g_ms < eq_ms:
                    eq_ms, eq_launch = g_ms, "hip graph replay"
            except Exception as e:   # noqa: BLE001 -- keep the eager number
                log("graph [equalised] unavailable:", repr(e))
        kq = profiled([R.step_equalized], 2)
        R._use(0)
        for _ in range(2):
            R.step_equalized_two_calls()
        two_ms = timed(R.step_equalized_two_calls, max(2, K // 2))
        k2 = profiled([R.step_equalized_two_calls], 2)
        equalized = {"us_per_layer": eq_ms * 1e3 / L, "launch": eq_launch,
                     "over_value": eq_ms * 1e3 / L / (ms_per_step * 1e3 / L),
                     "eager_us_per_layer": eq_eager_us, "graph_us_per_layer": eq_graph_us,
                     "over_one_pass_sequence_without_equalisation":
                         (eq_ms * 1e3 / L / variants["speculate, gather+attention in one pass"]
                          if "speculate, gather+attention in one pass" in variants else None),
                     "selection_inside_the_scan_kernel": "select" not in kq,
                     "scan_kernel_us": kq["scan"]["avg_us"],
                     "gather_attention_kernel_us": kq["attention"]["avg_us"],
                     "two_calls": {"us_per_layer": two_ms * 1e3 / L, "launch": "eager",
                                   "scan_kernel_us_with_scores_kept": k2["scan"]["avg_us"],
                                   "equalize_kernel_us": k2["select"]["avg_us"]},
                     "tokens_per_head_last_layer_mean": R.sel_cnt.float().mean().item(),
                     "max_frac": 0.2}

    # ---- index-only partial weight (columns read out of the full weight at run time) ----
    index_only = None
    if not w.rope and not brief:
        R._use(0)
        R.speculate(L - 1)
        torch.cuda.synchronize()
        blob_cnt = R.sel_cnt.clone()
        for _ in range(2):
            R.step_index_only()
        torch.cuda.synchronize()
        differing = int((R.sel_cnt != blob_cnt).sum().item())
        io_ms = timed(R.step_index_only, max(2, K // 2))
        ki = profiled([R.step_index_only], 2)
        D_ = w.D
        eb = 2 if w.dtype == "f16" else 4
        index_only = {"us_per_layer": io_ms * 1e3 / L,
                      "launch": "eager, one stream" + (", rehearsal only" if R.host_pool else ""),
                      "project_kernel_us": ki["project"]["avg_us"],
                      "project_kernel_us_stored_blob": kernels["project"]["avg_us"],
                      "weight_bytes_read_MB": D_ * D_ * eb / 1e6,
                      "weight_bytes_read_MB_stored_blob": D_ * w.H * R.r * eb / 1e6,
                      "project_GBps": D_ * D_ * eb / (ki["project"]["avg_us"] * 1e-6) / 1e9,
                      "blob_bytes_saved_MB": R.wq.numel() / 1e6,
                      "lists_with_other_count_than_stored_blob_last_layer": differing}

    # ---- partial key cache in host memory, speculation on the CPU (Section 6.2) ----
    host_spec = None
    if not brief:
        R._use(0)
        n_host = min(L, 4)
        R.host_speculation_setup(slab_layers=n_host)
        R.step_host_speculation()
        torch.cuda.synchronize()
        host_cnt = R.sel_cnt.clone()          # the last layer's lists, made on the host
        R.ctx.ig_scan_select(R.desc, R.q_p, R.slab[(L - 1) % n_host], R.sel_idx, R.stride, R.sel_cnt)
        torch.cuda.synchronize()
        same = bool(torch.equal(R.sel_cnt, host_cnt))
        hs_ms = timed(R.step_host_speculation, 2)
        t0 = time.perf_counter()
        for l in range(n_host):
            ig.lib().ig_speculate_host(R.ctx._h, ctypes.byref(R.desc), R.q_p_host.data_ptr(),
                                       R.slab_host[l].data_ptr(), R.sel_idx_host.data_ptr(), R.stride,
                                       R.sel_cnt_host.data_ptr(), None, 0)
        host_us = (time.perf_counter() - t0) * 1e6 / n_host
        host_spec = {"us_per_layer": hs_ms * 1e3 / L, "launch": "eager, one stream, host threads",
                     "host_scan_select_us": host_us,
                     "host_scan_GBps": R.scan_bytes() / (host_us * 1e-6) / 1e9,
                     "host_threads": min(os.cpu_count() or 1, 64, w.B * w.H),
                     "partial_key_cache_MB_off_the_gpu_per_layer": R.slab[0].numel() / 1e6,
                     "host_slab_layers": n_host,
                     "same_counts_as_device_scan_last_layer": same}
        del R.slab_host
        log(f"host speculation {host_spec['us_per_layer']:.0f} us/layer")

    # ---- decode loop with a growing cache: append of the decoded token after every layer ----
    decode_loop = None
    if not args.no_decode_loop and not brief:
        T, L2 = 8, min(L, 8)
        R2 = Rehearsal(ig.Context(0), w, gain=args.gain or None, layers=L2, host_layers=2,
                       extra_tokens=T, offline_from=R)
        R2.decode(2)
        torch.cuda.synchronize()
        assert R2.ctx.ig_check_status() == ig.IG_OK
        t_sparse = timed(lambda: R2.decode(T, dense_first_layer=False), 2) * 1e3 / (T * L2)
        t_dense0 = timed(lambda: R2.decode(T, dense_first_layer=True), 2) * 1e3 / (T * L2)
        decode_loop = {"steps": T, "layers": L2, "launch": "eager, one stream",
                       "calls_per_layer": "ig_speculate, " + ("ig_gather_kv, ig_sparse_attention"
                                                              if R.host_pool else "ig_gather_attention")
                                          + " (cached tokens + the token being decoded), ig_append_token",
                       "us_per_layer_per_step": t_sparse,
                       "us_per_layer_per_step_first_layer_dense": t_dense0}
        del R2
        torch.cuda.empty_cache()

    # ---- literal variant (gain 1: every token selected), eager, a few steps ----
    literal = None
    if R.gain != 1.0 and not args.no_literal and not R.host_pool and not brief:
        scale = R.desc.scale
        R.desc.scale = 1.0 / (w.d ** 0.5)
        for _ in range(2):
            R.step()
        lit_ms = timed(R.step, max(2, K // 4))
        literal = {"us_per_layer": lit_ms * 1e3 / L,
                   "selected_fraction": R.sel_cnt.float().mean().item() / w.N}
        R.desc.scale = scale

    # ---- CPU oracle on layer 0 (one layer, whole batch), and parity of the GPU result ----
    cpu = cpu_all = None
    parity = None
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import ig_oracle as o
        h0 = R.layer0_host
        f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)   # noqa: E731
        x, Kt, V, q = f32(h0["x"]), f32(h0["K"]), f32(h0["V"]), f32(h0["q"])
        Wf = f32(R.W_host)
        posv = np.full(w.B, w.N, np.int32)

        def oracle_layer(x, Kt, V, q, heads=None, pos=posv):
            """One layer on the rows of x given; heads: (h0, h1) restricts scan ... attention to
            those heads (the projection is that of all heads, cut afterwards)."""
            if w.rope:
                q_p = o.project_rope(x, Wf, pos, R.A, R.idx_host)
            else:
                q_p = o.project(x, Wf, R.idx_host)
            idx_h = R.idx_host
            if heads is not None:
                q_p = np.ascontiguousarray(q_p[:, heads[0]:heads[1]])
                idx_h = np.ascontiguousarray(R.idx_host[heads[0]:heads[1]])
            s = o.scan(q_p, Kt, idx_h, R.desc.scale)
            sel_idx, sel_cnt = o.select(s, w.alpha)
            m = int(sel_cnt.max())
            sel_small = np.ascontiguousarray(sel_idx[:, :m])
            Ks = o.gather(Kt, sel_small, sel_cnt)
            Vs = o.gather(V, sel_small, sel_cnt)
            return s, sel_idx, sel_cnt, o.attend(q, Ks, Vs, sel_cnt, R.desc.scale)

        t = time.perf_counter()
        s, sel_idx, sel_cnt, out = oracle_layer(x, Kt, V, q)
        cpu_s = time.perf_counter() - t
        # more layers of the same step until about 15 s of oracle time (bounded sample)
        n_cpu = 1
        avail = R.n_pool if R.host_pool else L
        while n_cpu < avail and cpu_s * (n_cpu + 1) / n_cpu < 15.0:
            l = n_cpu
            xl, Kl, Vl, ql = (f32(t_.float().cpu().numpy()) for t_ in (R.x[l], R.K[l], R.V[l], R.q[l]))
            t = time.perf_counter()
            oracle_layer(xl, Kl, Vl, ql)
            cpu_s += time.perf_counter() - t
            n_cpu += 1
            del xl, Kl, Vl, ql
        cpu = {"value": cpu_s * 1e6 / n_cpu, "unit": "us/layer/decode step", "cores": 1, "kind": "oracle",
               "sample": f"{n_cpu} of {L} layers of one decode step, whole batch (project+scan+select+gather+"
                         f"attend, single thread, {cpu_s:.1f} s in total)"}
        # the same oracle, untouched, on all host cores this job may use: layer 0 cut into
        # (sequence, head group) slices that a thread pool runs side by side (the C calls release
        # the interpreter lock); the slices' results are not used, only timed
        nthreads = max(1, min(16, os.cpu_count() or 1))
        hg = max(1, w.H // max(1, (2 * nthreads + w.B - 1) // w.B))
        tasks = [(b, h_, min(w.H, h_ + hg)) for b in range(w.B) for h_ in range(0, w.H, hg)]

        def slice_task(tk):
            b, ha, hb = tk
            oracle_layer(x[b:b + 1], np.ascontiguousarray(Kt[b:b + 1, ha:hb]),
                         np.ascontiguousarray(V[b:b + 1, ha:hb]), np.ascontiguousarray(q[b:b + 1, ha:hb]),
                         heads=(ha, hb), pos=posv[b:b + 1])
        t = time.perf_counter()
        with ThreadPoolExecutor(nthreads) as ex:
            list(ex.map(slice_task, tasks))
        par_s = time.perf_counter() - t
        cpu_all = {"value": par_s * 1e6, "unit": "us/layer/decode step", "cores": nthreads,
                   "kind": "oracle, one layer cut into (sequence, head group) slices on a thread pool",
                   "nproc": os.cpu_count(), "cpu_model": cpu_model(),
                   "sample": f"layer 0 of one decode step, {len(tasks)} slices of {hg} heads, {par_s:.2f} s; every "
                             "slice repeats the layer's projection for its sequence"}
        # GPU result for the same layer
        R._use(0)
        R.layer(0)
        torch.cuda.synchronize()
        g_idx, g_cnt = R.sel_idx.cpu().numpy(), R.sel_cnt.cpu().numpy()
        g_out = R.out.float().cpu().numpy().reshape(-1, w.d)
        outside = 0
        differing = 0
        for i in range(w.B * w.H):
            diff = np.setxor1d(g_idx[i, :g_cnt[i]], sel_idx[i, :sel_cnt[i]])
            if diff.size:
                thr = np.float32(s.reshape(-1, w.N)[i].max()) - np.float32(w.alpha)
                outside += int((np.abs(s.reshape(-1, w.N)[i, diff] - thr) > 1e-3).sum())
                differing += int(diff.size)
        same = [i for i in range(w.B * w.H) if g_cnt[i] == sel_cnt[i]
                and np.array_equal(g_idx[i, :g_cnt[i]], sel_idx[i, :sel_cnt[i]])]
        err = np.abs(g_out[same] - out[same])
        ok = bool(np.all(err <= 2e-2 + 1e-2 * np.abs(out[same])))
        parity = {"layer": 0, "pairs": w.B * w.H, "tokens_differing_outside_1e-3_band": outside,
                  "tokens_differing_inside_band": differing - outside,
                  "attention_max_abs_err": float(err.max()) if len(same) else None,
                  "attention_within_2e-2_abs_1e-2_rel": ok}

    dtype = "f32" if w.dtype == "f32" else "f16"
    # algorithmic bytes per launch of every kernel (layer average) and the rate they imply
    esz = 4 if w.dtype == "f32" else 2
    row_bytes = float(np.mean(fr)) * w.N * w.B * w.H * w.d * esz * 2          # K and V rows of a layer
    joint_name = "next layer's scan + this layer's gather+attention in one launch"
    kbytes = {"project": ig.ig_wq_bytes(R.desc), "scan": scan_bytes, "gather": 2 * row_bytes,
              "attention": row_bytes, "gather+attention in one pass": 2 * row_bytes,
              joint_name: scan_bytes + 2 * row_bytes}
    if R.host_pool:
        kbytes["gather"] = row_bytes                                          # over PCIe; the HBM write is extra
    for name, kb in kbytes.items():
        if name in kernels:
            kernels[name]["algorithmic_MB"] = kb / 1e6
            kernels[name]["GBps"] = kb / (kernels[name]["avg_us"] * 1e-6) / 1e9
            if not (R.host_pool and name == "gather"):
                kernels[name]["frac_of_hbm_peak"] = kernels[name]["GBps"] / HBM_PEAK_GBS
    # the dominant kernel of the launch sequence `value` was measured on
    if R.host_pool and value_path == "overlapped":
        vp = {"kernel": "K/V row gather from the pinned host pool (side stream)", "bound": "pcie",
              "achieved": pcie["gather_GBps"], "peak": pcie["h2d_memcpy_GBps"], "unit": "GB/s",
              "frac": pcie["frac_of_memcpy"], "peak_is": "pinned->device hipMemcpyAsync rate measured in this run",
              "algorithmic_bytes_per_launch": row_bytes, "avg_kernel_us": kernels["gather"]["avg_us"]}
    else:
        dom = joint_name if (value_path == "joint" and joint_name in kernels) else "scan"
        vp = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBS,
              "unit": "GB/s", "frac": kernels[dom]["GBps"] / HBM_PEAK_GBS,
              "algorithmic_bytes_per_launch": kbytes[dom], "avg_kernel_us": kernels[dom]["avg_us"]}
    traffic, traffic_src = scan_traffic_from_profile(args.workload)
    res = {
        "metric": METRIC,
        "value": ms_per_step * 1e3 / L,
        "unit": "us/layer/decode step",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B{w.B} H{w.H} d{w.d} N{w.N} r{R.r} {dtype} KV, alpha {w.alpha}, "
                               f"{'rope' if w.rope else 'folded skew'}, KV pool in "
                               f"{'pinned host memory' if R.host_pool else 'HBM'}",
                   "variant": f"calibrated logit gain {R.gain:g} (scale = gain/sqrt(d))",
                   "layers_per_step": L, "launch": launch,
                   "selected_fraction_mean": float(np.mean(fr)), "selected_fraction_min_layer": float(np.min(fr)),
                   "selected_fraction_max_layer": float(np.max(fr))},
        "eager_us_per_layer": eager_ms * 1e3 / L,
        "graph_us_per_layer": variants or None,
        "fused_attention_eager_us_per_layer": None if fused_ms is None else fused_ms * 1e3 / L,
        "scan_GBps": achieved,
        "kernels": kernels,
        "kernels_while_overlapped": kernels_overlapped,
        "literal_variant": literal,
        "head_equalized_variant": equalized,
        "index_only_weight_variant": index_only,
        "host_speculation_variant": host_spec,
        "decode_loop_growing_cache": decode_loop,
        "roofline": {"kernel": "partial-K scan + max + threshold + compaction", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": traffic_src and f"{traffic_src} (rocprofv3 FETCH_SIZE + WRITE_SIZE of an "
                                                      "earlier run of this workload, not collected in this run)",
                     "algorithmic_bytes_per_launch": scan_bytes, "avg_kernel_us": scan_us,
                     "target_frac": 0.70, "target_met": bool(achieved / HBM_PEAK_GBS >= 0.70),
                     "plain_read_same_size": {"GBps": read_gbs, "avg_kernel_us": read_us,
                                              "scan_over_plain_read": read_us / scan_us}},
        "roofline_value_path": vp,
        "pcie": pcie,
        "cpu_baseline": cpu,
        "cpu_baseline_all_cores": cpu_all,
        "parity": parity,
    }
    return res


def child_flags(args, cfg):
    f = ["--workload", str(cfg), "--steps", str(args.steps), "--warmup", str(args.warmup)]
    if cfg != HEADLINE:
        f.append("--brief")
    for flag in ("no_graph", "no_cpu_baseline", "no_literal", "no_decode_loop"):
        if getattr(args, flag):
            f.append("--" + flag.replace("_", "-"))
    return f


def run_child(args, cfg):
    """One workload in a process of its own; returns its result dict or {"error": ...}."""
    cmd = [sys.executable, os.path.abspath(__file__)] + child_flags(args, cfg)
    log("workload", cfg, ":", " ".join(cmd[1:]))
    t = time.time()
    try:
        p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=None, text=True, timeout=args.child_timeout)
    except subprocess.TimeoutExpired:
        return {"error": f"bench.py --workload {cfg} exceeded {args.child_timeout} s"}
    log(f"workload {cfg} done in {time.time() - t:.0f} s, exit code {p.returncode}")
    lines = [ln for ln in p.stdout.strip().splitlines() if ln.startswith("{")]
    if p.returncode != 0 or not lines:
        return {"error": f"bench.py --workload {cfg} exited with code {p.returncode}"}
    return json.loads(lines[-1])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=0,
                    help="one documented workload (2..5) in this process; 0 = cfg 5 as the headline with "
                         "cfg 2, 3 and 4 under `workloads`, each in a child process")
    ap.add_argument("--only-headline", action="store_true", help="with --workload 0: skip cfg 2, 3 and 4")
    ap.add_argument("--brief", action="store_true",
                    help="skip the side variants (literal, head-equalised, index-only, decode loop)")
    ap.add_argument("--layers", type=int, default=0, help="layers per step (0 = the model's)")
    ap.add_argument("--gain", type=float, default=0.0, help="logit gain (0 = the workload's calibrated one)")
    ap.add_argument("--scan-only", action="store_true",
                    help="with --workload N: only the rehearsal kernels and plain reads of the slabs (profiling runs)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-literal", action="store_true", help="skip the gain-1 (select everything) variant")
    ap.add_argument("--no-decode-loop", action="store_true", help="skip the growing-cache decode loop")
    ap.add_argument("--copy-reference", action="store_true",
                    help="also launch a plain 256 MiB device copy (reference for scaling hardware counters)")
    ap.add_argument("--child-timeout", type=int, default=420, help="seconds a workload's child process may take")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); the path would shard over "
              "(sequence, head) pairs without communication, but no multi-GPU run is part of it",
              file=sys.stderr)
        sys.exit(2)
    if args.workload:
        print(json.dumps(run_workload(args)))
        return
    # this process never touches the GPU: every workload runs in a child of its own
    head = run_child(args, HEADLINE)
    if "error" in head:
        log(head["error"])
        sys.exit(1)
    if not args.only_headline:
        keep = ("value", "unit", "ms_per_step", "steps", "warmup", "dtype", "config", "eager_us_per_layer",
                "graph_us_per_layer", "scan_GBps", "kernels", "kernels_while_overlapped", "roofline",
                "roofline_value_path", "pcie", "parity", "cpu_baseline", "cpu_baseline_all_cores", "error")
        head["workloads"] = {}
        for cfg in OTHERS:
            r = run_child(args, cfg)
            head["workloads"][f"cfg{cfg}"] = {k: r[k] for k in keep if k in r}
    print(json.dumps(head))


if __name__ == "__main__":
    main()
