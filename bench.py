#!/usr/bin/env python3
"""Benchmark of the fused sample + mean forward on one MI355X.

Default workload: the web-scale citation shape (N = 111 M nodes, ~1.6 B edges, int64 indptr,
bf16 x[N,128], B = 4096 seeds, fanouts 15/10) -- the shape the headline metric (rows
aggregated per second and achieved HBM GB/s at fanout 15/10, D = 128) is quoted on.  One step
is one launch of the fused 2-hop forward with ID and per-slot emission over a fresh batch of
seeds; inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: throughput, roofline block (algorithmic bytes per launch over the launch
duration by HIP events, against the 8 TB/s HBM peak), oracle CPU baseline and a saturated-batch
block.  `--gpus N` with N > 1 is refused: this
build is single-GPU by scope.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# Bandwidth / atomic-rate microbenchmarks of `--ceilings`: a measurement aid of this script, not
# part of the product library.
CEILINGS_SRC = os.path.join(ROOT, "bench_ceilings.hip")
CEILINGS_LIB = os.path.join(ROOT, "libbench_ceilings.so")


def build_ceilings(verbose: bool = False) -> str:
    """Compile bench_ceilings.hip for gfx950 into libbench_ceilings.so (next to this script)."""
    import subprocess
    from paper_2511_13645_amd import build as hip_build
    tmp = CEILINGS_LIB + ".tmp.%d" % os.getpid()
    cmd = [hip_build.hipcc(), *hip_build.HIPCC_FLAGS, "-shared", "-o", tmp, CEILINGS_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, CEILINGS_LIB)
    return CEILINGS_LIB


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(leaf_rows, hop1_rows, B, k1, k2, D, elem, iptr, emit_ids=True, emit_h1=True):
    """Bytes the method itself must move for one launch (2-hop), from the actual counts:
    every aggregated leaf row is read once (D*elem) together with its `indices` entry; every
    sampled row owner (seed or live hop-1 slot) costs an indptr pair; hop-1 IDs are read from
    `indices`; outputs are written once (out, all B*k1 rows of out_h1, all ID slots)."""
    b = leaf_rows * (D * elem + 4)
    b += hop1_rows * (4 + 2 * iptr)
    b += B * (2 * iptr + 4 + D * elem)
    if emit_h1:
        b += B * k1 * D * elem
    if emit_ids:
        b += 4 * B * (k1 + k1 * k2)
    return b


def csrc_hash():
    """SHA-256 over the kernel sources the library is built from (file names and bytes, sorted)."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2511_13645_amd", "csrc")
    for fn in sorted(os.listdir(d)):
        if fn.endswith((".hip", ".h")):
            h.update(fn.encode())
            h.update(open(os.path.join(d, fn), "rb").read())
    return h.hexdigest()


def committed_traffic(workload):
    """HBM bytes per launch from the committed counter runs -- only while the kernel sources are
    the ones those runs were made with; otherwise None (the figure would be stale)."""
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % workload)
    try:
        t = json.load(open(tpath))
    except Exception:
        return None
    if t.get("csrc_sha256") != csrc_hash():
        log("[bench] %s was measured on other kernel sources: roofline.traffic = null" % os.path.basename(tpath))
        return None
    return t.get("hbm_bytes_per_launch")


def traffic_from_counters(args):
    """--traffic-from: turn two rocprofv3 --pmc counter CSVs (FETCH_SIZE run, WRITE_SIZE run; both made
    with --calibrate-copy) into profiles/traffic_<workload>.json, stamped with the source hash."""
    import csv
    fetch_csv, write_csv = args.traffic_from

    def mean_kib(path, counter, needle, largest_only=False):
        v = [float(r["Counter_Value"]) for r in csv.DictReader(open(path))
             if r["Counter_Name"] == counter and needle in r["Kernel_Name"]]
        if largest_only and v:                   # other, small copies of the run use the same kernel
            v = [a for a in v if a >= 0.5 * max(v)]
        if not v:
            raise RuntimeError("%s: no %s rows for a kernel named *%s*" % (path, counter, needle))
        return sum(v) / len(v), len(v)
    gib_kib = float(1 << 20)                     # the calibration copy moves 1 GiB each way
    f_copy, _ = mean_kib(fetch_csv, "FETCH_SIZE", "copyBuffer", largest_only=True)
    w_copy, _ = mean_kib(write_csv, "WRITE_SIZE", "copyBuffer", largest_only=True)
    f_k, n_f = mean_kib(fetch_csv, "FETCH_SIZE", args.traffic_kernel)
    w_k, n_w = mean_kib(write_csv, "WRITE_SIZE", args.traffic_kernel)
    f_scale, w_scale = gib_kib / f_copy, gib_kib / w_copy
    out = {"hbm_bytes_per_launch": int(round((f_k * f_scale + w_k * w_scale) * 1024)),
           "fetch_kib": f_k, "fetch_scale": f_scale, "write_kib": w_k, "write_scale": w_scale,
           "dispatches": [n_f, n_w], "kernel": args.traffic_kernel, "workload": args.workload,
           "csrc_sha256": csrc_hash()}
    path = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.workload)
    json.dump(out, open(path, "w"), indent=1)
    print(json.dumps(out))
    return 0


def trace_roots(L, binding, synth, torch, w, dev, batches=(4096, 65536)):
    """--trace-roots (needs --lib with a -DFSA_TRACE build): per-root start, gather-start and end times of
    the fused 2-hop forward, printed as the distribution of when roots begin to gather and when they finish."""
    import numpy as np
    g, x = w.graph, w.x
    fan = list(w.fanouts)
    L.fsa_debug_set_trace.argtypes = [ctypes.c_void_p]
    for B in batches:
        seeds = synth.seed_batches(g.num_nodes, B, 4, seed=2).to(dev)
        tr = torch.zeros((B, 4), dtype=torch.int64, device=dev)
        L.fsa_debug_set_trace(tr.data_ptr())
        for i in range(4):
            tr.zero_()
            binding.fsa_sample_mean_fwd(g.indptr, g.indices, x, seeds[i], fan, w.sampler_seed)
            torch.cuda.synchronize()
        L.fsa_debug_set_trace(None)
        t = tr.cpu().numpy().astype(np.float64)
        rows = t[:, 3]
        t0 = t[:, 0].min()
        st, gs, en = (t[:, 0] - t0) * 0.01, (t[:, 1] - t0) * 0.01, (t[:, 2] - t0) * 0.01      # 10 ns ticks -> us
        pc = np.percentile
        print("B=%d: first start to last end %.2f us (stamps add about a fifth); rows per root mean %.1f p50 %.0f p90 %.0f max %.0f"
              % (B, en.max(), rows.mean(), pc(rows, 50), pc(rows, 90), rows.max()))
        for name, a in (("wave start", st), ("gather start", gs), ("wave end", en), ("start -> gather", gs - st),
                        ("gather duration", en - gs)):
            print("   %-18s p1 %6.2f  p10 %6.2f  p50 %6.2f  p90 %6.2f  p99 %6.2f  max %6.2f us"
                  % (name, pc(a, 1), pc(a, 10), pc(a, 50), pc(a, 90), pc(a, 99), a.max()))
        for lo, hi in ((0, 1), (1, 33), (33, 65), (65, 97), (97, 129), (129, 100000)):
            m = (rows >= lo) & (rows < hi)
            if m.sum():
                print("   roots with %3d..%-3d rows: n=%6d  start->gather p50 %5.2f  gather p50 %5.2f p90 %5.2f  end p50 %6.2f p90 %6.2f max %6.2f"
                      % (lo, min(hi - 1, int(rows.max())), m.sum(), pc((gs - st)[m], 50), pc((en - gs)[m], 50),
                         pc((en - gs)[m], 90), pc(en[m], 50), pc(en[m], 90), en[m].max()))
        if B <= 8192:
            print("   time (us): roots still sampling / roots gathering / rows per us (each root's rows spread evenly over its gather)")
            for a in np.arange(0, en.max(), 2.0):
                b_ = a + 2.0
                ov = np.clip(np.minimum(en, b_) - np.maximum(gs, a), 0, None)
                print("   %5.0f %6d %6d %9.0f" % (a, ((st < b_) & (gs > a)).sum(), ((gs < b_) & (en > a)).sum(),
                                                  (rows * ov / np.maximum(en - gs, 1e-9)).sum() / 2.0))
    return 0


def measure_paths(L, binding, synth, torch, w, B, dev, n_launch=20, replay=True, backward=True):
    """Forward with ID and per-slot emission over `n_launch` fresh seed batches, then the replay forward
    and (fp32 tables) the backward on the IDs of those batches: launch duration by HIP events around
    back-to-back launches, algorithmic bytes from the actual counts, fraction of the HBM peak."""
    g, x = w.graph, w.x
    fan = list(w.fanouts)
    hops = len(fan)
    k1 = fan[0]
    k2 = fan[1] if hops == 2 else 0
    N, D = x.shape
    elem, iptr = x.element_size(), g.indptr.element_size()
    if B > N:
        return None
    x_code = {torch.float32: binding.FSA_F32, torch.bfloat16: binding.FSA_BF16, torch.float16: binding.FSA_F16}[x.dtype]
    n_all = n_launch + 2
    seeds = synth.seed_batches(N, B, n_all, seed=6).to(dev)
    out = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=dev) if hops == 2 else None
    ids1 = torch.empty((n_all, B, k1), dtype=torch.int32, device=dev)
    ids2 = torch.empty((n_all, B, k1, k2), dtype=torch.int32, device=dev) if hops == 2 else None
    fan_host = (ctypes.c_int32 * hops)(*fan)
    stream = torch.cuda.current_stream().cuda_stream
    h1_ptr = None if out_h1 is None else out_h1.data_ptr()
    # pointers are looked up once: a launch of a few microseconds must not wait for the host
    seed_p = [seeds[i].data_ptr() for i in range(n_all)]
    id1_p = [ids1[i].data_ptr() for i in range(n_all)]
    id2_p = [ids2[i].data_ptr() if hops == 2 else None for i in range(n_all)]
    i2 = id2_p.__getitem__
    p_indptr, p_indices, p_x, p_out = g.indptr.data_ptr(), g.indices.data_ptr(), x.data_ptr(), out.data_ptr()
    it_code = binding.FSA_I64 if iptr == 8 else binding.FSA_I32
    fan_p = ctypes.cast(fan_host, ctypes.c_void_p)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        for i in range(2):
            fn(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(2, n_all):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n_launch

    def fwd(i):
        rc = L.fsa_sample_mean_fwd(p_indptr, it_code, p_indices, N, p_x, x_code, D, seed_p[i], B, fan_p, hops,
                                   w.sampler_seed, p_out, h1_ptr, id1_p[i], i2(i), stream)
        if rc != 0:
            raise RuntimeError("fsa_sample_mean_fwd -> %d" % rc)
    f_ms = timed(fwd)
    if hops == 2:
        leaf = int((ids2[2:] >= 0).sum().item()) / n_launch
        hop1 = int((ids1[2:] >= 0).sum().item()) / n_launch
        f_alg = algorithmic_bytes(leaf, hop1, B, k1, k2, D, elem, iptr)
    else:
        leaf = int((ids1[2:] >= 0).sum().item()) / n_launch
        f_alg = leaf * (D * elem + 4) + B * (2 * iptr + 4 + D * elem) + 4 * B * k1

    def block(ms, alg, **more):
        gbps = alg / (ms * 1e-3) / 1e9
        return {"launch_us": ms * 1e3, "rows_per_s": leaf / (ms * 1e-3), "algorithmic_bytes_per_launch": alg,
                "hbm_gbps": gbps, "frac": gbps / HBM_PEAK_GBPS, **more}
    r = {"workload": w.name, "dtype": str(x.dtype).split(".")[1], "D": D, "fanouts": fan, "global_batch": B,
         "rows_per_launch": leaf, "forward": block(f_ms, f_alg)}
    if replay:
        def rep(i):
            rc = L.fsa_mean_replay_fwd(p_x, x_code, D, N, id1_p[i], i2(i), B, k1, k2, p_out, h1_ptr, stream)
            if rc != 0:
                raise RuntimeError("fsa_mean_replay_fwd -> %d" % rc)
        r_ms = timed(rep)
        # saved IDs read instead of the graph; the same rows and outputs
        r_alg = leaf * D * elem + 4 * B * (k1 + k1 * k2) + B * D * elem + (B * k1 * D * elem if hops == 2 else 0)
        r["replay_forward"] = block(r_ms, r_alg)
    if backward and x.dtype == torch.float32:
        g_out = synth.upstream_grad((B, D), seed=3, device=dev)
        g_h1 = synth.upstream_grad((B, k1, D), seed=4, device=dev) if hops == 2 else None
        grad_x = torch.zeros((N, D), dtype=torch.float32, device=dev)
        p_go, p_gh, p_gx = g_out.data_ptr(), None if g_h1 is None else g_h1.data_ptr(), grad_x.data_ptr()

        def bwd(i):
            rc = L.fsa_mean_bwd(p_go, p_gh, id1_p[i], i2(i), B, k1, k2, D, p_gx, N, stream)
            if rc != 0:
                raise RuntimeError("fsa_mean_bwd -> %d" % rc)
        b_ms = timed(bwd)                       # accumulates on; zero-filling grad_x is the caller's
        payload = leaf * D * 4
        # every leaf row of grad_x read and written once, its ID, the upstream gradient rows
        b_alg = 2 * payload + 4 * leaf + B * D * 4 + (B * k1 * D * 4 if hops == 2 else 0)
        r["backward"] = block(b_ms, b_alg, atomic_payload_gbps=payload / (b_ms * 1e-3) / 1e9,
                              vs_forward=b_ms / f_ms)
        # the same backward given a workspace: wide-row 2-hop shapes then update each destination
        # row once, without atomics (other shapes take the atomic route again and are not repeated)
        ws_bytes = int(L.fsa_mean_bwd_workspace_bytes(B, k1, k2, D)) if hops == 2 else 0
        if ws_bytes > 0:
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
            p_ws = ws.data_ptr()

            def bwd_ws(i):
                rc = L.fsa_mean_bwd_ws(p_go, p_gh, id1_p[i], i2(i), B, k1, k2, D, p_gx, N, p_ws, ws_bytes, stream)
                if rc != 0:
                    raise RuntimeError("fsa_mean_bwd_ws -> %d" % rc)
            w_ms = timed(bwd_ws)
            r["backward_with_workspace"] = block(w_ms, b_alg, payload_gbps=payload / (w_ms * 1e-3) / 1e9,
                                                 vs_forward=w_ms / f_ms, workspace_bytes=ws_bytes)
            del ws
        del g_out, g_h1, grad_x
    log("[bench] %s B=%d %s: %s" % (w.name, B, r["dtype"], ", ".join(
        "%s %.1f us (%.3f)" % (k, r[k]["launch_us"], r[k]["frac"])
        for k in ("forward", "replay_forward", "backward", "backward_with_workspace") if k in r)))
    return r


def load_or_make_workload(name, scale, cache, dev):
    """The seeded workload, generated on the GPU, or the same bytes re-read from raw files."""
    import numpy as np
    import torch
    from paper_2511_13645_amd import synth
    tdt = {"int32": torch.int32, "int64": torch.int64, "float32": torch.float32, "bfloat16": torch.bfloat16}
    ndt = {"int32": np.int32, "int64": np.int64, "float32": np.float32, "bfloat16": np.int16}
    meta_path = os.path.join(cache, "meta.json") if cache else ""
    if cache and os.path.exists(meta_path):
        m = json.load(open(meta_path))
        if m["name"] != name or m["scale"] != scale:
            raise RuntimeError("cache %s holds %s at scale %g" % (cache, m["name"], m["scale"]))

        def rd(fn, dt, shape):
            t = torch.from_numpy(np.fromfile(os.path.join(cache, fn), dtype=ndt[dt]).reshape(shape)).to(dev)
            return t.view(torch.bfloat16) if dt == "bfloat16" else t
        g = synth.Graph(rd("indptr.bin", m["indptr"], (m["N"] + 1,)), rd("indices.bin", "int32", (m["E"],)), m["N"])
        return synth.Workload(name, g, rd("x.bin", m["x"], (m["N"], m["D"])), m["B"], tuple(m["fan"]), m["seed"])
    w = synth.make_workload(name, device=dev, scale=scale)
    if cache:
        os.makedirs(cache, exist_ok=True)
        for fn, t in (("indptr.bin", w.graph.indptr), ("indices.bin", w.graph.indices), ("x.bin", w.x)):
            (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).cpu().numpy().tofile(os.path.join(cache, fn))
        json.dump({"name": name, "scale": scale, "N": w.graph.num_nodes, "E": w.graph.num_edges, "D": w.x.shape[1],
                   "indptr": str(w.graph.indptr.dtype).split(".")[1], "x": str(w.x.dtype).split(".")[1],
                   "B": w.batch, "fan": list(w.fanouts), "seed": w.sampler_seed}, open(meta_path, "w"))
    return w


def three_hop(args, L, binding, synth, torch, w, B, dev) -> int:
    """One step = fsa_sample_mean3_fwd (one-hop kernel, fused two-hop kernel over the B*k1 hop-1
    slots, slot mean) on a fresh seed batch, IDs of all three levels emitted."""
    g, x = w.graph, w.x
    k1, k2 = w.fanouts
    k3 = args.three_hop
    N, D = x.shape
    elem, iptr = x.element_size(), g.indptr.element_size()
    steps, warmup = args.steps, args.warmup
    emit = not args.no_emit
    seeds = synth.seed_batches(N, B, steps + warmup, seed=2).to(dev)
    out = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_m1 = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=dev)
    cnt2 = torch.empty((B, k1), dtype=torch.int32, device=dev)
    ids1 = torch.empty((B, k1), dtype=torch.int32, device=dev)
    ids2 = torch.empty((B, k1, k2), dtype=torch.int32, device=dev)
    ids3 = torch.empty((B, k1, k2, k3), dtype=torch.int32, device=dev)
    fan_host = (ctypes.c_int32 * 3)(k1, k2, k3)
    stream = torch.cuda.current_stream().cuda_stream
    x_code = {torch.float32: binding.FSA_F32, torch.bfloat16: binding.FSA_BF16, torch.float16: binding.FSA_F16}[x.dtype]

    def step(i, with_ids):
        rc = L.fsa_sample_mean3_fwd(g.indptr.data_ptr(), binding.FSA_I64 if iptr == 8 else binding.FSA_I32,
                                    g.indices.data_ptr(), N, x.data_ptr(), x_code, D, seeds[i].data_ptr(), B,
                                    ctypes.cast(fan_host, ctypes.c_void_p), w.sampler_seed, out.data_ptr(),
                                    out_h1.data_ptr(), None, out_m1.data_ptr(), ids1.data_ptr(),
                                    ids2.data_ptr() if with_ids else None, ids3.data_ptr() if with_ids else None,
                                    cnt2.data_ptr(), stream)
        if rc != 0:
            raise RuntimeError("fsa_sample_mean3_fwd -> %d" % rc)
    for i in range(warmup):
        step(i, emit)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_start = time.perf_counter()
    ev0.record()
    for i in range(warmup, warmup + steps):
        step(i, emit)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    step_ms = ev0.elapsed_time(ev1) / steps
    # rows of a few of the timed batches, counted by untimed emitting calls
    n_cnt = min(steps, 5)
    leaf = live2 = live1 = 0
    for i in range(warmup, warmup + n_cnt):
        step(i, True)
        leaf += int((ids3 >= 0).sum().item())
        live2 += int((ids2 >= 0).sum().item())
        live1 += int((ids1 >= 0).sum().item())
    leaf, live2, live1 = leaf / n_cnt, live2 / n_cnt, live1 / n_cnt
    # bytes the method must move per step: every leaf row once with its `indices` entry; an indptr
    # pair and an `indices` entry per sampled row owner; the hop-1 rows for out_m1; out_h1 written
    # and read back once by the slot mean; ids1 / cnt2 written and read back; the other outputs once
    alg = leaf * (D * elem + 4) + (live2 + live1) * (4 + 2 * iptr) + B * (2 * iptr + 4)
    alg += live1 * D * elem + 2 * B * D * elem + 2 * B * k1 * D * elem + 4 * 4 * B * k1
    if emit:
        alg += 4 * B * k1 * k2 * (1 + k3)
    achieved = alg / (step_ms * 1e-3) / 1e9
    log("[bench] three-hop %d/%d/%d: %.1f us/step by events, %.0f leaf rows/step, %.1f MB algorithmic/step" %
        (k1, k2, k3, step_ms * 1e3, leaf, alg / 1e6))
    other_paths = None
    if args.paths:
        other_paths = {}
        n_p = min(steps, 20)
        step(warmup, True)                              # IDs of one batch, reused below
        torch.cuda.synchronize()

        def timed(fn):
            fn(); fn()
            torch.cuda.synchronize()
            ev0.record()
            for _ in range(n_p):
                fn()
            ev1.record()
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) / n_p

        def replay():
            rc = L.fsa_mean3_replay_fwd(x.data_ptr(), x_code, D, N, ids1.data_ptr(), ids2.data_ptr(), ids3.data_ptr(),
                                        B, k1, k2, k3, out.data_ptr(), out_h1.data_ptr(), None, out_m1.data_ptr(),
                                        cnt2.data_ptr(), stream)
            if rc != 0:
                raise RuntimeError("fsa_mean3_replay_fwd -> %d" % rc)
        r_ms = timed(replay)
        rows_b = int((ids3 >= 0).sum().item())
        other_paths["replay_forward"] = {"launch_us": r_ms * 1e3, "rows_per_s": rows_b / (r_ms * 1e-3)}
        if x.dtype == torch.float32:
            g_out = synth.upstream_grad((B, D), seed=3, device=dev)
            g_h1 = synth.upstream_grad((B, k1, D), seed=4, device=dev)
            work = torch.empty((B, k1, D), dtype=torch.float32, device=dev)
            grad_x = torch.zeros((N, D), dtype=torch.float32, device=dev)

            def bwd():
                rc = L.fsa_mean3_bwd(g_out.data_ptr(), g_h1.data_ptr(), None, None, ids1.data_ptr(), ids2.data_ptr(),
                                     ids3.data_ptr(), B, k1, k2, k3, D, grad_x.data_ptr(), N, work.data_ptr(), stream)
                if rc != 0:
                    raise RuntimeError("fsa_mean3_bwd -> %d" % rc)
            b_ms = timed(bwd)
            other_paths["backward"] = {"launch_us": b_ms * 1e3, "rows_per_s": rows_b / (b_ms * 1e-3),
                                       "atomic_payload_gbps": rows_b * D * 4 / (b_ms * 1e-3) / 1e9}
        log("[bench] three-hop other paths: %s" % json.dumps(other_paths))

    line = {
        "metric": "sampled neighbor rows aggregated/sec + achieved HBM GB/s, fanout %d/%d/%d D=%d" % (k1, k2, k3, D),
        "value": leaf * steps / wall, "unit": "rows/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": wall * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if x.dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": "%s three-hop: N=%d, E=%d, D=%d, B=%d, fanouts=[%d, %d, %d], emit_ids=%s" %
                               (w.name, N, g.num_edges, D, B, k1, k2, k3, emit),
                   "global_batch": B, "rows_per_launch": leaf, "algorithmic_bytes_per_launch": alg},
        "hbm_gbps": achieved,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                     "kernel": "fwd1_kernel + fwd2_kernel + slot_mean_kernel (one step)", "launch_us": step_ms * 1e3},
        "cpu_baseline": None,
        "other_paths": other_paths,
    }
    print(json.dumps(line), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="citation", choices=["tiny", "products", "social", "kg", "citation"])
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graph (rehearsals only)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle leg (0 = skip)")
    ap.add_argument("--no-emit", action="store_true", help="do not emit IDs / per-slot means")
    ap.add_argument("--saturated-batch", type=int, default=65536,
                    help="also time a few launches at this batch size on the same graph (0 = skip)")
    ap.add_argument("--cache", default="", help="directory with raw copies of the workload: written if "
                    "absent, loaded if present (counter runs use it: rocprofv3 --pmc does not survive the "
                    "in-process generation of the full-size graph on this image)")
    ap.add_argument("--paths", action="store_true",
                    help="also time the replay forward and the backward variants on the same batches")
    ap.add_argument("--batch-sweep", default="", help="comma-separated batch sizes: time the forward at each, "
                    "with and without ID / per-slot emission, on the same graph")
    ap.add_argument("--feature-dtype", default="", choices=["", "f32", "bf16"],
                    help="convert the workload's feature table to this type first (fp32 variant of the headline)")
    ap.add_argument("--weighted", action="store_true",
                    help="also time the weighted-mean forward, replay and (fp32 tables) backward on the same batches")
    ap.add_argument("--three-hop", type=int, default=0, metavar="K3",
                    help="time the three-hop forward (workload fanouts + K3) instead of the workload's own path")
    ap.add_argument("--ceilings", type=int, default=0, metavar="GB",
                    help="first measure what this GPU sustains on plain access patterns over a table of GB GiB "
                         "(streaming read, copy, random row gather, row atomics, row stores); adds `ceilings`")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a 1 GiB device-to-device copy first, so a counter run can scale its byte counters")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the fp32-table variant of the headline shape and the other workload shapes "
                         "(`fp32_variant`, `workloads`), which the default run of the citation workload adds")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: write profiles/traffic_<workload>.json from two rocprofv3 --pmc counter CSVs")
    ap.add_argument("--traffic-kernel", default="fwd2_kernel", help="kernel name fragment for --traffic-from")
    ap.add_argument("--only-paths", default="", metavar="NAMES",
                    help="comma-separated workloads: measure forward, replay forward and backward (also with a "
                         "workspace) of each at its own batch size, print them as one JSON line and stop")
    ap.add_argument("--lib", default="", help="load this build of the library instead of libfsa_hip.so (debug builds)")
    ap.add_argument("--trace-roots", action="store_true",
                    help="per-root timeline of the 2-hop forward; needs --lib with a build made with -DFSA_TRACE")
    args = ap.parse_args()
    if args.traffic_from:
        return traffic_from_counters(args)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU by scope (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2511_13645_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    if args.lib:
        binding.LIB_PATH = os.path.abspath(args.lib)
    L = binding.lib()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ceilings = None
    if args.ceilings:
        if not os.path.exists(CEILINGS_LIB):
            raise RuntimeError("%s missing: build it with __graft_entry__.build()" % CEILINGS_LIB)
        C = ctypes.CDLL(CEILINGS_LIB)
        C.fsa_ceilings_measure.argtypes = [ctypes.c_int, ctypes.c_void_p]
        C.fsa_ceilings_measure.restype = ctypes.c_int
        vals = (ctypes.c_double * 7)()
        torch.cuda.synchronize()
        rc = C.fsa_ceilings_measure(args.ceilings, ctypes.cast(vals, ctypes.c_void_p))
        if rc != 0:
            raise RuntimeError("fsa_ceilings_measure -> %d" % rc)
        names = ("streaming_read", "copy_read_plus_write", "gather_256B_rows", "gather_512B_rows",
                 "atomic_add_f32_512B_rows", "atomic_pk_add_bf16_256B_rows", "store_512B_rows")
        ceilings = {"unit": "GB/s", "table_gib": args.ceilings, **{n: vals[i] for i, n in enumerate(names)}}
        log("[bench] ceilings: %s" % json.dumps(ceilings))

    if args.only_paths:
        res = []
        for name in args.only_paths.split(","):
            wk = synth.make_workload(name, device=dev, scale=args.scale)
            res.append(measure_paths(L, binding, synth, torch, wk, args.batch or wk.batch, dev, n_launch=args.steps if args.steps < 200 else 20))
            del wk
            torch.cuda.empty_cache()
        print(json.dumps({"workloads": res}), flush=True)
        return 0

    t0 = time.time()
    w = load_or_make_workload(args.workload, args.scale, args.cache, dev)
    torch.cuda.synchronize()
    want = {"": None, "f32": torch.float32, "bf16": torch.bfloat16}[args.feature_dtype]
    if want is not None and w.x.dtype != want:
        w.x = w.x.to(want)
    g, x = w.graph, w.x
    B = args.batch or w.batch
    fan = list(w.fanouts)
    hops = len(fan)
    k1 = fan[0]
    k2 = fan[1] if hops == 2 else 0
    N, D = x.shape
    elem = x.element_size()
    iptr = g.indptr.element_size()
    log("[bench] %s: N=%d E=%d D=%d %s B=%d fanouts=%s built in %.1fs" %
        (w.name, N, g.num_edges, D, str(x.dtype), B, fan, time.time() - t0))

    steps, warmup = args.steps, args.warmup
    if args.trace_roots:
        return trace_roots(L, binding, synth, torch, w, dev)
    if args.three_hop:
        if hops != 2:
            print("bench.py: --three-hop needs a two-hop workload", file=sys.stderr)
            return 2
        return three_hop(args, L, binding, synth, torch, w, B, dev)
    seeds = synth.seed_batches(N, B, steps + warmup, seed=2).to(dev)
    emit = not args.no_emit
    out = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=dev) if (hops == 2 and emit) else None
    # every launch emits its IDs into its own slice, so the rows it aggregated can be counted
    # after the timed region without launching anything else
    n_id = (steps + warmup) if emit else 1
    ids1 = torch.empty((n_id, B, k1), dtype=torch.int32, device=dev)
    ids2 = torch.empty((n_id, B, k1, k2), dtype=torch.int32, device=dev) if hops == 2 else None

    fan_host = (ctypes.c_int32 * hops)(*fan)
    stream = torch.cuda.current_stream().cuda_stream
    fixed_head = (g.indptr.data_ptr(), binding.FSA_I64 if iptr == 8 else binding.FSA_I32, g.indices.data_ptr(), N,
                  x.data_ptr(), binding.FSA_BF16 if x.dtype == torch.bfloat16 else binding.FSA_F32, D)
    fixed_mid = (B, ctypes.cast(fan_host, ctypes.c_void_p), hops, w.sampler_seed,
                 out.data_ptr(), None if out_h1 is None else out_h1.data_ptr())
    seed_ptrs = [seeds[i].data_ptr() for i in range(steps + warmup)]
    id1_ptrs = [ids1[i].data_ptr() if emit else None for i in range(steps + warmup)]
    id2_ptrs = [ids2[i].data_ptr() if (emit and hops == 2) else None for i in range(steps + warmup)]
    fwd = L.fsa_sample_mean_fwd

    def step(i):
        rc = fwd(*fixed_head, seed_ptrs[i], *fixed_mid, id1_ptrs[i], id2_ptrs[i], stream)
        if rc != 0:
            raise RuntimeError("fsa_sample_mean_fwd -> %d" % rc)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_start = time.perf_counter()
    ev0.record()
    for i in range(warmup, warmup + steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ev_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall * 1e3 / steps
    kern_ms = ev_ms / steps

    # per-launch durations (median, p10, p90) from an event pair around each launch of a second,
    # untimed pass over the same batches (the paper's protocol reports the median of 200)
    n_pl = min(steps, 200)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_pl)]
    for i in range(n_pl):
        evs[i][0].record()
        step(warmup + i)
        evs[i][1].record()
    torch.cuda.synchronize()
    per_launch = sorted(a.elapsed_time(b_) * 1e3 for a, b_ in evs)
    pct = {"median": per_launch[n_pl // 2], "p10": per_launch[n_pl // 10], "p90": per_launch[(9 * n_pl) // 10]}

    # what the timed launches actually aggregated
    leaf_rows = 0
    hop1_rows = 0
    if emit:
        if hops == 2:
            leaf_rows = int((ids2[warmup:] >= 0).sum().item())
            hop1_rows = int((ids1[warmup:] >= 0).sum().item())
        else:
            leaf_rows = int((ids1[warmup:] >= 0).sum().item())
    else:                            # nothing was emitted: count with untimed emitting launches
        for i in range(warmup, warmup + steps):
            rc = fwd(*fixed_head, seed_ptrs[i], *fixed_mid[:-1], None, ids1[0].data_ptr(),
                     ids2[0].data_ptr() if hops == 2 else None, stream)
            if rc != 0:
                raise RuntimeError("fsa_sample_mean_fwd -> %d" % rc)
            if hops == 2:
                leaf_rows += int((ids2[0] >= 0).sum().item())
                hop1_rows += int((ids1[0] >= 0).sum().item())
            else:
                leaf_rows += int((ids1[0] >= 0).sum().item())
    if hops == 2:
        alg = algorithmic_bytes(leaf_rows, hop1_rows, B * steps, k1, k2, D, elem, iptr, emit, emit)
    else:
        alg = leaf_rows * (D * elem + 4) + B * steps * (2 * iptr + 4 + D * elem) + (4 * B * steps * k1 if emit else 0)
    alg_per_launch = alg / steps
    rows_per_s = leaf_rows / wall
    achieved = alg_per_launch / (kern_ms * 1e-3) / 1e9
    log("[bench] %.1f us/step wall, %.1f us/launch by events, %.0f rows/launch, %.1f MB algorithmic/launch" %
        (ms_per_step * 1e3, kern_ms * 1e3, leaf_rows / steps, alg_per_launch / 1e6))

    traffic = None
    # the committed counter runs cover the workload as named (its own batch, table type, emission on)
    if not args.batch and not args.feature_dtype and emit and args.scale == 1.0:
        traffic = committed_traffic(w.name)

    other_paths = None
    if args.paths and emit:
        # replay forward and backward on the IDs the timed launches emitted (one launch per batch)
        other_paths = {}
        n_p = min(steps, 50)
        replay = L.fsa_mean_replay_fwd
        x_code = binding.FSA_BF16 if x.dtype == torch.bfloat16 else binding.FSA_F32

        def run_replay(i):
            rc = replay(x.data_ptr(), x_code, D, N, id1_ptrs[i], id2_ptrs[i], B, k1, k2, out.data_ptr(),
                        None if out_h1 is None else out_h1.data_ptr(), stream)
            if rc != 0:
                raise RuntimeError("fsa_mean_replay_fwd -> %d" % rc)
        for i in range(warmup, warmup + 3):
            run_replay(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(warmup, warmup + n_p):
            run_replay(i)
        e1.record()
        torch.cuda.synchronize()
        r_ms = e0.elapsed_time(e1) / n_p
        rows_p = leaf_rows / steps
        r_alg = rows_p * (D * elem + 4) + B * D * elem + (B * k1 * D * elem + 4 * B * k1 if hops == 2 else 0)
        other_paths["replay_forward"] = {"launch_us": r_ms * 1e3, "rows_per_s": rows_p / (r_ms * 1e-3),
                                         "hbm_gbps": r_alg / (r_ms * 1e-3) / 1e9,
                                         "frac": r_alg / (r_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        # backward: fp32 throughout (fp32 tables), then 16-bit upstream gradients into an fp32
        # master gradient, then a bf16 grad_x by packed atomics
        combos = [("backward_bf16_grads_f32_master", torch.bfloat16, torch.float32),
                  ("backward_bf16_packed_atomics", torch.bfloat16, torch.bfloat16)]
        if x.dtype == torch.float32:
            combos.insert(0, ("backward", torch.float32, torch.float32))
        if D % 2:
            combos = [c for c in combos if c[1] == torch.float32 and c[2] == torch.float32]
        code = {torch.float32: binding.FSA_F32, torch.bfloat16: binding.FSA_BF16}
        bwd_lp = L.fsa_mean_bwd_lp
        for key, g_dt, gx_dt in combos:
            g_out = synth.upstream_grad((B, D), seed=3, device=dev).to(g_dt)
            g_h1 = synth.upstream_grad((B, k1, D), seed=4, device=dev).to(g_dt) if hops == 2 else None
            grad_x = torch.zeros((N, D), dtype=gx_dt, device=dev)

            def run_bwd(i):
                rc = bwd_lp(g_out.data_ptr(), None if g_h1 is None else g_h1.data_ptr(), code[g_dt],
                            id1_ptrs[i], id2_ptrs[i], B, k1, k2, D, grad_x.data_ptr(), code[gx_dt], N, stream)
                if rc != 0:
                    raise RuntimeError("fsa_mean_bwd_lp -> %d" % rc)
            for i in range(warmup, warmup + 2):
                run_bwd(i)
            torch.cuda.synchronize()
            e0.record()
            for i in range(warmup, warmup + n_p):
                run_bwd(i)                          # accumulates on; zero-filling grad_x is the caller's
            e1.record()
            torch.cuda.synchronize()
            b_ms = e0.elapsed_time(e1) / n_p
            ge, xe = g_out.element_size(), grad_x.element_size()
            payload = rows_p * D * xe               # bytes added into grad_x by atomics
            b_alg = 2 * payload + 4 * rows_p + B * D * ge + (B * k1 * D * ge if hops == 2 else 0)
            other_paths[key] = {"launch_us": b_ms * 1e3, "rows_per_s": rows_p / (b_ms * 1e-3),
                                "atomic_payload_gbps": payload / (b_ms * 1e-3) / 1e9,
                                "hbm_gbps": b_alg / (b_ms * 1e-3) / 1e9,
                                "frac": b_alg / (b_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
            if "grad_x_zero_fill" not in other_paths or gx_dt == torch.float32:
                # the caller's zero-fill of the gradient table, never part of the backward's time
                grad_x.zero_()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(3):
                    grad_x.zero_()
                e1.record()
                torch.cuda.synchronize()
                other_paths["grad_x_zero_fill"] = {"launch_us": e0.elapsed_time(e1) / 3 * 1e3,
                                                   "bytes": grad_x.numel() * grad_x.element_size(),
                                                   "dtype": str(gx_dt).split(".")[1]}
            del g_out, g_h1, grad_x
        log("[bench] other paths: %s" % json.dumps(other_paths))

    weighted = None
    if args.weighted and emit:
        # the weighted mean on the same batches: hashed uniform weights in [0,1) per edge
        weighted = {}
        n_p = min(steps, 50)
        ew = synth.edge_weights(g.num_edges, seed=11, device=dev)
        x_code_w = {torch.float32: binding.FSA_F32, torch.bfloat16: binding.FSA_BF16, torch.float16: binding.FSA_F16}[x.dtype]
        w1 = torch.empty((n_p, B, k1), dtype=torch.float32, device=dev)
        w2 = torch.empty((n_p, B, k1, k2), dtype=torch.float32, device=dev) if hops == 2 else None
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def timed_w(fn):
            for i in range(2):
                fn(i)
            torch.cuda.synchronize()
            e0.record()
            for i in range(n_p):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n_p * 1e3

        def w_fwd(i):
            rc = L.fsa_sample_wmean_fwd(fixed_head[0], fixed_head[1], fixed_head[2], ew.data_ptr(), N, x.data_ptr(), x_code_w, D,
                                        seed_ptrs[warmup + i], B, ctypes.cast(fan_host, ctypes.c_void_p), hops, w.sampler_seed,
                                        out.data_ptr(), None if out_h1 is None else out_h1.data_ptr(),
                                        id1_ptrs[warmup + i], id2_ptrs[warmup + i], w1[i].data_ptr(),
                                        None if w2 is None else w2[i].data_ptr(), stream)
            if rc != 0:
                raise RuntimeError("fsa_sample_wmean_fwd -> %d" % rc)

        def w_replay(i):
            rc = L.fsa_wmean_replay_fwd(x.data_ptr(), x_code_w, D, N, id1_ptrs[warmup + i], id2_ptrs[warmup + i], w1[i].data_ptr(),
                                        None if w2 is None else w2[i].data_ptr(), B, k1, k2, out.data_ptr(),
                                        None if out_h1 is None else out_h1.data_ptr(), stream)
            if rc != 0:
                raise RuntimeError("fsa_wmean_replay_fwd -> %d" % rc)
        weighted["forward_us"] = timed_w(w_fwd)
        weighted["replay_forward_us"] = timed_w(w_replay)
        if x.dtype == torch.float32:
            g_out = synth.upstream_grad((B, D), seed=3, device=dev)
            grad_x = torch.zeros((N, D), dtype=torch.float32, device=dev)

            def w_bwd(i):
                rc = L.fsa_wmean_bwd(g_out.data_ptr(), None, id1_ptrs[warmup + i], id2_ptrs[warmup + i], w1[i].data_ptr(),
                                     None if w2 is None else w2[i].data_ptr(), B, k1, k2, D, grad_x.data_ptr(), N, stream)
                if rc != 0:
                    raise RuntimeError("fsa_wmean_bwd -> %d" % rc)
            weighted["backward_us"] = timed_w(w_bwd)
            del g_out, grad_x
        weighted["unweighted_forward_us"] = kern_ms * 1e3
        del ew, w1, w2
        log("[bench] weighted mean: %s" % json.dumps(weighted))

    def forward_at_batch(Bs, emit_s, n_launch=20):
        """Time `n_launch` back-to-back forward launches at batch size Bs on the same graph."""
        if Bs > N:                               # seeds are drawn without replacement
            log("[bench] B=%d exceeds the graph's %d nodes: skipped" % (Bs, N))
            return None
        s_seeds = synth.seed_batches(N, Bs, n_launch + 2, seed=5).to(dev)
        s_out = torch.empty((Bs, D), dtype=x.dtype, device=dev)
        s_h1 = torch.empty((Bs, k1, D), dtype=x.dtype, device=dev) if (emit_s and hops == 2) else None
        s_i1 = torch.empty((Bs, k1), dtype=torch.int32, device=dev) if emit_s else None
        s_i2 = torch.empty((Bs, k1, k2), dtype=torch.int32, device=dev) if (emit_s and hops == 2) else None
        tail = (Bs, ctypes.cast(fan_host, ctypes.c_void_p), hops, w.sampler_seed, s_out.data_ptr(),
                None if s_h1 is None else s_h1.data_ptr(), None if s_i1 is None else s_i1.data_ptr(),
                None if s_i2 is None else s_i2.data_ptr(), stream)
        for i in range(2):
            rc = fwd(*fixed_head, s_seeds[i].data_ptr(), *tail)
            if rc != 0:
                raise RuntimeError("fsa_sample_mean_fwd -> %d" % rc)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(2, n_launch + 2):
            fwd(*fixed_head, s_seeds[i].data_ptr(), *tail)
        e1.record()
        torch.cuda.synchronize()
        s_ms = e0.elapsed_time(e1) / n_launch
        # rows of one of the timed batches, counted by an untimed emitting launch
        o, h, i1, i2 = binding.fsa_sample_mean_fwd(g.indptr, g.indices, x, s_seeds[2], fan, w.sampler_seed, emit_h1=False)
        if hops == 2:
            s_leaf, s_hop1 = int((i2 >= 0).sum().item()), int((i1 >= 0).sum().item())
            s_alg = algorithmic_bytes(s_leaf, s_hop1, Bs, k1, k2, D, elem, iptr, emit_s, emit_s)
        else:
            s_leaf = int((i1 >= 0).sum().item())
            s_alg = s_leaf * (D * elem + 4) + Bs * (2 * iptr + 4 + D * elem) + (4 * Bs * k1 if emit_s else 0)
        r = {"global_batch": Bs, "emit": emit_s, "launch_us": s_ms * 1e3, "rows_per_s": s_leaf / (s_ms * 1e-3),
             "hbm_gbps": s_alg / (s_ms * 1e-3) / 1e9, "frac": s_alg / (s_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        log("[bench] B=%d emit=%s: %.1f us/launch, %.2f G rows/s, %.0f GB/s algorithmic (%.3f)" %
            (Bs, emit_s, s_ms * 1e3, r["rows_per_s"] / 1e9, r["hbm_gbps"], r["frac"]))
        return r

    saturated = forward_at_batch(args.saturated_batch, emit) if args.saturated_batch > 0 else None
    batch_sweep = None
    if args.batch_sweep:
        batch_sweep = [forward_at_batch(int(b), e) for b in args.batch_sweep.split(",") for e in (True, False)]

    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        t1 = time.time()
        h_indptr = g.indptr.cpu().numpy()
        h_indices = g.indices.cpu().numpy()
        if x.dtype == torch.bfloat16:
            h_x, is_bf16 = x.cpu().view(torch.int16).numpy().view(np.uint16), True
        else:
            h_x, is_bf16 = x.cpu().numpy(), False
        log("[bench] host copies for the oracle in %.1fs" % (time.time() - t1))
        h_seeds = seeds.cpu().numpy()
        oracle.lib()
        done_rows, done_batches, spent = 0, 0, 0.0
        sample_b = B
        while spent < args.cpu_seconds:
            sb = h_seeds[warmup + done_batches % steps][:sample_b]
            c0 = time.perf_counter()
            r = oracle.sample_mean_fwd(h_indptr, h_indices, h_x, sb, fan, w.sampler_seed, bf16=is_bf16)
            spent += time.perf_counter() - c0
            done_rows += int((r[3] >= 0).sum()) if hops == 2 else int((r[2] >= 0).sum())
            done_batches += 1
        cpu = {"value": done_rows / spent, "unit": "rows/s", "cores": 1, "kind": "oracle",
               "sample": "%d of the timed batches (B=%d each), %.1f s of single-thread oracle "
                         "(sampling + fp64 means, same graph and table on the host)" % (done_batches, sample_b, spent)}
        # the same unchanged oracle on every host core: this harness cuts a batch into one
        # contiguous slice of seeds per thread (ctypes releases the interpreter lock in the call)
        from concurrent.futures import ThreadPoolExecutor
        n_thr = max(1, min(int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1), os.cpu_count() or 1))
        if n_thr > 1 and B >= n_thr:
            bounds = [B * t // n_thr for t in range(n_thr + 1)]

            def run_slice(args_):
                sb, lo, hi = args_
                r = oracle.sample_mean_fwd(h_indptr, h_indices, h_x, sb[lo:hi], fan, w.sampler_seed, bf16=is_bf16)
                return int((r[3] >= 0).sum()) if hops == 2 else int((r[2] >= 0).sum())
            rows_mt, batches_mt, spent_mt = 0, 0, 0.0
            with ThreadPoolExecutor(max_workers=n_thr) as pool:
                while spent_mt < max(2.0, args.cpu_seconds / 3):
                    sb = h_seeds[warmup + batches_mt % steps]
                    c0 = time.perf_counter()
                    rows_mt += sum(pool.map(run_slice, [(sb, bounds[t], bounds[t + 1]) for t in range(n_thr)]))
                    spent_mt += time.perf_counter() - c0
                    batches_mt += 1
            cpu["all_cores"] = {"value": rows_mt / spent_mt, "unit": "rows/s", "cores": n_thr,
                                "sample": "%d batches in %.1f s, one slice of seeds per thread" % (batches_mt, spent_mt)}

    # the claims about the other shapes, under the same clock as the headline: the same graph with
    # the table widened to fp32 (D = 128, 56.8 GB) at the headline batch and at the saturating one,
    # then the product, social and KG shapes, each with forward, replay forward and backward
    workload_text = ("%s: N=%d, E=%d, D=%d %s, %s indptr, B=%d, fanouts=%s, emit_ids=%s, scale=%g" %
                     (w.name, N, g.num_edges, D, "bf16" if elem == 2 else "fp32",
                      "int64" if iptr == 8 else "int32", B, fan, emit, args.scale))
    x_is_bf16 = x.dtype == torch.bfloat16
    fp32_variant = None
    workloads = None
    if (not args.no_extras and w.name == "citation" and not args.batch and not args.feature_dtype
            and args.scale == 1.0 and emit):
        del seeds, out, out_h1, ids1, ids2
        w32 = synth.Workload(w.name, g, x.float(), B, tuple(fan), w.sampler_seed)
        fp32_variant = [measure_paths(L, binding, synth, torch, w32, B, dev),
                        measure_paths(L, binding, synth, torch, w32, 65536, dev, replay=False, backward=False)]
        del w32, w, g, x
        torch.cuda.empty_cache()
        workloads = []
        for name in ("products", "social", "kg"):
            wk = synth.make_workload(name, device=dev)
            workloads.append(measure_paths(L, binding, synth, torch, wk, wk.batch, dev))
            if name == "kg":
                workloads.append(measure_paths(L, binding, synth, torch, wk, 65536, dev))
            del wk
            torch.cuda.empty_cache()

    line = {
        "metric": "sampled neighbor rows aggregated/sec + achieved HBM GB/s, fanout %s D=%d" % ("/".join(map(str, fan)), D),
        "value": rows_per_s, "unit": "rows/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if x_is_bf16 else "f32", "data": "synthetic",
        "config": {"workload": workload_text,
                   "global_batch": B, "rows_per_launch": leaf_rows / steps,
                   "algorithmic_bytes_per_launch": alg_per_launch},
        "hbm_gbps": achieved,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "fwd2_kernel" if hops == 2 else "fwd1_kernel", "launch_us": kern_ms * 1e3,
                     "launch_us_event_pairs": pct},
        "cpu_baseline": cpu,
        "saturated": saturated,
        "fp32_variant": fp32_variant,
        "workloads": workloads,
        "other_paths": other_paths,
        "batch_sweep": batch_sweep,
        "ceilings": ceilings,
        "weighted": weighted,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
