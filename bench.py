#!/usr/bin/env python3
"""Benchmark of the fused sample + mean forward on one MI355X.

Default workload: the web-scale citation shape (N = 111 M nodes, ~1.6 B edges, int64 indptr,
bf16 x[N,128], B = 4096 seeds, fanouts 15/10) -- the shape the headline metric (rows
aggregated per second and achieved HBM GB/s at fanout 15/10, D = 128) is quoted on.  One step
is one launch of the fused 2-hop forward with ID and per-slot emission over a fresh batch of
seeds; inputs are resident in HBM before the timed region starts.

Prints ONE JSON line (see the design doc for every field).  `--gpus N` with N > 1 is refused: this
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
    args = ap.parse_args()
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
    L = binding.lib()

    t0 = time.time()
    w = synth.make_workload(args.workload, device=dev, scale=args.scale)
    torch.cuda.synchronize()
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
    seeds = synth.seed_batches(N, B, steps + warmup, seed=2).to(dev)
    emit = not args.no_emit
    out = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=dev) if (hops == 2 and emit) else None
    ids1 = torch.empty((B, k1), dtype=torch.int32, device=dev) if emit else None
    ids2 = torch.empty((B, k1, k2), dtype=torch.int32, device=dev) if (hops == 2 and emit) else None

    fan_host = (ctypes.c_int32 * hops)(*fan)
    stream = torch.cuda.current_stream().cuda_stream
    fixed_head = (g.indptr.data_ptr(), binding.FSA_I64 if iptr == 8 else binding.FSA_I32, g.indices.data_ptr(), N,
                  x.data_ptr(), binding.FSA_BF16 if x.dtype == torch.bfloat16 else binding.FSA_F32, D)
    fixed_tail = (B, ctypes.cast(fan_host, ctypes.c_void_p), hops, w.sampler_seed,
                  out.data_ptr(), None if out_h1 is None else out_h1.data_ptr(),
                  None if ids1 is None else ids1.data_ptr(), None if ids2 is None else ids2.data_ptr(), stream)
    seed_ptrs = [seeds[i].data_ptr() for i in range(steps + warmup)]
    fwd = L.fsa_sample_mean_fwd

    def step(i):
        rc = fwd(*fixed_head, seed_ptrs[i], *fixed_tail)
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

    # what the timed launches actually aggregated (untimed recount of the same batches)
    leaf_rows = 0
    hop1_rows = 0
    for i in range(warmup, warmup + steps):
        o, h, i1, i2 = binding.fsa_sample_mean_fwd(g.indptr, g.indices, x, seeds[i], fan, w.sampler_seed,
                                                   emit_h1=False, emit_ids=True)
        if hops == 2:
            leaf_rows += int((i2 >= 0).sum().item())
            hop1_rows += int((i1 >= 0).sum().item())
        else:
            leaf_rows += int((i1 >= 0).sum().item())
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
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % w.name)
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
        except Exception:
            traffic = None

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

    line = {
        "metric": "sampled neighbor rows aggregated/sec + achieved HBM GB/s, fanout %s D=%d" % ("/".join(map(str, fan)), D),
        "value": rows_per_s, "unit": "rows/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if x.dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": "%s: N=%d, E=%d, D=%d %s, %s indptr, B=%d, fanouts=%s, emit_ids=%s, scale=%g" %
                               (w.name, N, g.num_edges, D, "bf16" if elem == 2 else "fp32",
                                "int64" if iptr == 8 else "int32", B, fan, emit, args.scale),
                   "global_batch": B, "rows_per_launch": leaf_rows / steps,
                   "algorithmic_bytes_per_launch": alg_per_launch},
        "hbm_gbps": achieved,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "fwd2_kernel" if hops == 2 else "fwd1_kernel", "launch_us": kern_ms * 1e3},
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
