"""Training step around the fused operator, timed the way the paper times its Tables 2-3
(Sec. 5: forward + backward + optimizer, device-synchronised, 20 warm-up + 200 timed steps,
median; peak transient memory of the timed region excluding parameters and resident features).

The encoder is the paper's "lightweight 2-hop encoder composed with an MLP": the fused
neighborhood context [B,D] feeds a two-layer MLP trained on synthetic labels.  With
``--learn-table`` the feature table is a learnable embedding (the KG-completion setting) and
the step also runs the operator's backward and a dense optimizer update of the table.

    python -m paper_2511_13645_amd.train_step --workload products --steps 200
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys
import time


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="products", choices=["tiny", "products", "social", "kg", "citation"])
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--fanouts", default="", help="override, e.g. 25,10")
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--hidden", type=int, default=256)
    ap.add_argument("--classes", type=int, default=47)
    ap.add_argument("--learn-table", action="store_true")
    ap.add_argument("--scale", type=float, default=1.0)
    args = ap.parse_args()

    import torch
    from . import synth
    from .autograd import fused_sample_mean

    dev = "cuda:0"
    w = synth.make_workload(args.workload, device=dev, scale=args.scale)
    g = w.graph
    fan = [int(t) for t in args.fanouts.split(",")] if args.fanouts else list(w.fanouts)
    B = args.batch or w.batch
    N, D = w.x.shape
    x = w.x.float() if args.learn_table else w.x
    if args.learn_table:
        x = torch.nn.Parameter(x)
    torch.manual_seed(0)
    mlp = torch.nn.Sequential(torch.nn.Linear(D, args.hidden), torch.nn.ReLU(),
                              torch.nn.Linear(args.hidden, args.classes)).to(dev)
    params = list(mlp.parameters()) + ([x] if args.learn_table else [])
    opt = torch.optim.SGD(params, lr=0.01)
    n = args.steps + args.warmup
    seeds = synth.seed_batches(N, B, n, seed=2).to(dev)
    labels = (synth.hash64(9, 0, torch.arange(n * B, device=dev)) % args.classes).abs().view(n, B)
    loss_fn = torch.nn.CrossEntropyLoss()

    times = []
    resident = 0
    for i in range(n):
        if i == args.warmup:                       # library workspaces exist by now: not transient
            torch.cuda.synchronize()
            resident = torch.cuda.memory_allocated()
            torch.cuda.reset_peak_memory_stats()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx_vec, _, _, _ = fused_sample_mean(x, g.indptr, g.indices, seeds[i], fan, w.sampler_seed)
        loss = loss_fn(mlp(ctx_vec.float()), labels[i])
        opt.zero_grad(set_to_none=True)
        loss.backward()
        opt.step()
        torch.cuda.synchronize()
        if i >= args.warmup:
            times.append((time.perf_counter() - t0) * 1e3)
    peak = torch.cuda.max_memory_allocated() - resident
    line = {"what": "training step (fused forward%s + MLP + SGD), device-synchronised" %
                    (" + operator backward + dense table update" if args.learn_table else ""),
            "workload": "%s: N=%d E=%d D=%d %s B=%d fanouts=%s" % (w.name, N, g.num_edges, D, str(w.x.dtype), B, fan),
            "steps": args.steps, "warmup": args.warmup,
            "median_ms": statistics.median(times), "p10_ms": sorted(times)[len(times) // 10],
            "p90_ms": sorted(times)[(len(times) * 9) // 10],
            "peak_transient_mb": peak / 1e6, "final_loss": float(loss.item())}
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
