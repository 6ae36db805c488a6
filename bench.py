#!/usr/bin/env python3
"""Benchmark of the GVote selection hot path on one MI355X.

A step = one pass of the whole path (fit -> sample/project/RoPE -> score/select -> union/compact)
over one batch of synthetic input that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]

metric: layer-tokens per second = (sum over items of context length L) / step time.
roofline: the kernel that dominates the step, priced on ALGORITHMIC bytes against 8 TB/s HBM.
cpu_baseline: the CPU oracle, untuned, on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(wl, lengths, rho):
    """Bytes the method itself must move per step (no re-reads, no intermediates), by stage."""
    e = wl.elem_bytes
    tok = sum(lengths)
    n_layers_w = 1 if wl.shared_weights else len(lengths)
    fit = tok * wl.d * e
    proj = n_layers_w * wl.n_q_heads * wl.d_k * wl.d * e
    score = tok * wl.n_kv_heads * wl.d_k * e
    compact = 4.0 * rho * tok * wl.n_kv_heads * wl.d_k * e
    return dict(fit=fit, sample=proj, select=score, compact=compact, total=fit + proj + score + compact)


def profiled_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE runs, scaled by a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", "cfg3_hbm_traffic_pmc.txt")
    if workload != "cfg3_llama8b_stack_32k" or not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith(kernel):
            cols = line[38:].split()
            try:
                return (float(cols[2]) + float(cols[3])) * 1e6
            except (IndexError, ValueError):
                return None
    return None


def cpu_baseline(wl, items, n_sample):
    import numpy as np
    import parity_util as U
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    cpu_items = [{k: (v.cpu() if hasattr(v, "cpu") else v) for k, v in it.items()} for it in items[:n_sample]]
    t0 = time.perf_counter()
    for it in cpu_items:
        U.oracle_item(wl, it)
    dt = time.perf_counter() - t0
    tok = sum(it["L"] for it in cpu_items)
    return {"value": tok / dt, "unit": "layer-tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_sample} of {len(items)} items of {wl.name} (L={cpu_items[0]['L']}), {dt:.1f} s, "
                      "NumPy fp64 oracle end to end"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--items", type=int, default=0, help="use only the first N items (debug)")
    ap.add_argument("--cpu-sample", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--traffic-kib", type=float, nargs=2, default=None, metavar=("FETCH", "WRITE"),
                    help="HBM KiB per launch of the dominant kernel from rocprofv3 --pmc runs, already scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(items are independent: more GPUs would each take a share of the items, with no communication)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2509_03136_amd as g
    from synth import workloads as W
    import parity_util as U

    g.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    wl = W.config(args.config)
    if args.items:
        wl = W.scaled(wl, lengths=wl.lengths[:args.items], n_planted=wl.n_planted[:args.items])
    t_gen = time.perf_counter()
    items = W.make_items(wl, dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    b = U.batch_from(g, wl, items)
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof, want_stats=False)
    stages = [("fit", pipe.fit), ("sample", pipe.sample), ("select", pipe.select), ("compact", pipe.compact)]

    for _ in range(args.warmup):
        pipe.run()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev[k][0].record()
        for j, (_, fn) in enumerate(stages):
            fn()
            ev[k][j + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    stage_ms = {name: sum(ev[k][j].elapsed_time(ev[k][j + 1]) for k in range(args.steps)) / args.steps
                for j, (name, _) in enumerate(stages)}

    pipe.select()
    torch.cuda.synchronize()
    fallback_rows = pipe.fallback_rows() if wl.dtype == "bf16" else None
    tok = sum(wl.lengths)
    budget = pipe.budget.cpu().numpy()
    kept = int(pipe.offsets[-1].item())
    rho = kept / float(tok * wl.n_kv_heads)
    ab = algorithmic_bytes(wl, wl.lengths, rho)
    dom = max(stage_ms, key=stage_ms.get)
    dom_kernel = {"fit": "moments_partial_kernel", "sample": "project_mfma_kernel",
                  "select": "score_hist_kernel", "compact": "gather_kernel"}[dom]
    if args.traffic_kib is not None:
        traffic = (args.traffic_kib[0] + args.traffic_kib[1]) * 1024.0
    else:
        traffic = profiled_traffic(wl.name, dom_kernel)
    ach = ab[dom] / (stage_ms[dom] * 1e-3) / 1e9
    out = {
        "metric": "KV tokens selected+compacted/sec (all layers, 32k ctx); achieved HBM GB/s vs peak",
        "value": tok / (ms_per_step * 1e-3),
        "unit": "layer-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "items": wl.n_items, "L": max(wl.lengths), "S": wl.S, "p": wl.p,
                   "d_model": wl.d, "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads, "head_dim": wl.d_k},
        "roofline": {"bound": "hbm", "kernel": dom_kernel, "stage": dom, "achieved": ach, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes": ab[dom], "ms": stage_ms[dom]},
        "end_to_end": {"algorithmic_GB": ab["total"] / 1e9,
                       "achieved_GBs": ab["total"] / (ms_per_step * 1e-3) / 1e9,
                       "frac_of_hbm_peak": ab["total"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "stage_ms": stage_ms,
        "stage_algorithmic_GBs": {k: ab[k] / (stage_ms[k] * 1e-3) / 1e9 for k in stage_ms},
        "kept_fraction": rho,
        "select_fallback_rows": fallback_rows,
        "budget_per_item": [int(x) for x in budget.sum(axis=1)],
        "compressed_bytes": kept * wl.d_k * wl.elem_bytes * 2,
        "input_generation_s": t_gen,
    }
    if args.copy_probe:
        a = torch.empty(1 << 30, device=dev, dtype=torch.uint8)
        bb = torch.empty_like(a)
        a.fill_(1)
        torch.cuda.synchronize()
        bb.copy_(a)
        torch.cuda.synchronize()
        del a, bb
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, items, min(args.cpu_sample, wl.n_items))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
