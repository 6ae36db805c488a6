#!/usr/bin/env python3
"""Benchmark of the GVote selection hot path on one MI355X.

A step = one pass of the whole path (fit -> sample/project/RoPE -> score/select -> union/compact)
over one batch of synthetic input that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--beta B] [--S n] [--p x]
                  [--sweep S|p] [--graph] [--no-cpu-baseline] [--copy-probe]

metric: layer-tokens per second = (sum over items of context length L) / step time.
roofline: the stage that dominates the step, priced on ALGORITHMIC bytes against 8 TB/s HBM.
end_to_end: all four stages, algorithmic bytes / step time, against the 8 TB/s peak and against a
            device-to-device copy measured in the same run (the achievable ceiling of this machine).
cpu_baseline: the CPU oracle, untuned, on a bounded sample of the same workload: all cores and one
            thread, per stage.
--sweep S / --sweep p: the cost trends of the paper's Sec. 4.4 (time grows with the number of
            samples S, is flat in p_nuc) on the chosen workload; the table goes into the JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
DOMINANT_KERNEL = {"fit": "moments_partial_kernel", "sample": "project_mfma_kernel",
                   "select": "score_hist_kernel", "compact": "gather_kernel"}
# fp32 storage takes the general kernels (no matrix-core path)
DOMINANT_KERNEL_F32 = dict(DOMINANT_KERNEL, sample="project_generic_kernel", select="select_row_kernel")


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
    (FETCH_SIZE and WRITE_SIZE runs, scaled by a plain copy of known size), or None when there is no
    such summary or it was taken from other kernel sources than the ones in this tree."""
    from paper_2509_03136_amd.build import sources_digest
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic_pmc.txt")
    if not os.path.exists(path):
        return None
    lines = open(path).read().splitlines()
    stamp = [l.split(":", 1)[1].strip() for l in lines if l.startswith("kernel sources sha256:")]
    if not stamp or stamp[0] != sources_digest():
        return None
    for line in lines:
        if line.startswith(kernel):
            cols = line[38:].split()
            try:
                return (float(cols[-2]) + float(cols[-1])) * 1e6     # the last two columns: MB read, MB written
            except (IndexError, ValueError):
                return None
    return None


def cpu_baseline(wl, items, n_sample):
    """The oracle as it stands, stage by stage, on the first items of the workload: with the BLAS pool
    at all host cores (n_sample items) and limited to one thread (one item)."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import oracle as O
    from parity_util import f32np, p32
    from threadpoolctl import threadpool_info, threadpool_limits

    def run_item(it, acc):
        hidden, w_q, k, v = f32np(it["hidden"]), f32np(it["w_q"]), f32np(it["k"]), f32np(it["v"])
        L = hidden.shape[0]
        t = [time.perf_counter()]
        mu, var = O.fit_gaussian(hidden, wl.n_skip, wl.ddof)
        t.append(time.perf_counter())
        z = O.standard_normals(it["seed"], it["stream_id"], wl.S, wl.d)
        h = O.sample_hidden(mu, var, z, wl.dtype)
        c, s = O.rope_cos_sin(float(np.float32(wl.theta)), wl.d_k, L, 1)
        q = O.project_rope(h, w_q, None, c, s, wl.n_q_heads, wl.d_k, wl.dtype)
        t.append(time.perf_counter())
        lg = O.scores(q, k)
        rm = O.select_rows(lg, p32(wl.p))
        t.append(time.perf_counter())
        un, _ = O.union_vote(rm, wl.n_kv_heads)
        O.compact(k, v, un)
        t.append(time.perf_counter())
        for name, a, b in zip(("fit", "sample", "select", "compact"), t[:-1], t[1:]):
            acc[name] = acc.get(name, 0.0) + (b - a)

    cpu_items = [{k: (v.cpu() if hasattr(v, "cpu") else v) for k, v in it.items()} for it in items[:n_sample]]
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    all_s, one_s = {}, {}
    for it in cpu_items:
        run_item(it, all_s)
    with threadpool_limits(limits=1):
        run_item(cpu_items[0], one_s)
    tok_all, tok_one = sum(it["L"] for it in cpu_items), cpu_items[0]["L"]
    dt_all, dt_one = sum(all_s.values()), sum(one_s.values())
    return {"value": tok_all / dt_all, "unit": "layer-tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_sample} of {len(items)} items of {wl.name} (L={cpu_items[0]['L']}), {dt_all:.1f} s at {cores} threads; "
                      f"1 item, {dt_one:.1f} s at 1 thread; NumPy fp64 oracle end to end",
            "nproc": os.cpu_count(), "cpu_model": model,
            "stage_s_per_item": {k: v / n_sample for k, v in all_s.items()},
            "one_thread": {"value": tok_one / dt_one, "cores": 1, "stage_s_per_item": one_s}}


def copy_ceiling(torch, dev, n_bytes=1 << 30, reps=5):
    """GB/s (read + write) of a plain device-to-device copy: what this machine's HBM delivers to a
    kernel that does nothing else."""
    a = torch.empty(n_bytes, device=dev, dtype=torch.uint8)
    b = torch.empty_like(a)
    a.fill_(1)
    b.copy_(a)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del a, b
    return 2.0 * n_bytes / (ms * 1e-3) / 1e9


def time_steps(torch, pipe, steps, warmup):
    stages = [("fit", pipe.fit), ("sample", pipe.sample), ("select", pipe.select), ("compact", pipe.compact)]
    for _ in range(warmup):
        pipe.run()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        ev[k][0].record()
        for j, (_, fn) in enumerate(stages):
            fn()
            ev[k][j + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stage_ms = {name: sum(ev[k][j].elapsed_time(ev[k][j + 1]) for k in range(steps)) / steps
                for j, (name, _) in enumerate(stages)}
    return dt * 1e3 / steps, stage_ms


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--items", type=int, default=0, help="use only the first N items")
    ap.add_argument("--length", type=int, default=0, help="override the context length of every item")
    ap.add_argument("--beta", type=float, default=None,
                    help="strength of the rank-one mean-reading term the input recipe adds to W_q (the "
                         "recipe's default is 1; 0 is the literal N(0, 1/d) recipe: diffuse attention)")
    ap.add_argument("--S", type=int, default=0, help="override the number of synthetic queries")
    ap.add_argument("--p", type=float, default=0.0, help="override the mass threshold")
    ap.add_argument("--sweep", choices=["S", "p"], default=None, help="Sec. 4.4 cost trends: vary S or p")
    ap.add_argument("--consumer", action="store_true",
                    help="also time one decode-attention step over the compressed cache (Sec. 3.4's consumer)")
    ap.add_argument("--alg1", action="store_true",
                    help="also time Algorithm 1 as printed: top-p of one real query per head -> B_step -> row-wise "
                         "TopK of the synthetic rows -> union / compaction (the first synthetic sample stands in "
                         "for the real current query)")
    ap.add_argument("--kv-head-major", action="store_true",
                    help="hold K and V as [H_kv, L, d_k] (a head's keys contiguous) instead of [L, H_kv, d_k]; the ABI takes "
                         "either through its token and head strides")
    ap.add_argument("--graph", action="store_true",
                    help="also record the four stage calls into a HIP graph and time its replays (the calls only enqueue kernels)")
    ap.add_argument("--cpu-sample", type=int, default=8, help="items the CPU oracle is timed on (about 1.3 s each at config 3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="(kept for profiling runs) the copy ceiling is always measured; this flag is accepted and ignored")
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

    g.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    wl = W.config(args.config)
    if args.items:
        wl = W.scaled(wl, lengths=wl.lengths[:args.items], n_planted=wl.n_planted[:args.items])
    if args.length:
        wl = W.scaled(wl, lengths=(args.length,) * wl.n_items)
    over = {}
    if args.beta is not None:
        over["beta"] = args.beta
    if args.S:
        over["S"] = args.S
    if args.p:
        over["p"] = args.p
    if over:
        wl = W.scaled(wl, **over)
    t_gen = time.perf_counter()
    items = W.make_items(wl, dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    if args.kv_head_major:
        for it in items:
            for name in ("k", "v"):
                it[name] = it[name].permute(1, 0, 2).contiguous().permute(1, 0, 2)      # same values, head-major memory
    b = g.Batch.from_workload(wl, items)
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof, want_stats=False)

    ms_per_step, stage_ms = time_steps(torch, pipe, args.steps, args.warmup)

    pipe.select()
    torch.cuda.synchronize()
    fallback_rows = pipe.fallback_rows() if wl.dtype == "bf16" else None
    fallback_why = pipe.fallback_reasons() if wl.dtype == "bf16" else None
    refined_rows = pipe.refined_rows() if wl.dtype == "bf16" else None
    tok = sum(wl.lengths)
    budget = pipe.budget.cpu().numpy()
    kept = int(pipe.offsets[-1].item())
    rho = kept / float(tok * wl.n_kv_heads)
    ab = algorithmic_bytes(wl, wl.lengths, rho)
    dom = max(stage_ms, key=stage_ms.get)
    dom_kernel = (DOMINANT_KERNEL if wl.dtype == "bf16" else DOMINANT_KERNEL_F32)[dom]
    if args.traffic_kib is not None:
        traffic = (args.traffic_kib[0] + args.traffic_kib[1]) * 1024.0
    else:
        traffic = profiled_traffic(wl.name, dom_kernel) if not over and not args.items and not args.length else None
    step_traffic = profiled_traffic(wl.name, "whole step") if traffic is not None and args.traffic_kib is None else None
    ach = ab[dom] / (stage_ms[dom] * 1e-3) / 1e9
    copy_gbs = copy_ceiling(torch, dev)
    e2e_gbs = ab["total"] / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "KV tokens selected+compacted/sec (all layers, 32k ctx); achieved HBM GB/s vs peak",
        "value": tok / (ms_per_step * 1e-3),
        "unit": "layer-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "items": wl.n_items, "L": max(wl.lengths), "S": wl.S, "p": wl.p,
                   "d_model": wl.d, "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads, "head_dim": wl.d_k,
                   "beta": wl.beta},
        "roofline": {"bound": "hbm", "kernel": dom_kernel, "stage": dom, "achieved": ach, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes": ab[dom], "ms": stage_ms[dom]},
        "end_to_end": {"algorithmic_GB": ab["total"] / 1e9, "achieved_GBs": e2e_gbs,
                       "frac_of_hbm_peak": e2e_gbs / HBM_PEAK_GBS,
                       "copy_ceiling_GBs": copy_gbs, "frac_of_copy_ceiling": e2e_gbs / copy_gbs,
                       # HBM bytes of a whole step from the committed counter runs, and the rate they mean at this step time
                       "traffic": step_traffic,
                       "traffic_GBs": None if step_traffic is None else step_traffic / (ms_per_step * 1e-3) / 1e9},
        "head_tokens_per_s": tok * wl.n_kv_heads / (ms_per_step * 1e-3),
        "stage_ms": stage_ms,
        "stage_algorithmic_GBs": {k: ab[k] / (stage_ms[k] * 1e-3) / 1e9 for k in stage_ms},
        "stage_frac_of_hbm_peak": {k: ab[k] / (stage_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBS for k in stage_ms},
        "kept_fraction": rho,
        "select_fallback_rows": fallback_rows,
        "select_fallback_by_reason": fallback_why,
        "select_rows_in_second_window": refined_rows,
        "budget_per_item": [int(x) for x in budget.sum(axis=1)],
        "compressed_bytes": kept * wl.d_k * wl.elem_bytes * 2,
        "input_generation_s": t_gen,
    }
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            pipe.run()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            pipe.run()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        out["graph_replay_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / args.steps
    if args.consumer:
        qd = torch.randn(wl.n_items, wl.n_q_heads, wl.d_k, device=dev, dtype=torch.float32).to(pipe.q.dtype)
        od = torch.empty_like(qd)
        lse = torch.empty(wl.n_items, wl.n_q_heads, device=dev, dtype=torch.float32)
        for _ in range(3):
            g.decode_attention(b, qd, pipe.k_out, pipe.v_out, pipe.offsets, od, pipe.ws, lse)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record()
        for _ in range(reps):
            g.decode_attention(b, qd, pipe.k_out, pipe.v_out, pipe.offsets, od, pipe.ws, lse)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        cache_bytes = kept * wl.d_k * wl.elem_bytes * 2
        out["consumer"] = {"decode_attention_ms": ms, "compressed_cache_bytes": cache_bytes,
                           "achieved_GBs": cache_bytes / (ms * 1e-3) / 1e9,
                           "frac_of_hbm_peak": cache_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "full_cache_bytes": tok * wl.n_kv_heads * wl.d_k * wl.elem_bytes * 2}
    if args.alg1:
        n, S, hq = wl.n_items, wl.S, wl.n_q_heads
        q0 = pipe.q[:, :1].contiguous()
        mask0 = torch.empty(sum(hq * b.words(i) for i in range(n)), device=dev, dtype=torch.int32)
        counts = torch.empty(n, S, hq, device=dev, dtype=torch.int32)

        def alg1_select():
            g.score_select(b, 1, q0, wl.p, mask0, ws=pipe.ws)
            g.count_rows(b, 1, mask0, S, counts)
            g.score_select(b, S, pipe.q, wl.p, pipe.rowmask, mode=g.SELECT_TOPK, k_per_row=counts, ws=pipe.ws)

        for _ in range(2):
            alg1_select()
            pipe.compact()
        torch.cuda.synchronize()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        reps = max(3, args.steps // 2)
        t_sel = t_cmp = 0.0
        for _ in range(reps):
            e[0].record(); alg1_select(); e[1].record(); pipe.compact(); e[2].record()
            torch.cuda.synchronize()
            t_sel += e[0].elapsed_time(e[1]); t_cmp += e[1].elapsed_time(e[2])
        g.score_select(b, S, pipe.q, wl.p, pipe.rowmask, mode=g.SELECT_TOPK, k_per_row=counts, ws=pipe.ws)
        torch.cuda.synchronize()
        out["alg1"] = {"select_ms": t_sel / reps, "compact_ms": t_cmp / reps,
                       "ms_per_step": stage_ms["fit"] + stage_ms["sample"] + (t_sel + t_cmp) / reps,
                       "topk_fallback_rows": pipe.fallback_rows(),
                       "kept_fraction": int(pipe.offsets[-1].item()) / float(tok * wl.n_kv_heads),
                       "mean_B_step": float(counts.float().mean().item())}
    if args.sweep:
        values = {"S": [4, 8, 16, 32, 64], "p": [0.5, 0.8, 0.9, 0.95, 0.99, 0.999, 0.9999]}[args.sweep]
        rows = []
        for x in values:
            S, p = (x, wl.p) if args.sweep == "S" else (wl.S, x)
            pp = g.Pipeline(b, S, p, ddof=wl.ddof, want_stats=False)
            ms, st = time_steps(torch, pp, max(3, args.steps // 2), 2)
            pp.select()
            torch.cuda.synchronize()
            fb = pp.fallback_rows()
            rows.append({args.sweep: x, "ms_per_step": ms, "stage_ms": st, "select_fallback_rows": fb,
                         "select_rows_in_second_window": pp.refined_rows(),
                         "kept_fraction": int(pp.offsets[-1].item()) / float(tok * wl.n_kv_heads)})
            del pp
            torch.cuda.empty_cache()
        out["sweep"] = {"over": args.sweep, "rows": rows}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, items, min(args.cpu_sample, wl.n_items))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
