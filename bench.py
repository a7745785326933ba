#!/usr/bin/env python3
"""Benchmark of the CurDKV selection path on one MI355X.

A step is one pass of the whole hot path -- scores, selection and gather, through
the one-call entry point curdkv_compress -- over a synthetic Llama-3-8B-shaped
cache (32 layers x 8 KV heads x 32768 tokens x d=128, bf16, r=64) that is already
resident in HBM.  The same work as three separate calls (curdkv_scores,
curdkv_select, curdkv_compact back to back on one stream) is timed as well and
reported under "three_calls".  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3] [--keep 0.10]
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, vendor figure
# what plain streaming kernels reach on this chip (measured once with hand-written read and copy
# kernels over 4 GiB; not re-measured here): context for the fraction of the vendor peak
READ_CEILING_GBS = 6150.0
COPY_CEILING_GBS = 5600.0


def algorithmic_bytes(cfg, budgets, esize=2, source="kv"):
    """Bytes the method has to move (per step and per part).  Per head: read K and
    V once (2*n*d*e; one of them only for the key-only / value-only ablation),
    write the scores (4n); select reads them (4n) and writes indices (4k); compact
    reads indices (4k), reads and writes k rows of K and V."""
    heads, n, d = cfg.layers * cfg.kv_heads, cfg.n, cfg.d
    ksum = int(np.sum(budgets.astype(np.int64)))
    row = d * esize
    scan = heads * n * ((2 if source == "kv" else 1) * row)
    scores_call = scan + heads * n * 4
    select_call = heads * n * 4 + ksum * 4
    compact_call = ksum * (4 + 4 * row)
    return dict(scan=scan, scores=scores_call, select=select_call, compact=compact_call,
                total=scores_call + select_call + compact_call)


def measured_traffic(cfg_name, keep, fused):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc
    (FETCH_SIZE and WRITE_SIZE, scaled by a copy of known size), read from the
    committed profile summary; None when no summary covers this workload."""
    import glob
    import re
    kern = "fused_kernel" if fused else "curdkv_compress"
    pat = re.compile(r"traffic_bytes_per_launch\s+%s\s+%s\s+keep=%g:\s*(\d+)" % (kern, cfg_name, keep))
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        m = pat.search(open(f).read())
        if m:
            return int(m.group(1))
    return None


def cpu_baseline(cfg, Kd, Vd, budgets, n_sink, max_seconds=25.0, source="kv", projection=True):
    """The CPU oracle, as it stands, on the same workload: groups in (layer, head)
    order, for as many as fit in the time budget (copies from the GPU not timed)."""
    import torch
    from oracle import curdkv_oracle as orc

    def to_host(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    H, n = cfg.kv_heads, cfg.n
    done, t_used = 0, 0.0
    for i in range(cfg.layers * H):
        l, h = divmod(i, H)
        K, V = to_host(Kd[l, h]), to_host(Vd[l, h])
        t0 = time.perf_counter()
        G = orc.sketch(cfg.sketch_seed, l, h, H, cfg.d, cfg.r, cfg.dtype) if projection else None
        orc.compress_group(K, V, cfg.dtype, G, int(budgets[l * H + h]), n_sink, source, projection)
        t_used += time.perf_counter() - t0
        done += 1
        if t_used > max_seconds:
            break
    return {"value": done * n / t_used, "unit": "KV tokens/s", "cores": int(threads),
            "kind": "oracle",
            "sample": f"the first {done} of {cfg.layers * H} (layer, head) groups of {n} tokens, "
                      f"{t_used:.1f} s of float64 numpy, single process"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="c3", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--keep", type=float, default=None, help="keep fraction (default: the config's first)")
    ap.add_argument("--source", default="kv", choices=["kv", "k", "v"],
                    help="ablation: score from keys and values (the method), keys only, values only")
    ap.add_argument("--no-projection", action="store_true", help="ablation: no Gaussian projection")
    ap.add_argument("--adaptive", type=float, default=None, metavar="ALPHA",
                    help="AdaCurDKV: also time scores -> head-wise budgets (safeguard ALPHA) -> "
                         "select -> compact and report it under 'adaptive'")
    ap.add_argument("--append", type=int, nargs="*", default=None, metavar="M",
                    help="scoring during generation: also time curdkv_scores_append of the last M "
                         "tokens of the cache (several M allowed) and curdkv_normalise")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (torch) three times, so that a counter "
                         "profile of this command holds a kernel of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (every (layer, head) is independent; "
              "there is nothing to exchange).  Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_15038_amd import binding as B, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    B.lib()
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.config]
    keep = cfg.keep[0] if args.keep is None else args.keep
    budgets = wl.budgets_for(cfg, keep)
    offsets = wl.offsets_for(budgets)
    total = int(offsets[-1])
    L, H, n, d = cfg.layers, cfg.kv_heads, cfg.n, cfg.d
    heads = L * H

    Kd, Vd = wl.device_cache(cfg)
    scores = torch.empty((heads, n), dtype=torch.float32, device="cuda")
    indices = torch.empty((max(total, 1),), dtype=torch.int32, device="cuda")
    Ko = torch.empty((max(total, 1), d), dtype=torch.bfloat16, device="cuda")
    Vo = torch.empty((max(total, 1), d), dtype=torch.bfloat16, device="cuda")
    ctx = B.Context(L, H, cfg.group, d, cfg.r, cfg.dtype, n, cfg.sketch_seed, args.source,
                    not args.no_projection)
    s = cfg.n_sink
    fused = ctx.uses_fused_kernel(n) and total * 4 <= heads * n

    def step_calls(ev=None):
        if ev:
            ev[0].record()
        ctx.scores(Kd, Vd, n, scores)
        if ev:
            ev[1].record()
        ctx.select(scores, n, budgets, s, offsets, indices)
        if ev:
            ev[2].record()
        ctx.compact(Kd, Vd, n, indices, offsets, Ko, Vo)
        if ev:
            ev[3].record()

    def step_one_call(ev=None):
        if ev:
            ev[0].record()
        ctx.compress(Kd, Vd, n, budgets, s, offsets, scores, indices, Ko, Vo)
        if ev:
            ev[3].record()

    def timed(step):
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(evs[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / args.steps, evs

    ab = algorithmic_bytes(cfg, budgets, source=args.source)
    kv_tokens = heads * n
    if args.copy_calibration:
        src = torch.ones((1 << 29,), dtype=torch.bfloat16, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # the three separate calls, with HIP events between them
    ms_calls, evs = timed(step_calls)
    part = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in evs]).mean(0)
    calls = {"ms_per_step": ms_calls, "KV_tokens_per_s": kv_tokens / (ms_calls * 1e-3),
             "path_GBps": ab["total"] / (ms_calls * 1e-3) / 1e9,
             "frac_of_hbm_peak": ab["total"] / (ms_calls * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "ms": {"scores": float(part[0]), "select": float(part[1]), "compact": float(part[2])},
             "GBps": {"scores": ab["scores"] / (part[0] * 1e-3) / 1e9,
                      "select": ab["select"] / (part[1] * 1e-3) / 1e9,
                      "compact": ab["compact"] / (part[2] * 1e-3) / 1e9}}

    # the one-call entry point (one fused kernel at this shape): the headline
    ms_per_step, evs = timed(step_one_call)
    kern_ms = float(np.mean([e[0].elapsed_time(e[3]) for e in evs]))
    value = kv_tokens / (ms_per_step * 1e-3)
    kern_gbs = ab["total"] / (kern_ms * 1e-3) / 1e9
    out = {
        "metric": "KV tokens scored+compacted/sec at 8B shape, 32k ctx; % of HBM peak",
        "value": value, "unit": "KV tokens/s (one token of one layer and KV head)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {L} layers x {H} KV heads (GQA group {cfg.group}), "
                               f"n={n}, d={d}, r={cfg.r}, keep={keep:g} (k/head mean "
                               f"{total / heads:.0f}), sinks={s}, bf16, resident in HBM; "
                               f"step = curdkv_compress (scores + select + compact)"
                               + ("" if args.source == "kv" and not args.no_projection else
                                  f"; ablation: source={args.source}, projection={not args.no_projection}"),
                   "layers": L, "kv_heads": H, "n": n, "d": d, "r": cfg.r, "keep": keep},
        "context_tokens_per_s": n / (ms_per_step * 1e-3),
        "path_GBps": ab["total"] / (ms_per_step * 1e-3) / 1e9,
        "path_frac_of_hbm_peak": ab["total"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm",
                     "kernel": "fused_kernel (whole path, one workgroup per head)" if fused else
                               "curdkv_compress (scores, select and compact kernels)",
                     "achieved": kern_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": kern_gbs / HBM_PEAK_GBS,
                     "traffic": measured_traffic(cfg.name, keep, fused)
                     if args.source == "kv" and not args.no_projection else None,
                     "algorithmic_bytes_per_launch": ab["total"], "avg_ms": kern_ms,
                     "measured_stream_ceilings_GBps": {"read_only": READ_CEILING_GBS, "copy": COPY_CEILING_GBS},
                     # time the same bytes would take at those ceilings: scan bytes at the read
                     # ceiling, everything else (scores, indices, gathered rows) at the copy ceiling
                     "frac_of_stream_ceiling": (ab["scan"] / READ_CEILING_GBS + (ab["total"] - ab["scan"]) / COPY_CEILING_GBS)
                                               / 1e9 / (kern_ms * 1e-3)},
        "three_calls": calls,
    }

    if args.adaptive is not None:
        kbase = int(np.sum(budgets) // heads)                   # the per-head budget the layers share out
        bd = torch.empty((heads,), dtype=torch.int32, device="cuda")
        ia = torch.empty((heads * kbase,), dtype=torch.int32, device="cuda")   # every layer keeps H*kbase rows
        Ka = torch.empty((heads * kbase, d), dtype=Ko.dtype, device="cuda"); Va = torch.empty_like(Ka)
        bh = torch.empty((heads,), dtype=torch.int32, pin_memory=True)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        parts = []
        for it in range(args.warmup + args.steps):
            ev[0].record()
            ctx.scores(Kd, Vd, n, scores)
            ev[1].record()
            ctx.adaptive_budgets(scores, n, kbase, s, args.adaptive, bd)
            bh.copy_(bd, non_blocking=True)
            ev[2].record()
            torch.cuda.current_stream().synchronize()          # budgets are needed on the host
            ab_ = bh.numpy().copy()
            ao = wl.offsets_for(ab_)
            ctx.select(scores, n, ab_, s, ao, ia)
            ev[3].record()
            ctx.compact(Kd, Vd, n, ia, ao, Ka, Va)
            ev[4].record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                parts.append([ev[j].elapsed_time(ev[j + 1]) for j in range(4)])
        pm = np.array(parts).mean(0)
        # the same in one call, budgets and offsets staying on the device
        od = torch.empty((heads + 1,), dtype=torch.int64, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        one = []
        for it in range(args.warmup + args.steps):
            e0.record()
            ctx.compress_adaptive(Kd, Vd, n, kbase, s, args.adaptive, scores, bd, od, ia, Ka, Va)
            e1.record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                one.append(e0.elapsed_time(e1))
        assert bd.cpu().numpy().tolist() == ab_.tolist()
        out["adaptive"] = {"alpha": args.adaptive, "base_budget": kbase,
                           "ms": {"scores": float(pm[0]), "budgets_incl_copy": float(pm[1]),
                                  "select_incl_host_gap": float(pm[2]), "compact": float(pm[3]),
                                  "total": float(pm.sum())},
                           "one_call_ms": float(np.mean(one)),
                           "one_call_frac_of_hbm_peak": ab["total"] / (float(np.mean(one)) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "budget_min_max": [int(ab_.min()), int(ab_.max())]}
    if args.append:
        raw = torch.empty((heads, n), dtype=torch.float32, device="cuda")
        sums = torch.zeros((heads,), dtype=torch.float64, device="cuda")
        K4, V4 = Kd.view(L, H, n, d), Vd.view(L, H, n, d)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        res = {}
        for m in args.append:
            Kc, Vc = K4[:, :, n - m:].contiguous(), V4[:, :, n - m:].contiguous()
            ts = []
            for it in range(args.warmup + args.steps):
                e0.record()
                ctx.scores_append(Kc, Vc, m, n - m, n, raw, sums)
                e1.record()
                torch.cuda.synchronize()
                if it >= args.warmup:
                    ts.append(e0.elapsed_time(e1))
            bytes_m = heads * m * ((2 if args.source == "kv" else 1) * d * 2 + 4)
            res[str(m)] = {"ms": float(np.mean(ts)), "GBps": bytes_m / (np.mean(ts) * 1e-3) / 1e9}
        ts = []
        for it in range(args.warmup + args.steps):
            e0.record()
            ctx.normalise(raw, sums, n, n, scores)
            e1.record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                ts.append(e0.elapsed_time(e1))
        out["incremental"] = {"scores_append": res, "normalise_ms": float(np.mean(ts))}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, Kd.view(L, H, n, d), Vd.view(L, H, n, d), budgets, s,
                                           source=args.source, projection=not args.no_projection)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
