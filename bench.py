#!/usr/bin/env python3
"""Benchmark of the CurDKV selection path on one MI355X.

A step is one pass of the whole hot path -- scores, selection and gather, through
the one-call entry point curdkv_compress -- over a synthetic Llama-3-8B-shaped
cache (32 layers x 8 KV heads x 32768 tokens x d=128, bf16, r=64, keep 10 %) that
is already resident in HBM.  The same work as three separate calls (curdkv_scores,
curdkv_select, curdkv_compact back to back on one stream) is timed as well and
reported under "three_calls".  The default run then times the rest of the headline
configuration on the same cache (keep 20 % and 50 %), the Mistral-shaped cache with
its high-norm prefix (C4), and two plain streams through the library's own kernels
(a key-only scan without projection, a gather with identity indices) that say what
this chip's memory system gives a pure read and a pure copy.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3] [--keep 0.10]
"""

from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, vendor figure
FP32_MFMA_PEAK_TFLOPS = 157.3     # MI355X, dense fp32 matrix rate
FUSED_GATHER_MAX_PERCENT = 11     # curdkv_compress: above this share of rows kept, the fused kernel only scores


def algorithmic_bytes(cfg, budgets, source="kv"):
    """Bytes the method has to move (per step and per part).  Per head: read K and
    V once (2*n*d*e; one of them only for the key-only / value-only ablation),
    write the scores (4n); select reads them (4n) and writes indices (4k); compact
    reads indices (4k), reads and writes k rows of K and V."""
    heads, n, d = cfg.layers * cfg.kv_heads, cfg.n, cfg.d
    ksum = int(np.sum(budgets.astype(np.int64)))
    row = d * (2 if cfg.dtype == "bf16" else 4)
    scan = heads * n * ((2 if source == "kv" else 1) * row)
    scores_call = scan + heads * n * 4
    select_call = heads * n * 4 + ksum * 4
    compact_call = ksum * (4 + 4 * row)
    return dict(scan=scan, scores=scores_call, select=select_call, compact=compact_call,
                total=scores_call + select_call + compact_call)


def kernel_sources_sha16():
    """Fingerprint of the HIP sources the library is built from; a profile summary records
    the one it was measured with, so that a figure taken from it is not quoted for other code."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2509_15038_amd", "csrc")
    for f in sorted(os.listdir(src)):
        h.update(f.encode())
        h.update(open(os.path.join(src, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(cfg_name, keep, fused, heads):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc
    (FETCH_SIZE and WRITE_SIZE, scaled by a copy of known size).  Counters cannot be read
    from inside this run: the figure comes from the committed profile summary that covers
    this workload, and only if that summary was made from the kernel sources this run uses;
    otherwise None.  Returns (bytes or None, where it came from)."""
    kern = "fused_kernel" if fused else "curdkv_compress"
    pat = re.compile(r"traffic_bytes_per_launch\s+%s\s+%s\s+heads=%d\s+keep=%g:\s*(\d+)" % (kern, cfg_name, heads, keep))
    sha = kernel_sources_sha16()
    stale = None
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        text = open(f).read()
        m = pat.search(text)
        if not m:
            continue
        rec = re.search(r"kernel_sources_sha16:\s*([0-9a-f]{16})", text)
        if rec and rec.group(1) == sha:
            return int(m.group(1)), {"file": os.path.relpath(f, ROOT), "kernel_sources_sha16": sha}
        stale = {"file": os.path.relpath(f, ROOT), "stale": True,
                 "note": "the summary was measured with other kernel sources; figure withheld"}
    return None, stale


def cpu_baseline(cfg, Kd, Vd, budgets, n_sink, max_seconds=20.0, single_seconds=8.0, source="kv", projection=True):
    """The CPU oracle, as it stands, on the same workload, copies from the GPU not timed.
    Two flavours: the numpy/BLAS thread pool as the box gives it, on the groups in (layer,
    head) order for as many as fit in the time budget; and one BLAS thread, on one group per
    layer (head = layer mod H) for as many layers as fit in its budget."""
    import torch
    from oracle import curdkv_oracle as orc

    def to_host(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16)

    def one_group(l, h):
        K, V = to_host(Kd[l, h]), to_host(Vd[l, h])
        t0 = time.perf_counter()
        G = orc.sketch(cfg.sketch_seed, l, h, H, cfg.d, cfg.r, cfg.dtype) if projection else None
        orc.compress_group(K, V, cfg.dtype, G, int(budgets[l * H + h]), n_sink, source, projection)
        return time.perf_counter() - t0

    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        threads = os.cpu_count() or 1
    H, n = cfg.kv_heads, cfg.n
    done, t_used = 0, 0.0
    for i in range(cfg.layers * H):
        t_used += one_group(*divmod(i, H))
        done += 1
        if t_used > max_seconds:
            break
    out = {"value": done * n / t_used, "unit": "KV tokens/s", "cores": int(threads), "kind": "oracle",
           "sample": f"the first {done} of {cfg.layers * H} (layer, head) groups of {n} tokens, "
                     f"{t_used:.1f} s of float64 numpy, single process, {threads} BLAS threads",
           "host_cpu_count": os.cpu_count()}
    if threadpool_limits is not None:
        done1, t1 = 0, 0.0
        with threadpool_limits(limits=1):
            for l in range(cfg.layers):
                t1 += one_group(l, l % H)
                done1 += 1
                if t1 > single_seconds:
                    break
        out["single_thread"] = {"value": done1 * n / t1, "unit": "KV tokens/s", "cores": 1,
                                "sample": f"group (l, l mod {H}) of the first {done1} layers, {t1:.1f} s, "
                                          f"one BLAS thread"}
    return out


class Timer:
    """HIP events on torch's current stream (the stream the binding launches on)."""

    def __init__(self, steps, warmup):
        self.steps, self.warmup = steps, warmup

    def run(self, step, marks=2):
        import torch
        # (the events are made before the warm-up so that the GPU does not sit idle, and clock
        # down, between the warm-up and the timed steps)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(marks)] for _ in range(self.steps)]
        for _ in range(self.warmup):
            step(None)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(self.steps):
            step(evs[i])
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / self.steps
        seg = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(marks - 1)] for e in evs])
        return wall_ms, seg


def time_compress(ctx, timer, Kd, Vd, cfg, budgets, bufs, source="kv"):
    """One workload through the one-call entry point and through the three calls."""
    scores, indices, Ko, Vo = bufs
    n, s = cfg.n, cfg.n_sink
    heads = cfg.layers * cfg.kv_heads
    from paper_2509_15038_amd import workloads as wl
    offsets = wl.offsets_for(budgets)
    ab = algorithmic_bytes(cfg, budgets, source=source)

    def step_calls(ev):
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

    def step_one(ev):
        if ev:
            ev[0].record()
        ctx.compress(Kd, Vd, n, budgets, s, offsets, scores, indices, Ko, Vo)
        if ev:
            ev[1].record()

    wall_calls, seg = timer.run(step_calls, marks=4)
    part = seg.mean(0)
    calls = {"ms_per_step": wall_calls, "ms_median_events": float(np.median(seg.sum(1))),
             "KV_tokens_per_s": heads * n / (wall_calls * 1e-3),
             "path_GBps": ab["total"] / (wall_calls * 1e-3) / 1e9,
             "frac_of_hbm_peak": ab["total"] / (wall_calls * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "ms": {"scores": float(part[0]), "select": float(part[1]), "compact": float(part[2])},
             "GBps": {"scores": ab["scores"] / (part[0] * 1e-3) / 1e9,
                      "select": ab["select"] / (part[1] * 1e-3) / 1e9,
                      "compact": ab["compact"] / (part[2] * 1e-3) / 1e9}}
    wall_one, seg = timer.run(step_one, marks=2)
    one = {"ms_per_step": wall_one, "ms_mean_events": float(seg.mean()), "ms_median_events": float(np.median(seg)),
           "ms_min_events": float(seg.min()), "ms_max_events": float(seg.max())}
    return one, calls, ab


def stream_rates(timer, cfg, Kd, Vd):
    """What the memory system gives plain streams through the library's own kernels, at this
    workload's shape: curdkv_scores without projection on the keys alone (256 contiguous
    bytes per token and 4 written), the same on keys and values (512 bytes per token, the
    method's scan without its matrix work), and curdkv_compact with identity indices (every
    row read once and written once)."""
    import torch
    from paper_2509_15038_amd import binding as B, workloads as wl
    L, H, n, d = cfg.layers, cfg.kv_heads, cfg.n, cfg.d
    heads = L * H
    scores = torch.empty((heads, n), dtype=torch.float32, device="cuda")
    out = {}
    for name, source, tensors in (("read_keys_no_projection", "k", 1), ("read_keys_values_no_projection", "kv", 2)):
        with B.Context(L, H, cfg.group, d, cfg.r, cfg.dtype, n, cfg.sketch_seed, source, False) as c:
            def step(ev, c=c):
                if ev:
                    ev[0].record()
                c.scores(Kd, Vd, n, scores)
                if ev:
                    ev[1].record()
            _, seg = timer.run(step)
        ms = float(np.median(seg))
        out[name] = {"ms": ms, "GBps": heads * n * (tensors * d * 2 + 4) / (ms * 1e-3) / 1e9}
    budgets = np.full(heads, n, dtype=np.int32)
    offsets = wl.offsets_for(budgets)
    ident = torch.arange(n, dtype=torch.int32, device="cuda").repeat(heads)
    Ko = torch.empty((heads * n, d), dtype=torch.bfloat16, device="cuda")
    Vo = torch.empty_like(Ko)
    with B.Context(L, H, cfg.group, d, cfg.r, cfg.dtype, n, cfg.sketch_seed) as c:
        def step(ev, c=c):
            if ev:
                ev[0].record()
            c.compact(Kd, Vd, n, ident, offsets, Ko, Vo)
            if ev:
                ev[1].record()
        _, seg = timer.run(step)
    ms = float(np.median(seg))
    out["copy_identity_gather"] = {"ms": ms, "GBps": heads * n * (4 + 4 * d * 2) / (ms * 1e-3) / 1e9}
    return out, (Ko, Vo, ident, scores)           # kept alive by the caller: see the note on freeing in main()


def summary(one, ab):
    ms = one["ms_mean_events"]
    gbs = ab["total"] / (ms * 1e-3) / 1e9
    return {"ms": ms, "ms_median": one["ms_median_events"], "ms_per_step_wall": one["ms_per_step"],
            "GBps": gbs, "frac": gbs / HBM_PEAK_GBS, "algorithmic_bytes": ab["total"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="c3", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--keep", type=float, default=None, help="keep fraction (default: the config's first)")
    ap.add_argument("--layers", type=int, default=None,
                    help="number of layers (default: the config's 32): fewer layers are the slice of the cache "
                         "one GPU holds when the model's KV heads are spread over several")
    ap.add_argument("--tokens", type=int, default=None, help="tokens per head (default: the config's)")
    ap.add_argument("--sketch-dim", type=int, default=None, help="sketch width r (default: the config's)")
    ap.add_argument("--dtype", default=None, choices=["bf16", "fp32"],
                    help="storage type of the cache (default: the config's; fp32 doubles the cache's bytes)")
    ap.add_argument("--source", default="kv", choices=["kv", "k", "v"],
                    help="ablation: score from keys and values (the method), keys only, values only")
    ap.add_argument("--no-projection", action="store_true", help="ablation: no Gaussian projection")
    ap.add_argument("--adaptive", type=float, default=None, metavar="ALPHA",
                    help="AdaCurDKV: also time scores -> head-wise budgets (safeguard ALPHA) -> "
                         "select -> compact and report it under 'adaptive'")
    ap.add_argument("--append", type=int, nargs="*", default=None, metavar="M",
                    help="scoring during generation: also time curdkv_scores_append of the last M "
                         "tokens of the cache (several M allowed) and curdkv_normalise")
    ap.add_argument("--headline-only", action="store_true",
                    help="time the named workload only: no other budgets, no C4, no stream rates")
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
    if args.layers is not None:
        cfg = wl.scaled(cfg, layers=args.layers)
    if args.tokens is not None:
        cfg = wl.scaled(cfg, n=args.tokens)
    if args.sketch_dim is not None:
        cfg = wl.scaled(cfg, r=args.sketch_dim)
    if args.dtype is not None:
        cfg = wl.scaled(cfg, dtype=args.dtype)
    keep = cfg.keep[0] if args.keep is None else args.keep
    budgets = wl.budgets_for(cfg, keep)
    total = int(budgets.astype(np.int64).sum())
    L, H, n, d = cfg.layers, cfg.kv_heads, cfg.n, cfg.d
    heads = L * H
    plain = args.source == "kv" and not args.no_projection
    extras = (plain and not args.headline_only and args.config == "c3" and args.keep is None
              and args.layers is None and args.tokens is None and args.sketch_dim is None
              and args.dtype is None)

    Kd, Vd = wl.device_cache(cfg)
    rows_max = max(total, int(heads * n * 0.5) if extras else 0, 1)
    scores = torch.empty((heads, n), dtype=torch.float32, device="cuda")
    indices = torch.empty((rows_max,), dtype=torch.int32, device="cuda")
    Ko = torch.empty((rows_max, d), dtype=Kd.dtype, device="cuda")
    Vo = torch.empty((rows_max, d), dtype=Kd.dtype, device="cuda")
    bufs = (scores, indices, Ko, Vo)
    ctx = B.Context(L, H, cfg.group, d, cfg.r, cfg.dtype, n, cfg.sketch_seed, args.source,
                    not args.no_projection)
    s = cfg.n_sink
    fused = ctx.uses_fused_kernel(n) and total * 100 <= heads * n * FUSED_GATHER_MAX_PERCENT
    timer = Timer(args.steps, args.warmup)

    if args.copy_calibration:
        src = torch.ones((1 << 29,), dtype=torch.bfloat16, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    one, calls, ab = time_compress(ctx, timer, Kd, Vd, cfg, budgets, bufs, args.source)
    ms_per_step = one["ms_per_step"]
    kern_ms = one["ms_mean_events"]
    kv_tokens = heads * n
    value = kv_tokens / (ms_per_step * 1e-3)
    kern_gbs = ab["total"] / (kern_ms * 1e-3) / 1e9
    # (the profile summaries cover the configurations' own n, r and storage type, any head count)
    as_profiled = plain and args.tokens is None and args.sketch_dim is None and args.dtype is None
    traffic, traffic_src = measured_traffic(cfg.name, keep, fused, heads) if as_profiled else (None, None)
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
                               + ("" if plain else
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
                     "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": ab["total"], "avg_ms": kern_ms,
                     "median_ms": one["ms_median_events"], "min_ms": one["ms_min_events"],
                     "max_ms": one["ms_max_events"]},
        "three_calls": calls,
    }

    # An fp32 cache with a wide sketch is bound by the fp32 matrix rate, not by HBM: 4*d*r flop per
    # token (2*d*r for key-only / value-only) against 8*d bytes.  The scoring kernel is then the
    # dominant one and is priced against the fp32 MFMA peak; the HBM view stays beside it.
    if cfg.dtype == "fp32" and not args.no_projection:
        flops = (4 if args.source == "kv" else 2) * d * cfg.r * heads * n
        if flops / (FP32_MFMA_PEAK_TFLOPS * 1e12) > ab["total"] / (HBM_PEAK_GBS * 1e9):
            sc_ms = calls["ms"]["scores"]
            tf = flops / (sc_ms * 1e-3) / 1e12
            out["roofline"] = {"bound": "mfma", "kernel": "scores_f32_kernel (curdkv_scores: scoring kernel + normalisation)",
                               "achieved": tf, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                               "frac": tf / FP32_MFMA_PEAK_TFLOPS, "traffic": None,
                               "algorithmic_flops_per_launch": flops, "avg_ms": sc_ms,
                               "whole_path_against_hbm": out["roofline"]}

    if extras:
        # the rest of the headline configuration, driver-visible: the other two budgets on the same
        # cache, then the Mistral-shaped cache; each through curdkv_compress, HIP events around it
        more = {}
        for kp in cfg.keep[1:]:
            b = wl.budgets_for(cfg, kp)
            o, c3, a = time_compress(ctx, timer, Kd, Vd, cfg, b, bufs)
            more[f"c3 keep={kp:g}"] = dict(summary(o, a), three_calls_ms=c3["ms_per_step"],
                                           traffic=measured_traffic("c3", kp, ctx.uses_fused_kernel(n) and int(b.sum()) * 100 <= heads * n * FUSED_GATHER_MAX_PERCENT, heads)[0])
        c4 = wl.CONFIGS["c4"]
        K4, V4 = wl.device_cache(c4)
        b4 = wl.budgets_for(c4)
        with B.Context(c4.layers, c4.kv_heads, c4.group, c4.d, c4.r, c4.dtype, c4.n, c4.sketch_seed) as ctx4:
            o, c3, a = time_compress(ctx4, timer, K4, V4, c4, b4, bufs)
            more[f"c4 keep={c4.keep[0]:g}"] = dict(summary(o, a), three_calls_ms=c3["ms_per_step"],
                                                   traffic=measured_traffic("c4", c4.keep[0], ctx4.uses_fused_kernel(c4.n) and int(b4.sum()) * 100 <= heads * c4.n * FUSED_GATHER_MAX_PERCENT, heads)[0])
        # (nothing is freed between the timed sections: the driver wipes freed device memory in
        # the background, and for some hundred milliseconds after a free of several GiB every
        # kernel here runs 3 to 4 % slower)
        rates, keep_alive = stream_rates(timer, cfg, Kd, Vd)
        out["stream_rates_measured_in_this_run"] = rates
        read = max(rates["read_keys_no_projection"]["GBps"], rates["read_keys_values_no_projection"]["GBps"])
        copy = rates["copy_identity_gather"]["GBps"]
        # time the same bytes would take as plain streams: the scan bytes at the better read rate,
        # everything else (scores, indices, gathered rows) at the copy rate
        out["roofline"]["frac_of_stream_rates"] = ((ab["scan"] / read + (ab["total"] - ab["scan"]) / copy) / 1e9
                                                    / (kern_ms * 1e-3))
        out["other_workloads"] = more

    if args.adaptive is not None:
        kbase = int(np.sum(budgets) // heads)                   # the per-head budget the layers share out
        offsets = wl.offsets_for(budgets)
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
        # (timed like the headline: the steps queued back to back, an event pair around each, so
        # that the host's launch latency hides behind the previous step)
        def step_ada(ev):
            if ev:
                ev[0].record()
            ctx.compress_adaptive(Kd, Vd, n, kbase, s, args.adaptive, scores, bd, od, ia, Ka, Va)
            if ev:
                ev[1].record()
        wall_ada, seg = timer.run(step_ada)
        one_ms = seg[:, 0]
        assert bd.cpu().numpy().tolist() == ab_.tolist()
        out["adaptive"] = {"alpha": args.adaptive, "base_budget": kbase,
                           "ms": {"scores": float(pm[0]), "budgets_incl_copy": float(pm[1]),
                                  "select_incl_host_gap": float(pm[2]), "compact": float(pm[3]),
                                  "total": float(pm.sum())},
                           "one_call_ms": float(np.mean(one_ms)), "one_call_ms_median": float(np.median(one_ms)),
                           "one_call_ms_per_step_wall": wall_ada,
                           "one_call_frac_of_hbm_peak": ab["total"] / (float(np.mean(one_ms)) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "budget_min_max": [int(ab_.min()), int(ab_.max())]}
    if args.append:
        raw = torch.empty((heads, n), dtype=torch.float32, device="cuda")
        sums = torch.zeros((heads,), dtype=torch.float64, device="cuda")
        K4, V4 = Kd.view(L, H, n, d), Vd.view(L, H, n, d)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        res = {}
        for m in args.append:
            Kc, Vc = K4[:, :, n - m:].contiguous(), V4[:, :, n - m:].contiguous()
            def step_app(ev, Kc=Kc, Vc=Vc, m=m):
                if ev:
                    ev[0].record()
                ctx.scores_append(Kc, Vc, m, n - m, n, raw, sums)
                if ev:
                    ev[1].record()
            _, seg = timer.run(step_app)
            ts = seg[:, 0]
            bytes_m = heads * m * ((2 if args.source == "kv" else 1) * d * 2 + 4)
            res[str(m)] = {"ms": float(np.mean(ts)), "GBps": bytes_m / (np.mean(ts) * 1e-3) / 1e9,
                           "frac_of_hbm_peak": bytes_m / (np.mean(ts) * 1e-3) / 1e9 / HBM_PEAK_GBS}
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
