#!/usr/bin/env python3
"""Benchmark of the PulseCol attention hot path on one MI355X.

A "step" is one attention layer-step of the denoising schedule: a column-sparse attention
call, preceded by the pattern-identification pass (scores + top-k) at the schedule's refresh
steps.  Default workload: LLaDA-8B-shaped single layer at 64K context, keep 10%, 1024 steps
with 4 refreshes.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llada_64k] [--keep 0.1]

`--steps K` times exactly K steps of the schedule (`ms_per_step`).  The headline `value` is the
workload's OWN schedule (all of its steps and refreshes, run for real): when K cuts the schedule
short, the whole schedule is run as well and `value` comes from that run (`value_from` says so).
"""

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="steps of the schedule to time (default: the workload's)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llada_64k")
    ap.add_argument("--keep", type=float, default=None)
    ap.add_argument("--dense-steps", type=int, default=32, help="dense-baseline launches timed beside the run")
    ap.add_argument("--cpu-rows", type=int, default=32768,
                    help="query rows of one head the CPU oracle's attention is timed on (in calls of 2048 rows); "
                         "its select pass is timed on half as many")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the MFMA-only / copy roofline probes")
    ap.add_argument("--no-sides", action="store_true", help="skip the other configurations (4K, 16K drift, 32K, 128K)")
    ap.add_argument("--no-layers", action="store_true", help="skip the multi-layer schedule run")
    ap.add_argument("--no-groups", action="store_true", help="skip the side measurements with group-wise column sets / GQA")
    ap.add_argument("--no-sweep", action="store_true", help="skip the R = 8 / 16 schedule runs")
    ap.add_argument("--no-full-schedule", action="store_true",
                    help="do not run the workload's whole schedule when --steps cuts it short (value = the timed steps)")
    ap.add_argument("--cold-steps", type=int, default=8,
                    help="extra attention launches timed with a 1 GiB buffer overwritten before each (caches evicted)")
    ap.add_argument("--copy-gib", type=float, default=0.0,
                    help="also launch one plain device copy of this many GiB (the known-size kernel that "
                         "calibrates the FETCH_SIZE / WRITE_SIZE counters in a rocprofv3 --pmc run)")
    return ap.parse_args()


def timed(torch, fn, reps):
    """Average milliseconds of `reps` back-to-back calls (events on the launch stream), after one warm call."""
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def run_schedule(torch, ctx, Q, K, V, O, idx, keep, steps, refresh, events=None):
    """`steps` layer-steps for real: select at the refresh steps, column-sparse attention at every step.
    Returns wall milliseconds (host clock around the whole run, device drained on both sides)."""
    refresh = frozenset(refresh)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        if s in refresh:
            ctx.select(Q, K, keep, refresh=True, idx_out=idx)
        if events is not None:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        ctx.attn(Q, K, V, idx, O=O)
        if events is not None:
            e1.record()
            events.append((e0, e1))
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3


def measured_traffic(workload, keep):
    """HBM bytes per launch of the column-sparse kernel from the committed rocprofv3 --pmc summary
    of this workload (a line `traffic_bytes_per_launch: X` and one `collected_at_commit: SHA`), or
    (None, why) when no such summary travels with this tree."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_{workload}_keep{int(round(keep * 100))}.md")
    try:
        text = open(path).read()
        val = float(re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text).group(1))
        sha = re.search(r"collected_at_commit:\s*(\w+)", text)
        return val, f"profiles/{os.path.basename(path)} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, collected at commit {sha.group(1) if sha else 'unknown'})"
    except Exception:
        return None, "no committed counter summary for this workload next to this script"


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every head is independent: sharding by head needs no "
              "collective); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_20813_amd import pulsecol as pc
    from paper_2605_20813_amd import schedule as sch
    from paper_2605_20813_amd import workloads as wl

    w = wl.WORKLOADS[a.workload]
    keep = a.keep if a.keep is not None else (0.10 if 0.10 in w.keep_ratios else w.keep_ratios[0])
    steps = a.steps if a.steps is not None else w.steps
    cfg_refresh = sorted(set(w.refresh_steps) | {0})
    refresh = [s for s in cfg_refresh if s < steps]
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)

    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    k = pc.num_keep(n, keep)
    Qh, Kh, Vh = wl.make_qkv(w)
    Q, K, V = Qh.to(dev), Kh.to(dev), Vh.to(dev)
    O = torch.empty_like(Q)
    idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)
    ctx = pc.Context(B, H, n, d, w.torch_dtype, max_keep_ratio=keep)
    block_m, block_n = ctx.tile_shape(k)

    if a.copy_gib > 0:
        src = torch.zeros(int(a.copy_gib * 2**30) // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up (untimed): the first step selects, the rest reuse
    run_schedule(torch, ctx, Q, K, V, O, idx, keep, max(a.warmup, 1), [0])

    # ---- timed region: exactly `steps` steps of the schedule
    events = []
    total_ms = run_schedule(torch, ctx, Q, K, V, O, idx, keep, steps, refresh, events)
    ms_per_step = total_ms / steps
    per_launch = sorted(e0.elapsed_time(e1) for e0, e1 in events)
    attn_ms = sum(per_launch) / len(per_launch)
    attn_ms_median = per_launch[len(per_launch) // 2]
    attn_ms_min = per_launch[0]

    # ---- the workload's own schedule, whole, when --steps cut it short
    value, value_steps, value_refresh = ms_per_step, steps, refresh
    value_from = f"the {steps} timed steps (the workload's whole schedule)"
    schedule_total_ms = total_ms
    if steps < w.steps and not a.no_full_schedule:
        schedule_total_ms = run_schedule(torch, ctx, Q, K, V, O, idx, keep, w.steps, cfg_refresh)
        value, value_steps, value_refresh = schedule_total_ms / w.steps, w.steps, cfg_refresh
        value_from = (f"a separate run of the workload's whole schedule ({w.steps} steps, select at {cfg_refresh}, every "
                      f"launch for real); --steps {steps} cuts that schedule short and is reported as ms_per_step")
    elif steps < w.steps:
        value_from = f"the {steps} timed steps only: a truncated schedule (the workload's has {w.steps} steps, select at {cfg_refresh})"

    # ---- cold regime: L2 and the 256 MB memory-side cache evicted before every launch
    attn_ms_cold = None
    if a.cold_steps > 0:
        flush = torch.empty(2**30 // 4, dtype=torch.float32, device=dev)
        cold = []
        for _ in range(a.cold_steps):
            flush.fill_(1.0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ctx.attn(Q, K, V, idx, O=O)
            e1.record()
            cold.append((e0, e1))
        torch.cuda.synchronize()
        attn_ms_cold = sum(e0.elapsed_time(e1) for e0, e1 in cold) / len(cold)
        del flush

    # ---- the pieces, each timed alone with events on the launch stream
    select_ms = timed(torch, lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 2)
    scores = torch.empty(B, H, 1, n, dtype=torch.float32, device=dev)
    scores_ms = timed(torch, lambda: ctx.scores(Q, K, scores_out=scores), 2)
    topk_ms = timed(torch, lambda: ctx.topk(scores, k, idx_out=idx), 5)
    # top-k is the memory-bound stage of select: algorithmic bytes = the fp32 score rows read once
    # (the kernel holds a row in registers) and k int32 indices written per row
    topk_bytes = B * H * (4 * n + 4 * k)
    dense_ms = timed(torch, lambda: ctx.attn_dense(Q, K, V, O=O), a.dense_steps) if a.dense_steps > 0 else None
    # a refresh step that keeps the dense output: dense attention + column pass + top-k in one call
    refresh_dense_ms = timed(torch, lambda: ctx.refresh_dense(Q, K, V, keep, O=O, idx_out=idx), 2)
    ctx.select(Q, K, keep, refresh=True, idx_out=idx)
    torch.cuda.synchronize()

    kept_flop = 4.0 * B * H * n * k * d
    dense_flop = 4.0 * B * H * float(n) * n * d
    peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_F32_TFLOPS
    achieved = kept_flop / (attn_ms * 1e-3) * 1e-12
    algorithmic_bytes = B * H * (2 * n * d + 2 * k * d) * Q.element_size() + B * H * 4 * k     # Q, O, selected K and V rows once, idx
    traffic, traffic_source = measured_traffic(w.name, keep)
    kernel = (f"{'attn_bf16_kernel' if block_m == 256 else 'attn_bf16_group_kernel'}<{d}, sparse> ({block_m}-row query blocks, "
              f"{block_n}-column tiles)" if w.dtype == "bf16"
              else f"attn_f32_kernel<{d}, sparse> ({block_m}-row query blocks, {block_n}-column tiles)")

    out = {
        "metric": "ms per attention layer-step (select amortised over the refresh schedule)",
        "value": round(value, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "heads": H, "seq": n, "head_dim": d, "keep_ratio": keep,
                   "k": k, "schedule_steps": w.steps, "schedule_refresh_steps": cfg_refresh,
                   "timed_steps": steps, "timed_refresh_steps": refresh, "block_m": block_m, "block_n": block_n},
        "value_from": value_from,
        # the same figure put together from the launch times of the timed steps (short bursts run at a higher clock
        # than the sustained run of the whole schedule that `value` comes from)
        "value_from_launch_times": round(attn_ms + select_ms * len(cfg_refresh) / w.steps, 4),
        "value_steps": value_steps,
        "value_refresh_steps": value_refresh,
        "attn_ms": round(attn_ms, 4),
        "attn_ms_median": round(attn_ms_median, 4),
        "attn_ms_min": round(attn_ms_min, 4),
        "attn_ms_cold": None if attn_ms_cold is None else round(attn_ms_cold, 4),
        # the same layer-step with every attention launch behind a 1 GiB fill (caches flushed, as
        # when the other layers of a model run in between); `value` is the back-to-back figure
        "value_cold": None if attn_ms_cold is None else round(value - attn_ms + attn_ms_cold, 4),
        "kept_tflops_cold": None if attn_ms_cold is None else round(kept_flop / (attn_ms_cold * 1e-3) * 1e-12, 2),
        "select_ms": round(select_ms, 4),
        "scores_ms": round(scores_ms, 4),
        "topk_ms": round(topk_ms, 4),
        "topk_gbps": round(topk_bytes / (topk_ms * 1e-3) * 1e-9, 1),
        "dense_ms": None if dense_ms is None else round(dense_ms, 4),
        "refresh_dense_ms": round(refresh_dense_ms, 4),
        # against dense attention at every step of the same schedule (`dense-steps` identical launches, scaled)
        "speedup_vs_dense": None if dense_ms is None else round(dense_ms / value, 3),
        "schedule_total_ms": round(schedule_total_ms, 1),
        "dense_schedule_total_ms_scaled": None if dense_ms is None else round(dense_ms * value_steps, 1),
        "kept_tflops": round(achieved, 2),
        "dense_equivalent_tflops": round(dense_flop / (attn_ms * 1e-3) * 1e-12, 2),
        "dense_kernel_tflops": None if dense_ms is None else round(dense_flop / (dense_ms * 1e-3) * 1e-12, 2),
        "select_tflops": round(dense_flop / (select_ms * 1e-3) * 1e-12, 2),
        "roofline": {"bound": "mfma", "kernel": kernel,
                     "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(achieved / peak, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": algorithmic_bytes},
        "paper_context": "paper: 1.95x end-to-end over FlashAttention at 64K/1024 steps, keep 20%, whole model, RTX PRO 6000",
    }

    # The paper's schedule settings (refresh window eta = 30% of the steps, R refreshes placed by its
    # schedule equation): R = 4 is the workload's own schedule above; R = 8 and 16 are run here, whole,
    # with select at the refresh steps.  The fused-refresh column is the same runs with the select
    # launches replaced by refresh_dense at their measured time.
    if not a.no_sweep and a.workload == "llada_64k":
        sweep = []
        for R in (4, 8, 16):
            placed = sch.refresh_steps(w.steps, 0.30, R)
            if R == 4 and placed == cfg_refresh and value_steps == w.steps:
                run_ms, how = schedule_total_ms, "the headline run"
            else:
                run_ms, how = run_schedule(torch, ctx, Q, K, V, O, idx, keep, w.steps, placed), "run for real"
            per = run_ms / w.steps
            sweep.append({"eta": 0.30, "R": R, "first_and_last_refresh_step": [placed[0], placed[-1]], "how": how,
                          "ms_per_step_select": round(per, 4),
                          "ms_per_step_refresh_dense_estimate": round(per + R * (refresh_dense_ms - select_ms - attn_ms) / w.steps, 4),
                          "speedup_vs_dense": None if dense_ms is None else round(dense_ms / per, 3)})
        out["schedule_sweep"] = sweep

    ctx.close()
    del Q, K, V, O, scores, idx
    torch.cuda.empty_cache()
    main_64k = a.workload == "llada_64k"
    if not a.no_sides and main_64k:
        out["config_4k"] = reuse_config(pc, wl, torch, dev, "llada_4k")
        out["config_16k_drift"] = drift_config(pc, wl, torch, dev, "llada_16k")
        out["context_32k"] = side_config(pc, wl, torch, dev, "llada_32k")
        out["context_128k"] = side_config(pc, wl, torch, dev, "llada_128k_8h")
    if not a.no_layers and main_64k:
        out["multilayer"] = multilayer_run(pc, torch, dev, w, keep, (Qh, Kh, Vh))
    if not a.no_groups and main_64k:
        out["gqa"] = gqa_config(pc, torch, dev, w, keep, (Qh, Kh, Vh))
        out["groupwise"] = [groupwise_config(pc, torch, dev, w, keep, G, (Qh, Kh, Vh)) for G in (256, 128, 64, 32)]
    if not a.no_probes:
        out["probes"] = roofline_probes(achieved, dense_ms and dense_flop / (dense_ms * 1e-3) * 1e-12)
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, Qh, Kh, Vh, k, a.cpu_rows, len(cfg_refresh))
    print(json.dumps(out), flush=True)


def reuse_config(pc, wl, torch, dev, name):
    """Select at step 0, then the workload's steps of column-sparse attention on the same indices,
    all for real; the pieces timed alone beside it."""
    w = wl.WORKLOADS[name]
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    keep = w.keep_ratios[0]
    k = pc.num_keep(n, keep)
    Q, K, V = (t.to(dev) for t in wl.make_qkv(w))
    O = torch.empty_like(Q)
    idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)
    ctx = pc.Context(B, H, n, d, w.torch_dtype, max_keep_ratio=keep)
    run_schedule(torch, ctx, Q, K, V, O, idx, keep, 2, [0])
    runs = sorted(run_schedule(torch, ctx, Q, K, V, O, idx, keep, w.steps, [0]) for _ in range(5))
    total_ms = runs[len(runs) // 2]
    attn_ms = timed(torch, lambda: ctx.attn(Q, K, V, idx, O=O), 50)
    select_ms = timed(torch, lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 5)
    dense_ms = timed(torch, lambda: ctx.attn_dense(Q, K, V, O=O), 10)
    block_m, block_n = ctx.tile_shape(k)
    ctx.close()
    return {"workload": name, "seq": n, "keep": keep, "k": k, "steps": w.steps, "refresh_steps": [0],
            "block_m": block_m, "block_n": block_n,
            "total_ms": round(total_ms, 4), "ms_per_step": round(total_ms / w.steps, 4),
            "attn_ms": round(attn_ms, 4), "select_ms": round(select_ms, 4), "dense_ms": round(dense_ms, 4),
            "kept_tflops": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12, 2),
            "dense_kernel_tflops": round(4.0 * B * H * float(n) * n * d / (dense_ms * 1e-3) * 1e-12, 2),
            "speedup_vs_dense": round(dense_ms * w.steps / total_ms, 3),
            "note": "total_ms = one select + the steps' attention launches, host clock, median of 5 runs"}


def drift_config(pc, wl, torch, dev, name):
    """The drifting schedule: before every step the fp32 masters of Q, K, V take 0.05 N(0,1) noise
    and are rounded to bf16 again (on the device, untimed); select runs at the refresh steps on the
    inputs of that step, attention at every step.  The library calls of each step are timed with
    events on the launch stream; the noise generation in between is not."""
    w = wl.WORKLOADS[name]
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    keep = w.keep_ratios[0]
    k = pc.num_keep(n, keep)
    masters = [t.to(dev) for t in wl.make_qkv(w, master=True)]
    Q, K, V = (m.to(w.torch_dtype) for m in masters)
    O = torch.empty_like(Q)
    idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)
    ctx = pc.Context(B, H, n, d, w.torch_dtype, max_keep_ratio=keep)
    ctx.select(Q, K, keep, refresh=True, idx_out=idx)
    ctx.attn(Q, K, V, idx, O=O)
    torch.cuda.synchronize()
    refresh = sorted(set(w.refresh_steps) | {0})
    ev, patterns, stale_overlap = [], [], []
    for s in range(w.steps):
        if s > 0:
            wl.drift_(masters, w, s)
            for dst, m in zip((Q, K, V), masters):
                dst.copy_(m)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if s in refresh:
            ctx.select(Q, K, keep, refresh=True, idx_out=idx)
        ctx.attn(Q, K, V, idx, O=O)
        e1.record()
        ev.append((s, e0, e1))
        if s in refresh:
            patterns.append(idx.clone())
    torch.cuda.synchronize()
    times = {s: e0.elapsed_time(e1) for s, e0, e1 in ev}
    total_ms = sum(times.values())
    reuse = [t for s, t in times.items() if s not in refresh]
    # how far the pattern moved between refreshes: share of a head's columns kept from the previous pattern
    for prev, cur in zip(patterns, patterns[1:]):
        both = torch.cat([prev, cur], dim=-1).sort(dim=-1).values
        same = (both[..., 1:] == both[..., :-1]).sum(dim=-1).float() / k
        stale_overlap.append(round(same.mean().item(), 4))
    dense_ms = timed(torch, lambda: ctx.attn_dense(Q, K, V, O=O), 4)
    ctx.close()
    return {"workload": name, "seq": n, "keep": keep, "k": k, "steps": w.steps, "refresh_steps": refresh,
            "drift_sigma": w.drift_sigma, "total_ms": round(total_ms, 3), "ms_per_step": round(total_ms / w.steps, 4),
            "attn_ms": round(sum(reuse) / len(reuse), 4),
            "refresh_step_ms": [round(times[s], 3) for s in refresh],
            "kept_tflops": round(4.0 * B * H * n * k * d / (sum(reuse) / len(reuse) * 1e-3) * 1e-12, 2),
            "dense_ms": round(dense_ms, 4), "speedup_vs_dense": round(dense_ms * w.steps / total_ms, 3),
            "columns_kept_from_previous_pattern": stale_overlap}


def side_config(pc, wl, torch, dev, name):
    """The same kernels at another context length: per keep ratio the column-sparse attention
    launch alone (20 launches), beside one select and the dense launch."""
    w = wl.WORKLOADS[name]
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    Q, K, V = (t.to(dev) for t in wl.make_qkv(w))
    O = torch.empty_like(Q)
    ctx = pc.Context(B, H, n, d, w.torch_dtype, max_keep_ratio=max(w.keep_ratios))
    res = {"workload": name, "heads": H, "seq": n, "dense_ms": round(timed(torch, lambda: ctx.attn_dense(Q, K, V, O=O), 4), 4), "keep": {}}
    res["dense_kernel_tflops"] = round(4.0 * B * H * float(n) * n * d / (res["dense_ms"] * 1e-3) * 1e-12, 2)
    for keep in w.keep_ratios:
        k = pc.num_keep(n, keep)
        idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)
        select_ms = timed(torch, lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 1)
        attn_ms = timed(torch, lambda: ctx.attn(Q, K, V, idx, O=O), 20)
        res["keep"][str(keep)] = {"k": k, "attn_ms": round(attn_ms, 4), "select_ms": round(select_ms, 4),
                                  "kept_tflops": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12, 2),
                                  "speedup_vs_dense_launch": round(res["dense_ms"] / attn_ms, 2)}
    ctx.close()
    return res


def multilayer_run(pc, torch, dev, w, keep, host_qkv):
    """The schedule driver over a whole model's worth of layers: 32 layers, each with its own
    context and cached pattern, 16 denoising steps, refreshes placed by the schedule equation in a
    window of eta = 0.5 with R = 2 -- every select and every attention launch runs for real; all
    layers see the same synthetic Q, K, V and write one shared output."""
    from paper_2605_20813_amd import schedule as sch
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    L, T, eta, R = 32, 16, 0.5, 2
    steps = sch.refresh_steps(T, eta, R)
    Q, K, V = (t.to(dev) for t in host_qkv)
    O = torch.empty_like(Q)
    out = [O] * L
    qkv = [(Q, K, V)] * L
    with sch.LayerStack(L, B, H, n, d, w.torch_dtype, keep, steps) as stack:
        stack.step(0, qkv, out)                     # warm-up (also allocates the index tensors)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        selects = sum(stack.step(t, qkv, out) for t in range(T))
        torch.cuda.synchronize()
        total_ms = (time.perf_counter() - t0) * 1e3
    return {"layers": L, "steps": T, "eta": eta, "R": R, "kind": "uniform", "refresh_steps": steps,
            "selects_run": selects, "total_ms": round(total_ms, 1),
            "ms_per_layer_step": round(total_ms / (L * T), 4)}


def gqa_config(pc, torch, dev, w, keep, host_qkv):
    """Grouped-query layout at the headline shape: 32 query heads on 8 K/V heads (the workload's
    first 8 K/V heads), one pattern per query head."""
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    Hkv = 8
    Q, K, V = (t.to(dev) for t in host_qkv)
    K, V = (torch.empty(B, Hkv, n, d, dtype=t.dtype, device=dev).copy_(t[:, :Hkv]) for t in (K, V))
    O = torch.empty_like(Q)
    ctx = pc.Context(B, H, n, d, w.torch_dtype, kv_heads=Hkv, max_keep_ratio=keep)
    k = pc.num_keep(n, keep)
    idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)
    select_ms = timed(torch, lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 1)
    attn_ms = timed(torch, lambda: ctx.attn(Q, K, V, idx, O=O), 20)
    dense_ms = timed(torch, lambda: ctx.attn_dense(Q, K, V, O=O), 3)
    ctx.close()
    res = {"heads": H, "kv_heads": Hkv, "k": k, "select_ms": round(select_ms, 3), "attn_ms": round(attn_ms, 4),
           "dense_ms": round(dense_ms, 3), "kept_tflops": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12, 2)}
    del Q, K, V, O, idx
    torch.cuda.empty_cache()
    return res


def groupwise_config(pc, torch, dev, w, keep, G, host_qkv):
    """The paper's own pattern format at the headline shape: one column set per query group of
    G rows (256: the main kernel's query block; 128 / 64 / 32: the paper's group sizes, small-group
    kernel).  The score pass writes [B,H,U,n] fp32, top-k runs over B*H*U rows (the memory-bound
    stage), and the attention gathers are no longer shared between the query blocks of a head."""
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    Q, K, V = (t.to(dev) for t in host_qkv)
    O = torch.empty_like(Q)
    ctx = pc.Context(B, H, n, d, w.torch_dtype, group_size=G, max_keep_ratio=keep)
    U = ctx.groups
    k = pc.num_keep(n, keep)
    idx = torch.empty(B, H, U, k, dtype=torch.int32, device=dev)
    scores = torch.empty(B, H, U, n, dtype=torch.float32, device=dev)

    scores_ms = timed(torch, lambda: ctx.scores(Q, K, scores_out=scores), 2)
    topk_ms = timed(torch, lambda: ctx.topk(scores, k, idx_out=idx), 3)
    select_ms = timed(torch, lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 1)
    attn_ms = timed(torch, lambda: ctx.attn(Q, K, V, idx, O=O), 10 if G >= 256 else 4)
    extra = {}
    if G >= 256:
        # In-house block-sparse point at the same budget (the paper's Sec. 3.1 block mask
        # S(i,j) = G(b(i), b(j)) with query blocks = the groups and key blocks of 64): the library's block
        # selection (key blocks by block mass) and its block-sparse kernel (a tile = one key block, fetched
        # as 64 consecutive rows from one block number), beside the same sets expanded to columns and fed
        # to the column-sparse kernel.  "mass" = share of a group's softmax mass that the kept columns
        # carry (the scores of a group sum to one), from the scores with torch ops (a report, not the path).
        kb = pc.num_keep_blocks(n, keep)
        blk = torch.empty(B, H, U, kb, dtype=torch.int32, device=dev)
        bs_select_ms = timed(torch, lambda: ctx.select_blocks(Q, K, keep, block_idx_out=blk), 1)
        bs_ms = timed(torch, lambda: ctx.attn_block(Q, K, V, blk, O=O), 10)
        bs_idx = (blk[..., None].long() * 64 + torch.arange(64, device=dev)).view(B, H, U, kb * 64).to(torch.int32).contiguous()
        bs_cols_ms = timed(torch, lambda: ctx.attn(Q, K, V, bs_idx, O=O), 10)
        ctx.scores(Q, K, scores_out=scores)
        mass_cs = scores.gather(-1, idx.long()).sum(-1).mean().item()
        mass_bs = scores.gather(-1, bs_idx.long()).sum(-1).mean().item()
        extra = {"block_sparse_same_budget": {"key_block": 64, "kept_blocks": kb, "kept_columns": kb * 64,
                                              "select_blocks_ms": round(bs_select_ms, 3), "attn_block_ms": round(bs_ms, 4),
                                              "kept_tflops": round(4.0 * B * H * n * kb * 64 * d / (bs_ms * 1e-3) * 1e-12, 2),
                                              "same_sets_through_column_kernel_ms": round(bs_cols_ms, 4),
                                              "mass_kept": round(mass_bs, 4)},
                 "column_sparse_mass_kept": round(mass_cs, 4)}
        del blk, bs_idx
    topk_bytes = B * H * U * (4 * n + 4 * k)
    gather_bytes = B * H * U * 2 * k * d * 2 + 2 * B * H * n * d * 2      # K and V rows per group, Q, O
    res = {"group_size": G, "groups_per_head": U, "k": k,
           "scores_ms": round(scores_ms, 3), "topk_ms": round(topk_ms, 3),
           "topk_gbps": round(topk_bytes / (topk_ms * 1e-3) * 1e-9, 1),
           "topk_frac_of_hbm_peak": round(topk_bytes / (topk_ms * 1e-3) * 1e-9 / PEAK_HBM_GBPS, 4),
           "select_ms": round(select_ms, 3), "attn_ms": round(attn_ms, 4),
           "kept_tflops": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12, 2),
           "kept_frac_of_mfma_peak": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 4),
           "attn_requested_gbps": round(gather_bytes / (attn_ms * 1e-3) * 1e-9, 1)}
    res.update(extra)
    ctx.close()
    del Q, K, V, O, idx, scores
    torch.cuda.empty_cache()
    return res


def roofline_probes(kept_tflops, dense_tflops):
    """What the simplest kernels reach on this machine (stand-alone program, child process): an
    MFMA-only loop with constant and with random operands, the same loop with one or two softmax
    weights per matrix instruction (the instruction mix of the attention kernels and of the select
    passes), and a 1 GiB copy."""
    import subprocess
    exe = os.path.join(ROOT, "roofline_probe.bin")
    if not os.path.exists(exe):
        return {"error": "roofline_probe.bin is not built (python -m paper_2605_20813_amd.build)"}
    try:
        r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
        p = json.loads(r.stdout.strip().splitlines()[-1])
    except Exception as e:       # a probe that does not run is reported, it never stops the benchmark
        return {"error": f"{type(e).__name__}: {e}"}
    ceil = p["mfma_only_tflops_random_operands"]
    p["attn_frac_of_mfma_only_random_operands"] = round(kept_tflops / ceil, 4)
    if dense_tflops:
        p["dense_frac_of_mfma_only_random_operands"] = round(dense_tflops / ceil, 4)
    # the same matrix instructions with the attention kernels' one softmax weight per instruction beside them
    mix = p.get("mfma_plus_1_weight_tflops")
    if mix:
        p["attn_frac_of_mfma_plus_1_weight"] = round(kept_tflops / mix, 4)
    return p


def cpu_baseline(w, Qh, Kh, Vh, k, rows, refreshes):
    """The oracle as it stands (numpy: fp64 matrix products through its threaded BLAS, everything
    else plain numpy) on a bounded sample of the same workload, scaled to a whole layer-step:
    the masked sparse attention on `rows` evenly spaced query rows of head 0, and the select pass
    (column scores + top-k) on rows/2 of them."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    n = w.seq
    rows = min(rows, n)
    sel = np.linspace(0, n - 1, rows).astype(np.int64)
    q, kk, v = (t[0, 0].double().numpy() for t in (Qh, Kh, Vh))
    # k distinct seeded columns: the cost of the masked attention does not depend on which ones
    cols = np.sort(np.random.default_rng(w.seed).choice(n, size=k, replace=False)).astype(np.int32)[None, :]
    t0 = time.perf_counter()
    for c in range(0, rows, 2048):           # bounded memory: 2048 x n logits in fp64 per call
        oracle.sparse_attention_masked(q, kk, v, cols, rows=sel[c:c + 2048])
    dt = time.perf_counter() - t0
    scale = (w.batch * w.heads * n) / rows
    attn_ms = dt * 1e3 * scale
    # select: the scores of a query-row sample against all keys (the cost is linear in the rows), then top-k
    srows = max(1, rows // 2)
    ssel = np.linspace(0, n - 1, srows).astype(np.int64)
    t0 = time.perf_counter()
    s = oracle.column_scores(q[ssel], kk)
    dt_scores = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.topk_columns(s, k)
    dt_topk = time.perf_counter() - t0
    select_ms = (dt_scores * (n / srows) + dt_topk) * 1e3 * w.batch * w.heads
    value = attn_ms + refreshes * select_ms / w.steps
    return {"value": round(value, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
            "attn_ms_per_layer_step": round(attn_ms, 1), "select_ms_per_refresh": round(select_ms, 1),
            "sample": f"numpy + threaded BLAS, {int(cores)} threads. oracle.sparse_attention_masked on {rows} evenly spaced query "
                      f"rows of head 0 ({dt:.2f} s), scaled by heads*seq/rows = {scale:.0f} to one layer-step; "
                      f"oracle.column_scores on {srows} rows of head 0 against all keys ({dt_scores:.2f} s, scaled by "
                      f"seq/rows and heads) + oracle.topk_columns of one head ({dt_topk * 1e3:.1f} ms, scaled by heads) = "
                      f"one select; value = attention + {refreshes} selects / {w.steps} steps (extrapolated, labelled as such)"}


if __name__ == "__main__":
    main()
