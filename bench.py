#!/usr/bin/env python3
"""Benchmark of the PulseCol attention hot path on one MI355X.

A "step" is one attention layer-step of the denoising schedule: a column-sparse attention
call, preceded by the pattern-identification pass (scores + top-k) at the schedule's refresh
steps.  Default workload: LLaDA-8B-shaped single layer at 64K context, keep 10%, 1024 steps
with 4 refreshes.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llada_64k] [--keep 0.1]
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_F32_TFLOPS = 157.3
# HBM-side bytes per launch of the column-sparse attention kernel, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this script scaled by a 1 GiB copy in the same run (summary under profiles/);
# a measured constant of the workload, not something this script can read live.
MEASURED_TRAFFIC_BYTES = {("llada_64k", 0.10): 1.906e9}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="steps of the schedule to time (default: the workload's)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llada_64k")
    ap.add_argument("--keep", type=float, default=None)
    ap.add_argument("--dense-steps", type=int, default=32, help="dense-baseline launches timed beside the run")
    ap.add_argument("--cpu-rows", type=int, default=32768,
                    help="query rows of one head the CPU oracle is timed on (in calls of 2048 rows)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the MFMA-only / copy roofline probes")
    ap.add_argument("--no-32k", action="store_true", help="skip the short side measurement at 32K context")
    ap.add_argument("--no-layers", action="store_true", help="skip the short multi-layer schedule run")
    ap.add_argument("--no-groups", action="store_true", help="skip the short side measurement with group-wise column sets")
    ap.add_argument("--cold-steps", type=int, default=8,
                    help="extra attention launches timed with a 1 GiB buffer overwritten before each (caches evicted)")
    ap.add_argument("--copy-gib", type=float, default=0.0,
                    help="also launch one plain device copy of this many GiB (the known-size kernel that "
                         "calibrates the FETCH_SIZE / WRITE_SIZE counters in a rocprofv3 --pmc run)")
    return ap.parse_args()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every head is independent: sharding by head needs no "
              "collective); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_20813_amd import pulsecol as pc
    from paper_2605_20813_amd import workloads as wl

    w = wl.WORKLOADS[a.workload]
    keep = a.keep if a.keep is not None else (0.10 if 0.10 in w.keep_ratios else w.keep_ratios[0])
    steps = a.steps if a.steps is not None else w.steps
    refresh = sorted(s for s in set(w.refresh_steps) | {0} if s < steps)
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)

    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    k = pc.num_keep(n, keep)
    Qh, Kh, Vh = wl.make_qkv(w)
    Q, K, V = Qh.to(dev), Kh.to(dev), Vh.to(dev)
    O = torch.empty_like(Q)
    idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)
    ctx = pc.Context(B, H, n, d, w.torch_dtype)
    block_m, block_n = ctx.tile_shape()

    def one_step(step, events=None):
        if step in refresh:
            ctx.select(Q, K, keep, refresh=True, idx_out=idx)
        if events is not None:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        ctx.attn(Q, K, V, idx, O=O)
        if events is not None:
            e1.record()
            events.append((e0, e1))

    if a.copy_gib > 0:
        src = torch.zeros(int(a.copy_gib * 2**30) // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up (untimed): the first step selects, the rest reuse
    for s in range(max(a.warmup, 1)):
        one_step(0 if s == 0 else -1)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps of the schedule
    events = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        one_step(s, events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    total_ms = (t1 - t0) * 1e3
    ms_per_step = total_ms / steps
    per_launch = sorted(e0.elapsed_time(e1) for e0, e1 in events)
    attn_ms = sum(per_launch) / len(per_launch)
    attn_ms_median = per_launch[len(per_launch) // 2]
    attn_ms_min = per_launch[0]

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
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    select_ms = timed(lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 2)
    scores = torch.empty(B, H, 1, n, dtype=torch.float32, device=dev)
    ctx.scores(Q, K, scores_out=scores)
    scores_ms = timed(lambda: ctx.scores(Q, K, scores_out=scores), 2)
    topk_ms = timed(lambda: ctx.topk(scores, k, idx_out=idx), 5)
    # top-k is the memory-bound stage of select: algorithmic bytes = the fp32 score rows read once
    # (the kernel holds a row in registers) and k int32 indices written per row
    topk_bytes = B * H * (4 * n + 4 * k)
    dense_ms = timed(lambda: ctx.attn_dense(Q, K, V, O=O), a.dense_steps) if a.dense_steps > 0 else None
    # a refresh step that keeps the dense output: dense attention + column pass + top-k in one call
    refresh_dense_ms = timed(lambda: ctx.refresh_dense(Q, K, V, keep, O=O, idx_out=idx), 2)
    ctx.select(Q, K, keep, refresh=True, idx_out=idx)
    torch.cuda.synchronize()

    kept_flop = 4.0 * B * H * n * k * d
    dense_flop = 4.0 * B * H * float(n) * n * d
    peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_F32_TFLOPS
    achieved = kept_flop / (attn_ms * 1e-3) * 1e-12

    out = {
        "metric": "ms per attention layer-step (select amortised over the refresh schedule)",
        "value": round(ms_per_step, 4),
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
                   "k": k, "refresh_steps": refresh, "block_m": block_m, "block_n": block_n},
        "attn_ms": round(attn_ms, 4),
        "attn_ms_median": round(attn_ms_median, 4),
        "attn_ms_min": round(attn_ms_min, 4),
        "attn_ms_cold": None if attn_ms_cold is None else round(attn_ms_cold, 4),
        # the same layer-step with every attention launch behind a 1 GiB fill (caches flushed, as
        # when the other layers of a model run in between); `value` is the back-to-back figure
        "ms_per_step_cold": None if attn_ms_cold is None else round(ms_per_step - attn_ms + attn_ms_cold, 4),
        "kept_tflops_cold": None if attn_ms_cold is None else round(kept_flop / (attn_ms_cold * 1e-3) * 1e-12, 2),
        "select_ms": round(select_ms, 4),
        "scores_ms": round(scores_ms, 4),
        "topk_ms": round(topk_ms, 4),
        "topk_gbps": round(topk_bytes / (topk_ms * 1e-3) * 1e-9, 1),
        "dense_ms": None if dense_ms is None else round(dense_ms, 4),
        "refresh_dense_ms": round(refresh_dense_ms, 4),
        "speedup_vs_dense": None if dense_ms is None else round(dense_ms / ms_per_step, 3),
        # the whole schedule of one layer: every sparse step and select run for real; the dense side
        # is `dense-steps` identical launches scaled to the same number of steps
        "schedule_total_ms": round(total_ms, 1),
        "dense_schedule_total_ms_scaled": None if dense_ms is None else round(dense_ms * steps, 1),
        "kept_tflops": round(achieved, 2),
        "dense_equivalent_tflops": round(dense_flop / (attn_ms * 1e-3) * 1e-12, 2),
        "dense_kernel_tflops": None if dense_ms is None else round(dense_flop / (dense_ms * 1e-3) * 1e-12, 2),
        "select_tflops": round(dense_flop / (select_ms * 1e-3) * 1e-12, 2),
        "roofline": {"bound": "mfma", "kernel": "attn_bf16_kernel<128, sparse>" if w.dtype == "bf16" else "attn_f32_kernel",
                     "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(achieved / peak, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, round(keep, 4)))},
        "paper_context": "paper: 1.95x end-to-end over FlashAttention at 64K/1024 steps, keep 20%, whole model, RTX PRO 6000",
    }
    # The paper's schedule settings (refresh window eta = 30% of 1024 steps, R = 4 / 8 / 16 refreshes,
    # placed by its schedule equation): ms per layer-step from the times measured above (no extra
    # launches: steps are identical in cost), with the refresh done by select and by the fused
    # refresh_dense that also yields the dense output of the refresh step.
    from paper_2605_20813_amd import schedule as sch
    sweep = []
    for R in (4, 8, 16):
        placed = sch.refresh_steps(1024, 0.30, R)
        sweep.append({"eta": 0.30, "R": R, "first_and_last_refresh_step": [placed[0], placed[-1]],
                      "ms_per_step_select": round(attn_ms + R * select_ms / 1024.0, 4),
                      "ms_per_step_refresh_dense": round((attn_ms * (1024 - R) + R * refresh_dense_ms) / 1024.0, 4),
                      "speedup_vs_dense": None if dense_ms is None else round(dense_ms / (attn_ms + R * select_ms / 1024.0), 3)})
    out["schedule_sweep_1024_steps"] = sweep

    ctx.close()
    del Q, K, V, O, scores, idx
    torch.cuda.empty_cache()
    if not a.no_32k and a.workload == "llada_64k":
        out["context_32k"] = side_config(pc, wl, torch, dev, "llada_32k")
    if not a.no_layers and a.workload == "llada_64k":
        out["multilayer"] = multilayer_run(pc, torch, dev, w, keep, (Qh, Kh, Vh))
    if not a.no_groups and a.workload == "llada_64k":
        out["gqa"] = gqa_config(pc, torch, dev, w, keep, (Qh, Kh, Vh))
    if not a.no_groups and a.workload == "llada_64k":
        out["groupwise"] = [groupwise_config(pc, torch, dev, w, keep, G, (Qh, Kh, Vh)) for G in (256, 128)]
    if not a.no_probes:
        out["probes"] = roofline_probes(achieved, dense_ms and dense_flop / (dense_ms * 1e-3) * 1e-12)
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, Qh, Kh, Vh, k, a.cpu_rows)
    print(json.dumps(out), flush=True)


def side_config(pc, wl, torch, dev, name):
    """The same kernels at the other context length the metric names: per keep ratio the
    column-sparse attention launch alone (20 launches), beside one select and the dense launch."""
    w = wl.WORKLOADS[name]
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    Q, K, V = (t.to(dev) for t in wl.make_qkv(w))
    O = torch.empty_like(Q)
    ctx = pc.Context(B, H, n, d, w.torch_dtype)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    res = {"workload": name, "seq": n, "dense_ms": round(timed(lambda: ctx.attn_dense(Q, K, V, O=O), 4), 4), "keep": {}}
    res["dense_kernel_tflops"] = round(4.0 * B * H * float(n) * n * d / (res["dense_ms"] * 1e-3) * 1e-12, 2)
    for keep in w.keep_ratios:
        k = pc.num_keep(n, keep)
        idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)
        select_ms = timed(lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 1)
        attn_ms = timed(lambda: ctx.attn(Q, K, V, idx, O=O), 20)
        res["keep"][str(keep)] = {"k": k, "attn_ms": round(attn_ms, 4), "select_ms": round(select_ms, 4),
                                  "kept_tflops": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12, 2),
                                  "speedup_vs_dense_launch": round(res["dense_ms"] / attn_ms, 2)}
    ctx.close()
    return res


def multilayer_run(pc, torch, dev, w, keep, host_qkv):
    """A short run of the schedule driver: 4 layers (each with its own cached pattern), 32
    denoising steps, refreshes placed by the schedule equation in a window of eta = 0.5 with
    R = 4 -- every select and every attention launch runs for real; all layers see the same
    synthetic Q, K, V."""
    from paper_2605_20813_amd import schedule as sch
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    L, T, eta, R = 4, 32, 0.5, 4
    steps = sch.refresh_steps(T, eta, R)
    Q, K, V = (t.to(dev) for t in host_qkv)
    out = [torch.empty_like(Q) for _ in range(L)]
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
    ctx = pc.Context(B, H, n, d, w.torch_dtype, kv_heads=Hkv)
    k = pc.num_keep(n, keep)
    idx = torch.empty(B, H, 1, k, dtype=torch.int32, device=dev)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    select_ms = timed(lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 1)
    attn_ms = timed(lambda: ctx.attn(Q, K, V, idx, O=O), 20)
    dense_ms = timed(lambda: ctx.attn_dense(Q, K, V, O=O), 3)
    ctx.close()
    res = {"heads": H, "kv_heads": Hkv, "k": k, "select_ms": round(select_ms, 3), "attn_ms": round(attn_ms, 4),
           "dense_ms": round(dense_ms, 3), "kept_tflops": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12, 2)}
    del Q, K, V, O, idx
    torch.cuda.empty_cache()
    return res


def groupwise_config(pc, torch, dev, w, keep, G, host_qkv):
    """The paper's own pattern format at the headline shape: one column set per query group of
    G rows (256: the main kernel's query block; 128: the paper's largest group size, small-group
    kernel).  The score pass writes [B,H,U,n] fp32, top-k runs over B*H*U rows (the memory-bound
    stage), and the attention gathers are no longer shared between the query blocks of a head."""
    B, H, n, d = w.batch, w.heads, w.seq, w.head_dim
    Q, K, V = (t.to(dev) for t in host_qkv)
    O = torch.empty_like(Q)
    ctx = pc.Context(B, H, n, d, w.torch_dtype, group_size=G)
    U = ctx.groups
    k = pc.num_keep(n, keep)
    idx = torch.empty(B, H, U, k, dtype=torch.int32, device=dev)
    scores = torch.empty(B, H, U, n, dtype=torch.float32, device=dev)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    scores_ms = timed(lambda: ctx.scores(Q, K, scores_out=scores), 2)
    topk_ms = timed(lambda: ctx.topk(scores, k, idx_out=idx), 3)
    select_ms = timed(lambda: ctx.select(Q, K, keep, refresh=True, idx_out=idx), 1)
    attn_ms = timed(lambda: ctx.attn(Q, K, V, idx, O=O), 10 if G >= 256 else 4)
    extra = {}
    if G >= 256:
        # In-house block-sparse point at the same budget (the paper's Sec. 3.1 block mask
        # S(i,j) = G(b(i), b(j)) with query blocks = the groups and key blocks of 64): the same
        # kernel fed whole key blocks, chosen by block mass.  Index bookkeeping with torch ops --
        # this is a comparison input, not part of the product path.  "mass" = share of the
        # group's softmax mass that the kept columns carry (the scores of a group sum to one).
        kb = max(1, k // 64)
        blocks = scores.view(B, H, U, n // 64, 64).sum(-1).topk(kb, dim=-1).indices.sort(dim=-1).values
        bs_idx = (blocks[..., None] * 64 + torch.arange(64, device=dev)).view(B, H, U, kb * 64).to(torch.int32).contiguous()
        bs_ms = timed(lambda: ctx.attn(Q, K, V, bs_idx, O=O), 10)
        mass_cs = scores.gather(-1, idx.long()).sum(-1).mean().item()
        mass_bs = scores.gather(-1, bs_idx.long()).sum(-1).mean().item()
        extra = {"block_sparse_same_budget": {"key_block": 64, "kept_columns": kb * 64, "attn_ms": round(bs_ms, 4),
                                              "mass_kept": round(mass_bs, 4)},
                 "column_sparse_mass_kept": round(mass_cs, 4)}
        del blocks, bs_idx
    topk_bytes = B * H * U * (4 * n + 4 * k)
    gather_bytes = B * H * U * 2 * k * d * 2 + 2 * B * H * n * d * 2      # K and V rows per group, Q, O
    res = {"group_size": G, "groups_per_head": U, "k": k,
           "scores_ms": round(scores_ms, 3), "topk_ms": round(topk_ms, 3),
           "topk_gbps": round(topk_bytes / (topk_ms * 1e-3) * 1e-9, 1),
           "select_ms": round(select_ms, 3), "attn_ms": round(attn_ms, 4),
           "kept_tflops": round(4.0 * B * H * n * k * d / (attn_ms * 1e-3) * 1e-12, 2),
           "attn_requested_gbps": round(gather_bytes / (attn_ms * 1e-3) * 1e-9, 1)}
    res.update(extra)
    ctx.close()
    del Q, K, V, O, idx, scores
    torch.cuda.empty_cache()
    return res


def roofline_probes(kept_tflops, dense_tflops):
    """What the simplest kernels reach on this machine (stand-alone program, child process): an
    MFMA-only loop with constant and with random operands, and a 1 GiB copy."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2605_20813_amd", "roofline_probe")
    if not os.path.exists(exe):
        return {"error": "paper_2605_20813_amd/roofline_probe is not built"}
    try:
        r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
        p = json.loads(r.stdout.strip().splitlines()[-1])
    except Exception as e:       # a probe that does not run is reported, it never stops the benchmark
        return {"error": f"{type(e).__name__}: {e}"}
    ceil = p["mfma_only_tflops_random_operands"]
    p["attn_frac_of_mfma_only_random_operands"] = round(kept_tflops / ceil, 4)
    if dense_tflops:
        p["dense_frac_of_mfma_only_random_operands"] = round(dense_tflops / ceil, 4)
    return p


def cpu_baseline(w, Qh, Kh, Vh, k, rows):
    """The oracle's masked sparse attention, as it stands, on a bounded sample of the same
    workload: `rows` evenly spaced query rows of head 0; scaled to a whole layer-step."""
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
    return {"value": round(dt * 1e3 * scale, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle.sparse_attention_masked on {rows} evenly spaced query rows of head 0 "
                      f"({dt:.2f} s), scaled by heads*seq/rows = {scale:.0f} to one layer-step; select pass not included"}


if __name__ == "__main__":
    main()
