#!/usr/bin/env python3
"""Benchmark of the NOVA hot path on one MI355X.

A "step" is one next-scale step of the named workload: its L transformer blocks, each
nova_entropy -> nova_select -> nova_pruned_block -> nova_merge_cache, enqueued back to back
on one stream with every input (logits, weights, KV caches, residual caches) already
resident in HBM.  Prints ONE JSON line:

  value        kept tokens per second through the pruned blocks (B * sum_j k_j / step time)
  ms_per_step  milliseconds per last-scale step
  roofline     the dominant kernel (attention) against the bf16 MFMA peak, timed with HIP
               events on the launch stream inside the timed region
  kernels      per-stage device time from a second, fully instrumented pass (entropy / merge
               as HBM GB/s, GEMMs / attention as TFLOP/s)
  cpu_baseline the CPU oracle timed on this machine's host cores on a bounded sample

Synthetic data: block 0 comes from the seeded host generators (the oracle sees the same
bytes); the other blocks are drawn on the device with the same distributions.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
METRIC = "pruned-block kept tokens/sec + ms per last-scale step; entropy/select HBM GB/s"


def device_block(wl, scale, j, k, gen, dtype, cap, host_block=None):
    """Device tensors of block j.  With host_block the seeded host tensors are uploaded."""
    import torch
    from paper_2602_01345_amd import pack_k_cache, pack_v_cache
    from paper_2602_01345_amd.step import BlockState
    dev = "cuda"
    B, N, C, H, dh, V, F = wl.B, scale.N, wl.C, wl.heads, wl.dh, wl.V, wl.F
    P = scale.kv_len
    if host_block is not None:
        hb = host_block
        return BlockState(k=k, logits=hb.logits.to(dev), weights={n: t.to(dev) for n, t in hb.weights.items()},
                          k_cache=pack_k_cache(hb.k_prior.to(dev), H, cap), v_cache=pack_v_cache(hb.v_prior.to(dev), H, cap),
                          cache_prev=hb.cache_prev.to(dev))

    def randn(shape, std=1.0):
        t = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
        if std != 1.0:
            t *= std
        return t.to(dtype)

    temp = torch.exp(torch.empty((B, N, 1), device=dev).uniform_(math.log(0.1), math.log(10.0), generator=gen))
    logits = (torch.randn((B, N, V), generator=gen, device=dev) * temp).to(dtype)
    shapes = {"w_qkv": (3 * C, C), "b_qkv": (3 * C,), "w_o": (C, C), "b_o": (C,),
              "w_fc1": (F, C), "b_fc1": (F,), "w_fc2": (C, F), "b_fc2": (C,)}
    weights = {n: randn(s, 0.02) for n, s in shapes.items()}
    kc = randn((B, H, cap, dh))
    vc = randn((B, H, dh, cap))
    kc[:, :, P:] = 0
    vc[:, :, :, P:] = 0
    prev = randn((B, scale.prev_grid ** 2, C))
    return BlockState(k=k, logits=logits, weights=weights, k_cache=kc, v_cache=vc, cache_prev=prev)


def stage_work(wl, scale, k):
    """Algorithmic bytes / flops of each stage for one block with keep count k."""
    e = 2 if wl.dtype == "bf16" else 4
    B, N, C, V, F = wl.B, scale.N, wl.C, wl.V, wl.F
    M, kv = B * k, scale.kv_len + k
    hpwp = scale.prev_grid ** 2
    return {
        "entropy": ("bytes", B * N * (V * e + 4)),
        "select": ("bytes", B * (4 * N + 4 * k + N)),
        "gather_ln": ("bytes", 2 * M * C * e),
        "qkv": ("flops", 2 * M * C * 3 * C),
        "attention": ("flops", 4 * B * k * kv * C),
        "oproj": ("flops", 2 * M * C * C),
        "ln2": ("bytes", 2 * M * C * e),
        "ffn1": ("flops", 2 * M * C * F),
        "ffn2": ("flops", 2 * M * C * F),
        "merge": ("bytes", B * (N + hpwp + k) * C * e + 2 * B * N * C * e),
    }


def cpu_baseline(hb0, wl, scale, ks):
    """Times the CPU oracle, as it stands, on four blocks of the step (first, two in between, last: from the most
    to the fewest kept tokens), every batch row, one after the other: 10-15 s of float64 NumPy on the host
    cores.  Input generation is not timed."""
    import numpy as np
    import workloads as WL
    from oracle import nova_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    torch = __import__("torch")
    blocks = sorted({0, wl.L // 3, 2 * wl.L // 3, wl.L - 1})
    rows = min(wl.B, 4)
    dt, kept = 0.0, 0
    for j in blocks:
        if j == 0:
            logits, x, weights, kp, vp, cp = hb0.logits, hb0.x, hb0.weights, hb0.k_prior, hb0.v_prior, hb0.cache_prev
        else:
            kp, vp = WL.make_kv_prior(wl, j, scale)
            logits, x, weights = WL.make_logits(wl, j, scale), WL.make_x(wl, scale), WL.make_weights(wl, j)
            cp = WL.make_cache_prev(wl, j, scale)
        W = {n: t.double().numpy() for n, t in weights.items()}
        k = ks[j]
        t0 = time.perf_counter()
        for b in range(rows):
            f64 = lambda t: t[b:b + 1].to(dtype=torch.float64).numpy()
            H = O.entropy(f64(logits))
            idx, mask = O.select(H.astype(np.float32), k)
            y, _, _ = O.pruned_block(f64(x), idx, W, f64(kp), f64(vp), wl.heads)
            O.merge_cache(f64(x), y, idx, f64(cp), scale.prev_grid, scale.prev_grid, scale.grid, scale.grid)
        dt += time.perf_counter() - t0
        kept += rows * k
    return {"value": kept / dt, "unit": "kept tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{wl.name} blocks {blocks}, batch rows 0..{rows - 1} of {wl.B} ({kept} kept tokens): "
                      f"entropy+select+pruned block+merge in float64 NumPy, {dt:.1f} s"}


def compact_config(nova, wl, scale, steps=3, warmup=2, reps=2):
    """One workload scale, measured compactly: ms per step (all L blocks, one stream) and, from an instrumented
    pass, the fraction of the bf16 MFMA peak of attention and of the four projections together and the fraction of
    the HBM peak of entropy and merge.  Inputs are drawn on the device; everything is freed on return."""
    import torch
    import workloads as WL
    from paper_2602_01345_amd.binding import STAGES
    from paper_2602_01345_amd.step import StepRunner
    dtype = WL.torch_dtype(wl.dtype)
    cap = wl.kv_capacity(scale)
    runner = StepRunner(nova, B=wl.B, grid=scale.grid, prev_grid=scale.prev_grid, C=wl.C, heads=wl.heads,
                        kv_len=scale.kv_len, kv_capacity=cap, dtype=dtype, ffn_mult=wl.ffn_mult)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.seed + scale.grid)
    ks = wl.k_table(scale)
    for j in range(wl.L):
        runner.add_block(device_block(wl, scale, j, ks[j], gen, dtype, cap))
    x = torch.randn((wl.B, scale.N, wl.C), generator=gen, device="cuda").to(dtype)
    for _ in range(warmup):
        runner.run_step(x)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        runner.run_step(x)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    nova.profile_stages(range(len(STAGES)))
    for _ in range(reps):
        runner.run_step(x)
    torch.cuda.synchronize()
    nova.profile_stages([])
    work = [stage_work(wl, scale, k) for k in ks]
    t = {}
    for si, name in enumerate(STAGES):
        t[name], _ = nova.profile_collect(si)
    tot = lambda name: sum(w[name][1] for w in work) * reps
    gemms = ("qkv", "oproj", "ffn1", "ffn2")
    kept = wl.B * sum(ks)
    res = {"grid": scale.grid, "kv_len": scale.kv_len, "kept_tokens_per_step": kept, "ms_per_step": round(ms, 3),
           "kept_tokens_per_s": round(kept / (ms * 1e-3)),
           "attention_frac_mfma_peak": round(tot("attention") / (t["attention"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
           "gemm_frac_mfma_peak": round(sum(tot(g) for g in gemms) / (sum(t[g] for g in gemms) * 1e-3) / 1e12
                                        / MFMA_BF16_PEAK_TFLOPS, 4),
           "entropy_frac_hbm_peak": round(tot("entropy") / (t["entropy"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "merge_frac_hbm_peak": round(tot("merge") / (t["merge"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "stage_ms_per_step": {n: round(v / reps, 3) for n, v in t.items()}}
    del runner, x
    torch.cuda.empty_cache()
    return res


def image_chain(nova, wl, weights, gen):
    """All scales of the workload's grid list for one batch of images: dense up to the scale before the
    first pruned one (which also builds the residual caches), then the pruned scales with the workload's
    keep table.  Inputs of every scale (hidden states, logits) are generated on the device beforehand."""
    import torch
    import workloads as WL
    from paper_2602_01345_amd.image import ImageRunner
    grids = WL.grid_list(wl)
    first_pruned = grids.index(wl.scales[0].grid)
    dtype = WL.torch_dtype(wl.dtype)
    runner = ImageRunner(nova, B=wl.B, C=wl.C, heads=wl.heads, grids=grids, dtype=dtype, weights=weights,
                         ffn_mult=wl.ffn_mult)
    xs = [torch.randn((wl.B, g * g, wl.C), generator=gen, device="cuda").to(dtype) for g in grids]
    # logits of the pruned scales (one tensor per block); the dense scales need none
    logits = {}
    for t in range(first_pruned, len(grids)):
        N = grids[t] * grids[t]
        logits[t] = [(torch.randn((wl.B, N, wl.V), generator=gen, device="cuda") * 3.0).to(dtype) for _ in range(wl.L)]
    tables = {t: [WL.keep_count(wl.keep_ratio(j), grids[t] * grids[t]) for j in range(wl.L)]
              for t in range(first_pruned, len(grids))}

    plans = runner.plan_image(tables, logits, first_cache_scale=first_pruned - 1)
    for p, x in zip(plans, xs):
        p.x.copy_(x)
    del xs

    def time_image(reps):
        ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in grids]
              for _ in range(reps)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(reps):
            for t, p in enumerate(plans):
                ev[r][t][0].record()
                runner.launch(p)
                ev[r][t][1].record()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        per_scale = [round(sum(ev[r][t][0].elapsed_time(ev[r][t][1]) for r in range(reps)) / reps, 3)
                     for t in range(len(grids))]
        return ms, per_scale

    time_image(1)                                        # warm-up, launches issued one by one
    eager_ms, eager_scales = time_image(2)
    for p in plans:
        runner.capture(p)                                # one HIP graph per scale
    time_image(1)
    graph_ms, graph_scales = time_image(3)
    return {"grids": grids, "first_pruned_grid": grids[first_pruned],
            "ms_per_image": round(graph_ms / wl.B, 3), "ms_per_batch": round(graph_ms, 3), "ms_per_scale": graph_scales,
            "launched_one_by_one": {"ms_per_batch": round(eager_ms, 3), "ms_per_scale": eager_scales},
            "note": "one HIP graph per scale; dense scales keep every token; pruned scales use the workload's "
                    "keep table; synthetic inputs"}


def variant_step(nova, runner, wl, x, gen, dtype, steps):
    """The same step with every block variant switched on (inputs drawn on the device; timing only), and the
    merge kernel of the middle block with each interpolation kernel."""
    import torch
    from paper_2602_01345_amd import BlockVariant, pack_k_cache, pack_v_cache
    Lt, cap_t = 77, 128
    rnd = lambda shape, std: (torch.randn(shape, generator=gen, device="cuda") * std).to(dtype)
    res = {"variants": f"modulation+gates, unit-length q/k, tanh GELU, cross-attention over {Lt} condition tokens"}

    def timed_step():
        for _ in range(2):
            runner.run_step(x)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            runner.run_step(x)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    res["base_ms_per_step"] = round(timed_step(), 3)
    # a model with unit-length queries and keys holds unit-length keys in its cache: the prior rows are rescaled
    # for this measurement and put back afterwards (un-normalised keys times the per-head multiplier would make
    # the scores tens of nats wide, which no such model produces)
    P = runner.kv_len
    saved = []
    for st in runner.blocks:
        prior = st.k_cache[:, :, :P, :]
        saved.append(prior.clone())
        prior.copy_(torch.nn.functional.normalize(prior.to(torch.float32), dim=-1).to(dtype))
    for st in runner.blocks:
        ada = rnd((wl.B, 6, wl.C), 0.2)
        ada[:, 2] += 1.0
        ada[:, 5] += 1.0
        cross = {"w_cq": rnd((wl.C, wl.C), 0.02), "b_cq": rnd((wl.C,), 0.02), "w_co": rnd((wl.C, wl.C), 0.02),
                 "b_co": rnd((wl.C,), 0.02), "text_len": Lt,
                 "k_text": pack_k_cache(rnd((wl.B, Lt, wl.C), 1.0), wl.heads, cap_t),
                 "v_text": pack_v_cache(rnd((wl.B, Lt, wl.C), 1.0), wl.heads, cap_t)}
        st.variant = BlockVariant(gelu_tanh=True, qk_scale=torch.rand(wl.heads, generator=gen, device="cuda") * 12 + 4,
                                  ada=ada, cross=cross)
    res["ms_per_step"] = round(timed_step(), 3)
    for st, prior in zip(runner.blocks, saved):
        st.variant = None
        st.k_cache[:, :, :P, :].copy_(prior)
    del saved
    s, st = wl.last, runner.blocks[len(runner.blocks) // 2]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for interp, name in ((0, "bilinear"), (1, "nearest"), (2, "bicubic")):
        run = lambda: nova.merge_cache_interp(interp, s.grid, s.grid, s.prev_grid, s.prev_grid, st.k, x, st.y_kept,
                                              st.kept_idx, st.keep_mask, st.cache_prev, st.out, st.cache_new)
        for _ in range(5):
            run()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(20):
            run()
        e1.record()
        torch.cuda.synchronize()
        res[f"merge_{name}_us"] = round(e0.elapsed_time(e1) * 1e3 / 20, 2)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg5", help="cfg2..cfg5 (default: the largest, cfg5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stage-pass", action="store_true")
    ap.add_argument("--overlap", action="store_true",
                    help="run entropy + selection of the next block on a second stream next to the current block's "
                         "gather and QKV projection (default: every kernel on one stream)")
    ap.add_argument("--no-image", action="store_true",
                    help="skip the chained multi-scale run (all scales of the config's grid list, ms per image)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the compact measurements of the other workloads' last scales and of this workload's "
                         "earlier pruned scales")
    ap.add_argument("--variants", action="store_true",
                    help="also time the step with the block variants on (modulation and gates, unit-length q/k, "
                         "tanh GELU, a cross-attention sub-layer over 77 condition tokens) and the other "
                         "cache interpolation kernels")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (known HBM traffic) for scaling rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as WL
    from paper_2602_01345_amd import Nova
    from paper_2602_01345_amd.binding import STAGES
    from paper_2602_01345_amd.step import StepRunner
    sys.path.insert(0, os.path.join(ROOT, "tests"))

    wl = WL.WORKLOADS[args.config]
    scale = wl.last
    dtype = WL.torch_dtype(wl.dtype)
    cap = wl.kv_capacity(scale)
    nova = Nova(0)
    runner = StepRunner(nova, B=wl.B, grid=scale.grid, prev_grid=scale.prev_grid, C=wl.C, heads=wl.heads,
                        kv_len=scale.kv_len, kv_capacity=cap, dtype=dtype, ffn_mult=wl.ffn_mult)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.seed)
    ks = wl.k_table(scale)

    # block 0 from the host generators (shared with the oracle), the rest drawn on the device
    from dataclasses import dataclass

    @dataclass
    class _HB:
        logits: object; x: object; weights: object; k_prior: object; v_prior: object; cache_prev: object
    kp, vp = WL.make_kv_prior(wl, 0, scale)
    hb0 = _HB(WL.make_logits(wl, 0, scale), WL.make_x(wl, scale), WL.make_weights(wl, 0), kp, vp,
              WL.make_cache_prev(wl, 0, scale))
    for j in range(wl.L):
        runner.add_block(device_block(wl, scale, j, ks[j], gen, dtype, cap, hb0 if j == 0 else None))
    x = hb0.x.cuda()
    torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB per launch
        torch.cuda.synchronize()
        del src, dst

    dom = STAGES.index("attention")
    overlap = args.overlap
    for _ in range(args.warmup):
        runner.run_step(x, overlap_selection=overlap)
    torch.cuda.synchronize()

    nova.profile_stages([dom])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        runner.run_step(x, overlap_selection=overlap)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    nova.profile_stages([])
    dom_ms, dom_n = nova.profile_collect(dom)

    ms_step = dt / args.steps * 1e3
    kept = wl.B * sum(ks)
    work = [stage_work(wl, scale, k) for k in ks]
    dom_flops = sum(w["attention"][1] for w in work) / len(work)          # per launch
    dom_avg_s = dom_ms / max(dom_n, 1) * 1e-3
    achieved = dom_flops / dom_avg_s / 1e12 if dom_avg_s > 0 else 0.0

    kernels = {}
    if not args.no_stage_pass:
        nova.profile_stages(range(len(STAGES)))
        reps = max(2, min(args.steps, 5))
        for _ in range(reps):
            runner.run_step(x, overlap_selection=False)      # one kernel at a time: clean per-kernel durations
        torch.cuda.synchronize()
        nova.profile_stages([])
        for si, name in enumerate(STAGES):
            ms, n = nova.profile_collect(si)
            if n == 0:
                continue
            kind, _ = work[0][name]
            total = sum(w[name][1] for w in work) * reps
            rate = total / (ms * 1e-3)
            ent = {"ms_per_step": ms / reps, "launches_per_step": n // reps}
            if kind == "bytes":
                ent["GB/s"] = rate / 1e9
                ent["frac_hbm_peak"] = rate / 1e9 / HBM_PEAK_GBS
            else:
                ent["TFLOP/s"] = rate / 1e12
                ent["frac_mfma_peak"] = rate / 1e12 / MFMA_BF16_PEAK_TFLOPS
            kernels[name] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in ent.items()}

    # sustained HBM rate of the bandwidth-bound calls: the L blocks' launches back to back under one
    # pair of events (an isolated 60 MB launch is dominated by launch ramp; a plain read kernel of
    # that size behaves the same), every launch on its own, distinct tensors
    hbm = {}
    if not args.no_stage_pass:
        def sustained(name, fn):
            fn()                                   # warm the code path
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            total = sum(w[name][1] for w in work)
            hbm[name] = {"us_per_launch": round(ms * 1e3 / len(work), 2), "GB/s": round(total / (ms * 1e-3) / 1e9, 1),
                         "frac_hbm_peak": round(total / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        blocks = runner.blocks
        sustained("entropy", lambda: [nova.entropy(st.logits, st.entropy) for st in blocks])
        if wl.dtype == "bf16":
            # the same kernel on fp32 logits (twice the bytes, the same arithmetic)
            f32 = [(torch.randn((wl.B, scale.N, wl.V), generator=gen, device="cuda") * 3.0) for _ in range(8)]
            Hs = [torch.empty((wl.B, scale.N), dtype=torch.float32, device="cuda") for _ in f32]
            work_f32 = [{"entropy_f32": ("bytes", wl.B * scale.N * (wl.V * 4 + 4))}] * len(f32)
            keep, work = work, work_f32
            sustained("entropy_f32", lambda: [nova.entropy(a, h) for a, h in zip(f32, Hs)])
            work = keep
            del f32, Hs
        sustained("select", lambda: [nova.select(st.entropy, st.k, st.kept_idx, st.keep_mask) for st in blocks])
        # entropy and selection as the step issues them, one after the other per block: the pair's rate over the
        # bytes of both (selection alone is latency: tens of kilobytes per launch)
        for w in work:
            w["entropy_select_pair"] = ("bytes", w["entropy"][1] + w["select"][1])
        sustained("entropy_select_pair", lambda: [(nova.entropy(st.logits, st.entropy),
                                                   nova.select(st.entropy, st.k, st.kept_idx, st.keep_mask))
                                                  for st in blocks])
        sustained("merge", lambda: [nova.merge_cache(scale.grid, scale.grid, scale.prev_grid, scale.prev_grid, st.k, x,
                                                     st.y_kept, st.kept_idx, st.keep_mask, st.cache_prev, st.out,
                                                     st.cache_new) for st in blocks])

        # the selector's own throughput, which B = 2 images cannot show: 4096 rows of 4096 entropies, half kept
        # (one workgroup per row; read 4N, write 4k + N bytes per row)
        sB, sN, sk = 4096, 4096, 2048
        sH = torch.rand((sB, sN), generator=gen, device="cuda") * 8.0
        sidx = torch.empty((sB, sk), dtype=torch.int32, device="cuda")
        smask = torch.empty((sB, sN), dtype=torch.uint8, device="cuda")
        for _ in range(2):
            nova.select(sH, sk, sidx, smask)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            nova.select(sH, sk, sidx, smask)
        e1.record()
        torch.cuda.synchronize()
        s_us = e0.elapsed_time(e1) * 1e3 / 5
        s_bytes = sB * (4 * sN + 4 * sk + sN)
        hbm["select_stress"] = {"shape": f"B={sB} rows of N={sN}, k={sk}", "us_per_launch": round(s_us, 1),
                                "GB/s": round(s_bytes / (s_us * 1e-6) / 1e9, 1),
                                "frac_hbm_peak": round(s_bytes / (s_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                "rows_per_s": round(sB / (s_us * 1e-6))}
        del sH, sidx, smask

        # the layer-linkage ratio kernel sits between entropy and select: a latency-bound launch
        # (B rows), reported as time per launch over one launch per block
        cm = torch.rand(wl.B, device="cuda") * 5.0 + 1.0
        cs = torch.zeros(wl.B, device="cuda")
        cr = torch.full((wl.B,), 0.5, device="cuda")
        co = torch.empty(wl.B, device="cuda")
        ck = torch.empty(wl.B, dtype=torch.int32, device="cuda")
        run_ratio = lambda: [nova.layer_ratio(cm, cs, cr, j + 1, scale.N, co, ck) for j in range(len(blocks))]
        run_ratio()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run_ratio()
        e1.record()
        torch.cuda.synchronize()
        hbm["layer_ratio"] = {"us_per_launch": round(e0.elapsed_time(e1) * 1e3 / len(blocks), 2), "bound": "latency"}

        # entropy straight from a linear head of the workload's width: logits never reach HBM (bf16 kernel only)
        if dtype == torch.bfloat16:
            hh = torch.randn((wl.B, scale.N, wl.C), generator=gen, device="cuda").to(dtype)
            hw = (torch.randn((wl.V, wl.C), generator=gen, device="cuda") * 0.02).to(dtype)
            hH = torch.empty((wl.B, scale.N), dtype=torch.float32, device="cuda")
            hws = torch.empty(nova.head_entropy_workspace_bytes(scale.N, wl.B, wl.V), dtype=torch.uint8, device="cuda")
            reps = 8
            run_head = lambda: [nova.head_entropy(hh, hw, None, hH, hws) for _ in range(reps)]
            run_head()
            torch.cuda.synchronize()
            e0.record()
            run_head()
            e1.record()
            torch.cuda.synchronize()
            hus = e0.elapsed_time(e1) * 1e3 / reps
            hfl = 2.0 * wl.B * scale.N * wl.C * wl.V
            hbm["head_entropy"] = {"us_per_launch": round(hus, 2), "TFLOP/s": round(hfl / (hus * 1e-6) / 1e12, 1),
                                   "frac_mfma_peak": round(hfl / (hus * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                                   "bound": "mfma", "logits_bytes_not_written": wl.B * scale.N * wl.V * 2}
            del hh, hw, hH, hws

    # The attention kernel's time depends mildly on the scores (its softmax reference point moves only when a score
    # lies far above it): the workload's weights give near-uniform scores, the favourable case.  The same step with
    # the query projections scaled up 16-fold (scores tens of nats wide, peaked attention) is timed for comparison.
    wide = None
    if not args.no_stage_pass and wl.dtype == "bf16":
        C = wl.C
        for st in runner.blocks:
            st.weights["w_qkv"][:C] *= 16.0
            st.weights["b_qkv"][:C] *= 16.0
        nova.profile_stages([dom])
        for _ in range(2):
            runner.run_step(x)
        torch.cuda.synchronize()
        nova.profile_stages([])
        w_ms, w_n = nova.profile_collect(dom)
        for st in runner.blocks:
            st.weights["w_qkv"][:C] /= 16.0            # powers of two: the bf16 weights come back bit for bit
            st.weights["b_qkv"][:C] /= 16.0
        w_avg_s = w_ms / max(w_n, 1) * 1e-3
        wide = {"achieved": dom_flops / w_avg_s / 1e12, "avg_launch_us": w_avg_s * 1e6,
                "frac": dom_flops / w_avg_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                "note": "query projection scaled 16-fold: scores tens of nats wide, the softmax reference moves often"}

    # what the chip sustains for plain kernels (published peaks: HBM 8 TB/s, dense bf16 MFMA 2.5 PFLOP/s)
    peaks = {}
    if not args.no_stage_pass:
        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            work = 0.0
            for _ in range(reps):
                work += fn()
            b.record()
            torch.cuda.synchronize()
            return work / (a.elapsed_time(b) * 1e-3)
        sink = torch.zeros(1, device="cuda")
        big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")      # 1 GiB: four times the infinity cache
        big.fill_(1)
        big2 = torch.empty_like(big)
        peaks["hbm_read_GBs"] = round(timed(lambda: nova.probe(0, big, None, 1, sink), 5) / 1e9, 1)
        peaks["hbm_copy_GBs"] = round(timed(lambda: nova.probe(1, big, big2, 1, sink), 5) / 1e9, 1)
        peaks["mfma_bf16_TFLOPs"] = round(timed(lambda: nova.probe(2, None, None, 2000, sink), 3) / 1e12, 1)
        rnd = torch.randn(16 << 20, generator=gen, device="cuda").to(torch.bfloat16)      # N(0,1) operands, 32 MiB
        peaks["mfma_bf16_random_operands_TFLOPs"] = round(timed(lambda: nova.probe(3, rnd, None, 2000, sink), 3) / 1e12, 1)
        del rnd
        peaks["note"] = ("plain kernels of this library (nova_probe): 1 GiB streaming read, 1 GiB copy (read+write bytes), "
                         "MFMA-only loop on constant register operands, and the same loop on N(0,1) operands (more bits "
                         "switch per MFMA: more power, lower clock)")
        del big, big2

    traffic = None
    tf = os.path.join(ROOT, "profiles", f"attention_{args.config}_hbm_traffic.txt")
    if os.path.exists(tf):
        for line in open(tf):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])

    out = {
        "metric": METRIC, "value": kept / (ms_step * 1e-3), "unit": "kept tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: last scale {scale.grid}x{scale.grid}, B={wl.B}, C={wl.C}, heads={wl.heads}, "
                               f"L={wl.L}, V={wl.V}, P={scale.kv_len}, keep {wl.keep_hi}->{wl.keep_lo}",
                   "kept_tokens_per_step": kept, "blocks": wl.L,
                   "streams": "2 (selection of block j+1 next to the matrix kernels of block j)" if overlap else "1"},
        "roofline": {"kernel": f"attention_bf16_kernel<{wl.dh},...> (+ its split-merge pass)", "bound": "mfma",
                     "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "launches": dom_n,
                     "avg_launch_us": dom_avg_s * 1e6, "flops_per_launch": dom_flops,
                     "scores": "near-uniform (weights N(0, 0.02^2)): the favourable case for the lazy softmax reference",
                     "frac_wide_scores": None if wide is None else wide["frac"], "wide_scores": wide},
        "kernels": kernels,
        "hbm_kernels_sustained": hbm,
        "achievable_peaks": peaks,
    }
    if args.variants:
        out["variant_step"] = variant_step(nova, runner, wl, x, gen, dtype, args.steps)
    if not args.no_image and not args.no_stage_pass:
        out["image_chain"] = image_chain(nova, wl, [st.weights for st in runner.blocks], gen)
    if not args.no_other_configs and not args.no_stage_pass and args.config == "cfg5":
        # the other workloads' last scales and this workload's earlier pruned scales, a few steps each
        del runner, x
        torch.cuda.empty_cache()
        other = {}
        for name in ("cfg2", "cfg3", "cfg4"):
            w2 = WL.WORKLOADS[name]
            other[name] = compact_config(nova, w2, w2.last)
        for sc in wl.scales[:-1]:
            other[f"cfg5@{sc.grid}x{sc.grid}"] = compact_config(nova, wl, sc)
        out["other_configs"] = other
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(hb0, wl, scale, ks)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
