#!/usr/bin/env python3
"""Benchmark of the L2A conditional-attention layer on one MI355X.

A step is one pass of the whole hot path -- l2a_route_compact, l2a_attn_fwd, l2a_attn_bwd --
over one synthetic batch that is already resident in HBM.  The default workload is the one the
headline metric is quoted on: the training-step shape (Hq=28, Hkv=4, D=128, W=4096) at
T=131072 with 80 % of the tokens skipping Global attention (per-head i.i.d. routing).
The same kernels' dense all-routed mode is timed next to it (the FlashAttention-style baseline).

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: this build is
single-GPU by design.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak

# HBM-side bytes per launch of each matrix-core kernel on the default workload (train_128k, seed 0,
# forward + backward), from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE, KiB per
# dispatch) scaled by what the same counters read for a plain 1 GiB device copy (--calibrate-copy):
# FETCH x 2.0, WRITE x 1.0.  The counters cannot be read from inside the process, so the figures of the
# committed profile are repeated here; they are reported only for exactly that workload.
TRAFFIC_SOURCE = ("NOT measured in this run: constant copied from profiles/all_kernels_train_128k_hbm_bytes.md, two "
                  "rocprofv3 --pmc runs of `bench.py --sparse-only --calibrate-copy` on the same workload")
MEASURED_TRAFFIC_BYTES = {"bwd_dkdv": 1.564e10, "bwd_dq_global": 2.966e10, "bwd_dq_local": 4.25e9,
                          "fwd_global": 2.646e10, "fwd_local": 5.44e9}


def pair_counts(mask: np.ndarray, Hq: int, Hkv: int, T: int, W: int, dense: bool):
    """(row, key) pairs each branch must score: global = sum over routed (head, t) of t+1,
    local = Hq * sum_t min(t+1, W+1).  Exact, from the mask."""
    t1 = np.arange(1, T + 1, dtype=np.float64)
    local = float(Hq) * float(np.minimum(t1, W + 1).sum())
    if dense:
        glob = float(Hq) * float(t1.sum())
        frac = 1.0
    else:
        rep = Hq // mask.shape[1]
        per = (mask != 0).astype(np.float64) @ t1               # [B, Hm]
        glob = float(per.sum()) * rep
        frac = float((mask != 0).mean())
    return local, glob, frac


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="train_128k")
    ap.add_argument("--fraction", type=float, default=None, help="override the routed fraction")
    ap.add_argument("--seq-len", type=int, default=None, help="override the workload's sequence length T")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-dense", action="store_true", help="skip timing the dense all-routed mode")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-step measurement")
    ap.add_argument("--sparse-only", action="store_true",
                    help="no routed-only pass, dense mode, short-context leg or CPU oracle: every launch of the layer's kernels that a "
                         "profiler sees then belongs to the timed workload (the router and decode kernels, measured "
                         "separately, have names of their own)")
    ap.add_argument("--graph", action="store_true",
                    help="time the sparse layer's step as replays of one captured HIP graph (removes the host's launch "
                         "gaps, which matter below ~16K tokens); the per-kernel durations still come from eager steps")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of 1 GiB (a known-size kernel to scale profiler byte counters)")
    args = ap.parse_args()
    if args.sparse_only:
        args.no_dense = args.no_cpu = True
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2603_17484_amd import binding as B
    from paper_2603_17484_amd import inputs as gen
    from paper_2603_17484_amd.runner import Layer

    B.lib()  # fails loudly if the HIP library has not been built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = gen.workload(args.workload)
    over = {}
    if args.fraction is not None:
        over["routed_fraction"] = args.fraction
    if args.seq_len is not None:
        over["T"] = args.seq_len
    if over:
        w = gen.workload(args.workload, **over)
    backward = w.backward and not args.forward_only
    D, T = w.D, w.T

    # ---- synthetic inputs, generated on the device (N(0,1), bf16), mask on the host
    g = torch.Generator(device=dev)
    g.manual_seed(args.seed)
    mk = lambda *s: torch.randn(*s, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q, k, v = mk(w.B, T, w.Hq, D), mk(w.B, T, w.Hkv, D), mk(w.B, T, w.Hkv, D)
    dO = mk(w.B, T, w.Hq, D) if backward else None
    mask_np = gen.make_mask(w, args.seed)
    mask = torch.from_numpy(mask_np).to(dev)

    def build(flags):
        p = B.make_params(w.B, T, w.Hq, w.Hkv, D, w.W, w.mask_heads, B.L2A_BF16, flags)
        return Layer(p, q, k, v, mask)

    def step(lay):
        lay.route()
        lay.forward(save_branches=backward)
        if backward:
            lay.backward(dO)

    def timed(lay, steps, warmup, profile=False, graph=False):
        for _ in range(warmup):
            step(lay)
        torch.cuda.synchronize()
        if graph:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step(lay)
            torch.cuda.current_stream().wait_stream(side)
            cg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(cg):
                step(lay)
            cg.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                cg.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps, {}
        if profile:
            B.profile_read()
            B.profile_enable(True)
        # one event per step boundary on the launch stream (recording does not synchronise): the spread of the steps
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            step(lay)
            marks[i + 1].record()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        timed.per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
        kern = {}
        if profile:
            B.profile_enable(False)
            for name, t in B.profile_read():
                kern.setdefault(name, []).append(t)
        return ms, {n: float(np.mean(ts)) for n, ts in kern.items()}

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: K steps of the sparse layer
    # (the per-kernel HIP events cost a few microseconds per launch: they are recorded in a pass of their own)
    sparse = build(0)
    ms_sparse, _ = timed(sparse, args.steps, args.warmup)
    per_step = sorted(timed.per_step)
    _, kern = timed(sparse, max(1, min(args.steps, 5)), 0, profile=True)
    ms_eager = None
    if args.graph:
        ms_eager = ms_sparse
        ms_sparse, _ = timed(sparse, args.steps, 0, graph=True)
    pl, pg, frac = pair_counts(mask_np, w.Hq, w.Hkv, T, w.W, dense=False)
    mult = 14.0 if backward else 4.0          # fwd 4 D, bwd 10 D FLOPs per (row, key) pair
    flops_layer = mult * D * (pl + pg)
    flops_routed = mult * D * pg
    tflops_layer = flops_layer / (ms_sparse * 1e-3) / 1e12

    # ---- router front-end on the Local branch's output viewed as [B, T, Hq*D]: an HBM-bound pass
    router = None
    if True:
        C = w.Hq * D
        xr = (sparse.S if backward else sparse.O).view(w.B, T, C)
        wr = torch.randn(C, generator=g, device=dev, dtype=torch.float32) / C ** 0.5
        rmask = torch.empty((w.B, 1, T), dtype=torch.uint8, device=dev)
        rdhat = torch.empty((w.B, T), dtype=torch.float32, device=dev)
        for _ in range(2):
            B.l2a_router_decide(sparse.p, xr, wr, 0.0, 0.5, rmask, rdhat)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            B.l2a_router_decide(sparse.p, xr, wr, 0.0, 0.5, rmask, rdhat)
        e1.record()
        torch.cuda.synchronize()
        ms_r = e0.elapsed_time(e1) / 10
        nbytes = w.B * T * C * 2 + w.B * T * 5 + C * 4          # x once, mask + score out, w
        router = {"ms": round(ms_r, 4), "bytes": nbytes, "achieved_GBps": round(nbytes / ms_r / 1e6, 1),
                  "peak_GBps": 8000.0, "frac": round(nbytes / ms_r / 1e6 / 8000.0, 4), "bound": "hbm",
                  "input": f"[{w.B},{T},{C}] bf16"}
        del rmask, rdhat, wr

    # ---- decode step (Sec. 3.4) on a batch of sequences with full-length caches: an HBM-bound pass
    decode = short = None
    if not args.no_decode:
        decode = decode_leg(torch, B, w, dev, g)
        if not args.sparse_only:   # its launches carry the layer's kernel names: kept out of profiler runs
            short = short_context_leg(torch, B, gen, Layer, dev, g)

    # ---- global branch alone (routed FLOPs only)
    ms_glob = tflops_routed = None
    if not args.sparse_only:
        glob = build(B.L2A_FLAG_SKIP_LOCAL)
        ms_glob, _ = timed(glob, max(1, min(args.steps, 3)), 1)
        del glob
        tflops_routed = flops_routed / (ms_glob * 1e-3) / 1e12

    # ---- dense all-routed mode of the same kernels
    ms_dense = None
    if not args.no_dense:
        dense = build(B.L2A_FLAG_DENSE)
        ms_dense, _ = timed(dense, max(1, min(args.steps, 5)) if T > 32768 else args.steps, 1)
        ms_dense_graph = None
        if args.graph:
            ms_dense_graph, _ = timed(dense, args.steps, 0, graph=True)
        _, kern_dense = timed(dense, 1, 0, profile=True)
        del dense
        _, pg_dense, _ = pair_counts(mask_np, w.Hq, w.Hkv, T, w.W, dense=True)

    # ---- roofline of the dominant kernel (live HIP-event durations over the timed region)
    alg = {  # algorithmic FLOPs per launch; the backward's 10 D per pair = 8 D (S, dP, dV, dK) + 2 D (dQ)
        "fwd_local": 4.0 * D * pl, "fwd_global": 4.0 * D * pg,
        "bwd_dq_local": 2.0 * D * pl, "bwd_dq_global": 2.0 * D * pg,
        "bwd_dkdv": 8.0 * D * (pl + pg),
        "fwd_pair": 4.0 * D * (pl + pg),   # short sequences: both branches of the forward in one launch
    }
    dom = max((n for n in kern if n in alg), key=lambda n: kern[n])
    achieved = alg[dom] / (kern[dom] * 1e-3) / 1e12
    default_workload = (args.workload == "train_128k" and not over and args.seed == 0 and backward)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(dom) if default_workload else None,
                "traffic_unit": "HBM-side bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
                "traffic_source": (TRAFFIC_SOURCE if default_workload else None),
                "algorithmic_flops_per_launch": alg[dom], "avg_ms": round(kern[dom], 3)}

    # ---- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(w, q, k, v, dO, mask_np, backward, args.seed)

    out = {
        "metric": "L2A layer effective TFLOP/s (route_compact + fwd + bwd, T=131072, 80% of tokens skip Global)"
                  if args.workload == "train_128k" and not over else
                  f"L2A layer effective TFLOP/s ({w.name})",
        "value": round(tflops_layer, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_sparse, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "T": T, "Hq": w.Hq, "Hkv": w.Hkv, "D": D, "W": w.W,
                   "mask": f"{w.mask_kind}, mask_heads={w.mask_heads}", "routed_fraction_measured": round(frac, 4),
                   "passes": "fwd+bwd" if backward else "fwd", "seed": args.seed},
        "ms_layer": round(ms_sparse, 3),
        "ms_per_step_min": round(per_step[0], 3), "ms_per_step_median": round(float(np.median(per_step)), 3),
        "launch": "hip graph replay" if args.graph else "eager",
        "ms_layer_eager": None if ms_eager is None else round(ms_eager, 3),
        "frac_of_bf16_peak_layer": round(tflops_layer / PEAK_BF16_TFLOPS, 4),
        "routed": None if ms_glob is None else {
            "tflops": round(tflops_routed, 2), "frac_of_bf16_peak": round(tflops_routed / PEAK_BF16_TFLOPS, 4),
            "ms_global_branch_only": round(ms_glob, 3), "flops": flops_routed},
        "dense_mode": None if ms_dense is None else {
            "ms_layer": round(ms_dense, 3),
            "ms_layer_graph_replay": None if ms_dense_graph is None else round(ms_dense_graph, 3),
            "speedup_sparse_vs_dense": round((ms_dense_graph or ms_dense) / ms_sparse, 3),
            # the kernels that run on Global rows only (the dK/dV kernel walks both row sets in one launch)
            "speedup_global_kernels": {k: round(kern_dense[k] / kern[k], 3) for k in ("fwd_global", "bwd_dq_global")
                                       if kern.get(k) and kern_dense.get(k)},
            "tflops_layer": round(mult * D * (pl + pg_dense) / (ms_dense * 1e-3) / 1e12, 2),
            "kernels_ms": {n: round(t, 3) for n, t in kern_dense.items()}},
        "kernels_ms": {n: round(t, 3) for n, t in kern.items()},
        "roofline": roofline,
        "router_front_end": router,
        "decode_step": decode,
        "short_context_forward": short,
        "cpu_baseline": cpu,
        "paper_context": "paper reports ~10x fwd / ~8x bwd kernel speed-ups over FlashAttention-2 at 128K and up "
                         "to 90% sparsity on NVIDIA H200 (Fig. 1 caption, Sec. 4.2); not comparable hardware",
    }
    print(json.dumps(out))
    return 0


def short_context_leg(torch, B, gen, Layer, dev, g, T=4096, fraction=0.2, steps=50):
    """Forward at a short sequence length (App. D.1: the regime where preprocessing and launch
    overheads decide): Qwen2.5-7B head layout, shared Bernoulli mask; the sparse step eager and as a
    HIP graph replay, and the dense mode of the same kernels."""
    w = gen.workload("qwen25_7b_32k", T=T, routed_fraction=fraction)
    mk = lambda *s: torch.randn(*s, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q, k, v = mk(w.B, T, w.Hq, w.D), mk(w.B, T, w.Hkv, w.D), mk(w.B, T, w.Hkv, w.D)
    mask = torch.from_numpy(gen.make_mask(w, 0)).to(dev)

    def timed(flags, graph):
        lay = Layer(B.make_params(w.B, T, w.Hq, w.Hkv, w.D, w.W, w.mask_heads, B.L2A_BF16, flags), q, k, v, mask)

        def step():
            lay.route()
            lay.forward(save_branches=False)
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        run = step
        if graph:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            cg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(cg):
                step()
            run = cg.replay
            run()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    sparse_eager, sparse_graph = timed(0, False), timed(0, True)
    dense_eager, dense_graph = timed(B.L2A_FLAG_DENSE, False), timed(B.L2A_FLAG_DENSE, True)
    return {"workload": f"qwen25_7b layout, T={T}, W={w.W}, routed fraction {fraction}, forward",
            "ms_sparse_eager": round(sparse_eager, 4), "ms_sparse_graph_replay": round(sparse_graph, 4),
            "ms_dense_eager": round(dense_eager, 4), "ms_dense_graph_replay": round(dense_graph, 4),
            "dense_over_sparse_eager": round(dense_eager / sparse_eager, 3),
            "dense_over_sparse_graph": round(dense_graph / sparse_graph, 3)}


def decode_leg(torch, B, w, dev, g, batch=8):
    """One decode step for `batch` sequences whose caches hold T tokens each: every sequence routed, and
    one in four routed.  Algorithmic bytes: each K and V row in reach once per branch that runs."""
    T, D = w.T, w.D
    mk = lambda *s: torch.randn(*s, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    kc, vc, qn = mk(batch, T, w.Hkv, D), mk(batch, T, w.Hkv, D), mk(batch, w.Hq, D)
    pos = torch.full((batch,), T - 1, dtype=torch.int32, device=dev)
    p = B.make_params(batch, T, w.Hq, w.Hkv, D, w.W, 1)
    O = torch.empty((batch, w.Hq, D), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(B.lib().l2a_decode_workspace_bytes(__import__("ctypes").byref(p)), dtype=torch.uint8, device=dev)
    out = {"batch": batch, "cache_tokens": T, "peak_GBps": 8000.0, "bound": "hbm"}
    row_bytes = w.Hkv * D * 2 * 2   # K and V
    for name, routed in (("all_routed", batch), ("one_in_four_routed", batch // 4)):
        d = torch.zeros((batch, 1), dtype=torch.uint8, device=dev)
        d[:routed] = 1
        run = lambda: B.l2a_attn_decode(p, qn, kc, vc, pos, d, O, workspace=ws)
        for _ in range(3):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 20
        nbytes = (batch * (w.W + 1) + routed * T) * row_bytes
        out[name] = {"ms": round(ms, 4), "bytes": nbytes, "achieved_GBps": round(nbytes / ms / 1e6, 1),
                     "frac": round(nbytes / ms / 1e6 / 8000.0, 4)}
    return out


def cpu_baseline(w, q, k, v, dO, mask_np, backward, seed, budget_s=15.0):
    """The CPU oracle, as it stands, on sampled routed rows of the same tensors: forward of both
    branches plus the dQ pass.  No dK/dV pass is run (a key's gradient needs the statistics of every
    row that can see it, i.e. a forward over most of the sequence).  Rate in algorithmic FLOPs of what the
    sample produces -- 4 D per (row, key) pair for the forward, 4 D for dP and dQ -- so the unit matches
    `value`; the scores the dQ pass recomputes are not counted."""
    import torch
    from oracle import l2a_oracle as orc
    orc.build()
    f32 = lambda t: t.detach().to(torch.float32).cpu().numpy()
    pr = orc.Problem(f32(q), f32(k), f32(v), mask_np, w.W)
    g = f32(dO) if backward else None
    rng = np.random.default_rng(seed + 12345)
    routed = np.argwhere(pr.mask_per_head())        # (b, h, t)
    if routed.shape[0] == 0:
        return None

    def run(rows):
        t0 = time.perf_counter()
        orc.fwd_rows(pr, rows)
        if backward:
            orc.bwd_dq_rows(pr, g, rows)
        dt = time.perf_counter() - t0
        t = rows[:, 2].astype(np.float64)
        pairs = float((t + 1).sum() + np.minimum(t + 1, w.W + 1).sum())
        return dt, pairs

    pick = lambda n: routed[rng.choice(routed.shape[0], size=min(n, routed.shape[0]), replace=False)].astype(np.int32)
    run(pick(32))                       # thread start-up, page faults
    dt, pairs = run(pick(256))
    n = int(max(256, min(40000, 256 * budget_s / max(dt, 1e-3))))
    dt, pairs = run(pick(n))
    per_pair = (8.0 if backward else 4.0) * w.D
    threads = orc.threads()
    return {"value": round(per_pair * pairs / dt / 1e12, 6), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} routed rows drawn uniformly: oracle forward (local+global) "
                      f"{'and dQ pass ' if backward else ''}over {pairs:.3e} (row,key) pairs in {dt:.1f} s; "
                      f"{'no dK/dV pass is run; ' if backward else ''}valued at {per_pair / w.D:.0f} D FLOP per pair "
                      f"(forward 4 D{', dP and dQ 4 D' if backward else ''})",
            "ns_per_row_key_pair": round(dt * 1e9 / pairs, 3)}


if __name__ == "__main__":
    sys.exit(main())
