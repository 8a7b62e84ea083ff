#!/usr/bin/env python3
"""Benchmark of the FlatParameter data path on one MI355X.

A step is one pass of the hot path over every FSDP unit of the workload, in
order: unshard (fp32 shards -> bf16 flat buffer, all W ranks' shards), then the
rank-0 share of the reduce-scatter over W simulated ranks' gradient buffers and
the sharded Adam step.  Inputs are synthetic, seeded, and resident in HBM before
the timed region starts.

Prints ONE JSON line:  metric = effective HBM GB/s (algorithmic bytes of
unshard + reduce-scatter + Adam, summed over the units, per second).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GRAPH_MIN_LAUNCHES = 16      # steps with more launches than this are captured in a HIP graph by default
HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=1, help="workload: 0 one GPT-2-small block, 1 full GPT-2-small (default), 2 1.3B blocks W=12, "
                         "3 Llama-7B blocks W=64, 4 one GPT-3-175B block W=16")
    ap.add_argument("--max-units", type=int, default=0, help="limit the number of units (0 = all)")
    ap.add_argument("--depth", type=int, default=0,
                    help="units per batch in --mode batch (prefetch depth); 0 = 6 when the units are small enough to "
                         "share grids (launch-bound), 1 when they are not (then only the pairing of unit i's update "
                         "with unit i+1's unshard matters)")
    ap.add_argument("--mode", choices=["batch", "prefetch", "fused", "separate", "lp", "batch-lp"], default="batch",
                    help="batch: the updates of `depth` units and the prefetched unshards of the next `depth` units "
                         "are independent and share one launch (fsdp_batch_*); "
                         "prefetch: unit i's fused reduce-scatter+Adam shares one launch with unit i+1's unshard "
                         "(backward prefetching); fused: reduce-scatter + Adam in one launch, unshard in another; "
                         "separate: the three required entry points, one launch each; lp: every rank keeps a bf16 "
                         "copy of its shard (written by the fused Adam), the unshard gathers bf16 (Sec. 4.4); "
                         "batch-lp: the same hand-off issued as batches (moves 4P instead of 6P per unshard; the "
                         "metric's numerator stays the fixed 6P)")
    ap.add_argument("--graph", action="store_true", help="always replay the step as a HIP graph")
    ap.add_argument("--no-graph", action="store_true", help="always launch eagerly")
    ap.add_argument("--probe-copy", type=int, default=0, metavar="N",
                    help="run only N launches of a plain 256 MiB copy kernel (calibrates rocprofv3 --pmc byte counters)")
    ap.add_argument("--next-rows", action="store_true",
                    help="measure the kernels beyond the hot path (hybrid-sharding reduce, gradient accumulation) "
                         "on the workload's largest unit and print their own JSON line")
    ap.add_argument("--unit-scale", type=int, default=1,
                    help="size study: every unit holds this many copies of its parameter list")
    ap.add_argument("--raf", action="store_true",
                    help="reshard after forward (Sec. 3, Sec. 4.4): every unit is unsharded twice per step, once for "
                         "the forward pass and once before its backward; the metric's bytes count both")
    ap.add_argument("--grad-dtype", choices=["f32", "bf16"], default=None,
                    help="override the workload's gradient dtype (the fp32 / bf16 variants of every configuration)")
    ap.add_argument("--walk", choices=["auto", "wide", "deep"], default="auto",
                    help="rank walk of the stand-alone reduce-scatter kernels (fsdp_set_reduce_walk)")
    ap.add_argument("--grad-sets", type=int, default=0,
                    help="cap the number of distinct sets of gradient buffers per unit shape (0 = as many as fit)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="rocprofv3 --pmc derived HBM bytes per launch (written by hand from profiles/)")
    return ap.parse_args()


class UnitState:
    """Device buffers of one FSDP unit (caller-owned, as the library expects)."""

    def __init__(self, F, wl, unit, index, torch, workloads, share_grads_with=None):
        W = wl.world_size
        self.name = unit.name
        self.lay = F.fsdp_layout_init(unit.shapes, W)
        S, P, N = self.lay.shard, self.lay.padded, self.lay.numel
        self.S, self.P, self.N, self.W = S, P, N, W
        self.gbytes = 4 if wl.grad_dtype == "f32" else 2
        params = workloads.gen_params(unit, index, device="cuda")
        self.shard_base = torch.empty(W * S, dtype=torch.float32, device="cuda")
        self.shards = [self.shard_base[w * S:(w + 1) * S] for w in range(W)]
        F.fsdp_flatten_shard(self.lay, params, self.shards)
        del params
        gdt = torch.float32 if wl.grad_dtype == "f32" else torch.bfloat16
        if share_grads_with is not None:
            # HBM cannot hold W gradient buffers for every unit of the largest workloads:
            # units of equal shape then rotate over a few distinct sets of buffers.
            assert share_grads_with.P == P
            self.grads = share_grads_with.grads
        else:
            self.grads = []
            for w in range(W):
                g = torch.empty(P, dtype=gdt, device="cuda")
                workloads.gen_rank_grad(P, N, w, index, wl.grad_dtype, device="cuda", outlier_frac=wl.outlier_frac,
                                        outlier_scale=wl.outlier_scale, out=g)
                self.grads.append(g)
        self.m = torch.zeros(S, dtype=torch.float32, device="cuda")
        self.v = torch.zeros(S, dtype=torch.float32, device="cuda")
        self.gshard = torch.empty(S, dtype=torch.float32, device="cuda")
        self.shard_tab = F.PtrArray(self.shards)
        self.lp_base = torch.empty(W * S, dtype=torch.bfloat16, device="cuda")
        self.lp_shards = [self.lp_base[w * S:(w + 1) * S] for w in range(W)]
        for w in range(W):
            F.fsdp_cast_shard(self.lay, self.shards[w], self.lp_shards[w])
        self.lp_tab = F.PtrArray(self.lp_shards)
        self.grad_tab = F.PtrArray(self.grads)
        # algorithmic bytes (fixed numerators, whatever the kernels really touch)
        self.b_unshard = 6 * P
        self.b_reduce = self.gbytes * P + 4 * S
        self.b_adam = 28 * S
        self.b_total = self.b_unshard + self.b_reduce + self.b_adam


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build simulates all W ranks on ONE GPU; --gpus must be 1 "
              "(no multi-GPU figure exists for it)", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    from paper_2304_11277_amd import build as fbuild
    fbuild.build_lib(force=False)
    import paper_2304_11277_amd as F

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.probe_copy:
        probe_copy(args.probe_copy, torch, fbuild)
        return
    F.fsdp_set_reduce_walk({"auto": F.FSDP_WALK_AUTO, "wide": F.FSDP_WALK_WIDE, "deep": F.FSDP_WALK_DEEP}[args.walk])
    wl = workloads.config(args.config)
    if args.grad_dtype:
        import dataclasses
        wl = dataclasses.replace(wl, grad_dtype=args.grad_dtype)
    if args.next_rows:
        next_rows(args, wl, F, torch, workloads)
        return
    units = list(wl.units)
    if args.max_units:
        units = units[:args.max_units]
    if args.unit_scale > 1:
        units = [workloads.Unit(f"{u.name}x{args.unit_scale}", tuple(u.shapes) * args.unit_scale) for u in units]
    pre, post = F.fsdp_default_divide_factors(wl.world_size)
    t0 = time.time()
    states = []
    grad_budget = 160e9          # bytes of HBM given to the simulated ranks' gradient buffers
    used = 0.0
    for i, u in enumerate(units):
        share = None
        need = wl.world_size * sum(workloads.numel(s) for s in u.shapes) * (4 if wl.grad_dtype == "f32" else 2)
        same = [s for s in states if s.unit_shapes == u.shapes and s.owns_grads]
        if used + need > grad_budget or (args.grad_sets and len(same) >= args.grad_sets):
            share = same[len(states) % len(same)] if same else None
        st = UnitState(F, wl, u, i, torch, workloads, share_grads_with=share)
        st.unit_shapes, st.owns_grads = u.shapes, share is None
        used += need if share is None else 0
        states.append(st)
    flat = torch.empty(max(s.P for s in states), dtype=torch.bfloat16, device="cuda")   # transient, reused
    torch.cuda.synchronize()
    log(f"[bench] {wl.name}: {len(states)} units, W={wl.world_size}, grads {wl.grad_dtype}, "
        f"setup {time.time() - t0:.1f}s, HBM in use {torch.cuda.memory_allocated() / 2**30:.2f} GiB")
    hp = (wl.lr, wl.beta1, wl.beta2, wl.eps)
    rank = 0

    # The unsharded flat parameter is transient (Sec. 3.2.1: peak memory is the
    # largest unit); two buffers alternate, as with at most two unshards in flight.
    batched = args.mode in ("batch", "batch-lp")
    if args.depth <= 0:
        small = sorted(s.b_unshard for s in states)[len(states) // 2] <= (128 << 20)
        args.depth = 6 if small else 1
    lp_handoff = args.mode in ("lp", "batch-lp")
    nflat = 2 * args.depth if batched else 2
    flats = [flat] + [torch.empty_like(flat) for _ in range(nflat - 1)]

    def unshard(s, buf):
        F.fsdp_unshard(s.lay, s.shard_tab, buf[:s.P])

    def reduce_adam(s, t):
        F.fsdp_reduce_scatter_adam_fused(s.lay, s.grad_tab, rank, pre, post, None, s.shards[rank], s.m, s.v, t,
                                         *hp, None)

    def reduce_adam_prefetch(s, t, nxt, buf):
        F.fsdp_reduce_scatter_adam_prefetch_unshard(s.lay, s.grad_tab, rank, pre, post, None, s.shards[rank], s.m,
                                                    s.v, t, *hp, None, nxt.lay, nxt.shard_tab, buf[:nxt.P])

    # One step as a list of launches: (kernel kind, callable(t), algorithmic bytes).
    launches = []
    n = len(states)
    bkind = "batch_lp" if lp_handoff else "batch"
    if batched:
        d = args.depth
        groups = [list(range(i, min(i + d, n))) for i in range(0, n, d)]

        def make_batch(red, uns):
            b = F.Batch()
            # updates and unshards alternate, so that the library can pair a large update with a large unshard
            for j in range(max(len(red), len(uns))):
                if j < len(red):
                    s = states[red[j]]
                    b.add_reduce_scatter_adam(s.lay, s.grad_tab, rank, pre, post, None, s.shards[rank], s.m, s.v, *hp,
                                              s.lp_shards[rank] if lp_handoff else None)
                if j < len(uns):
                    i = uns[j]
                    s = states[i]
                    if lp_handoff:
                        b.add_unshard_lp(s.lay, s.lp_tab, flats[i % nflat][:s.P])
                    else:
                        b.add_unshard(s.lay, s.shard_tab, flats[i % nflat][:s.P])
            nbytes = sum(states[i].b_reduce + states[i].b_adam for i in red) + sum(states[i].b_unshard for i in uns)
            return b, nbytes

        b0, nb0 = make_batch([], groups[0])
        launches.append((bkind, (lambda t, b=b0: b.launch(t)), nb0))
        for j, grp in enumerate(groups):
            nxt = groups[j + 1] if j + 1 < len(groups) else []
            bj, nbj = make_batch(grp, nxt)
            launches.append((bkind, (lambda t, b=bj: b.launch(t)), nbj))
    if args.raf:
        # forward pass: the unshards alone, in forward order (the list above then plays the backward pass)
        fwd = []
        if batched:
            for grp in groups:
                b, nb = make_batch([], grp)
                fwd.append((bkind, (lambda t, b=b: b.launch(t)), nb))
        else:
            for i, s in enumerate(states):
                if args.mode == "lp":
                    fwd.append(("unshard_lp", (lambda t, s=s, buf=flats[i % 2]:
                                               F.fsdp_unshard_lp(s.lay, s.lp_tab, buf[:s.P])), s.b_unshard))
                else:
                    fwd.append(("unshard", (lambda t, s=s, buf=flats[i % 2]: unshard(s, buf)), s.b_unshard))
        launches = fwd + launches
    for i, s in enumerate(states):
        buf = flats[i % 2]
        if batched:
            break
        if args.mode == "prefetch":
            if i == 0:
                launches.append(("unshard", (lambda t, s=s, buf=buf: unshard(s, buf)), s.b_unshard))
            if i + 1 < n:
                nxt, nbuf = states[i + 1], flats[(i + 1) % 2]
                launches.append(("reduce_adam+unshard",
                                 (lambda t, s=s, nxt=nxt, nbuf=nbuf: reduce_adam_prefetch(s, t, nxt, nbuf)),
                                 s.b_reduce + s.b_adam + nxt.b_unshard))
            else:
                launches.append(("reduce_adam", (lambda t, s=s: reduce_adam(s, t)), s.b_reduce + s.b_adam))
        elif args.mode == "lp":
            launches.append(("unshard_lp", (lambda t, s=s, buf=buf: F.fsdp_unshard_lp(s.lay, s.lp_tab, buf[:s.P])),
                             s.b_unshard))
            launches.append(("reduce_adam_lp", (lambda t, s=s: F.fsdp_reduce_scatter_adam_fused(
                s.lay, s.grad_tab, rank, pre, post, None, s.shards[rank], s.m, s.v, t, *hp, s.lp_shards[rank])),
                s.b_reduce + s.b_adam))
        else:
            launches.append(("unshard", (lambda t, s=s, buf=buf: unshard(s, buf)), s.b_unshard))
            if args.mode == "fused":
                launches.append(("reduce_adam", (lambda t, s=s: reduce_adam(s, t)), s.b_reduce + s.b_adam))
            else:
                launches.append(("reduce_scatter", (lambda t, s=s: F.fsdp_reduce_scatter_local(
                    s.lay, s.grad_tab, rank, pre, post, s.gshard)), s.b_reduce))
                launches.append(("adam", (lambda t, s=s: F.fsdp_shard_adam_step(
                    s.lay, s.shards[rank], s.gshard, s.m, s.v, t, *hp)), s.b_adam))

    main_s = torch.cuda.Stream()

    def step(t):
        """One pass over all units, in order, on main_s."""
        for _kind, fn, _b in launches:
            fn(t)

    # A graph replay costs a fixed 6-10 us per step on this machine, which a step of
    # a few long launches does not win back (measured: configuration 1, 6 launches,
    # 259 us eagerly against 265 us replayed); steps of many launches replay a graph.
    use_graph = args.graph or (not args.no_graph and len(launches) > GRAPH_MIN_LAUNCHES)
    graph = None
    with torch.cuda.stream(main_s):
        step(1)                      # first-touch / module load outside any capture
        torch.cuda.synchronize()
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=main_s):
                step(2)
        run = (lambda t: graph.replay()) if use_graph else step

        for i in range(args.warmup):
            run(3 + i)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.steps):
            run(3 + args.warmup + i)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - tb) * 1e3
        dev_ms = e0.elapsed_time(e1)
    ms_per_step = wall_ms / args.steps
    step_bytes = sum(s.b_total for s in states) + (sum(s.b_unshard for s in states) if args.raf else 0)
    # what the chosen mode's kernels really read and write per step (the metric's numerator above is fixed)
    n_unshard = 2 if args.raf else 1
    if args.mode == "separate":
        touched = step_bytes
    elif lp_handoff:
        touched = sum(n_unshard * 4 * s.P + s.gbytes * s.P + 26 * s.S for s in states)
    else:
        touched = sum(n_unshard * 6 * s.P + s.gbytes * s.P + 24 * s.S for s in states)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    log(f"[bench] {args.steps} steps: wall {wall_ms:.3f} ms, device {dev_ms:.3f} ms, "
        f"{ms_per_step * 1e3:.1f} us/step, {value:.1f} GB/s effective ({100 * value / HBM_PEAK_GBPS:.1f}% of peak)")

    # ---- per-kernel durations (HIP events on the launch stream) -> roofline of the dominant kernel
    roofline = None
    per_kernel = {}
    if not args.no_kernel_timing:
        # Each kernel kind alone, launched for unit 0, 1, ... in order and the
        # whole sequence repeated, bracketed by one pair of HIP events on the
        # launch stream: average duration per launch with the same cold-cache
        # rotation over the units' buffers as in the timed steps.
        reps = max(10, min(200, int(25.0 / max(ms_per_step, 1e-3))))      # about 25 ms of launches per kind
        kinds = []
        for kind, _fn, _b in launches:
            if kind not in kinds:
                kinds.append(kind)
        with torch.cuda.stream(main_s):
            for kind in kinds:
                mine = [(fn, b) for k, fn, b in launches if k == kind]
                for fn, _b in mine:
                    fn(2)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                a.record()
                for _ in range(reps):
                    for fn, _b in mine:
                        fn(2)
                b.record()
                torch.cuda.synchronize()
                tot_us = a.elapsed_time(b) * 1e3 / reps
                nb = sum(b_ for _fn, b_ in mine)
                per_kernel[kind] = {"launches_per_step": len(mine), "avg_us": tot_us / len(mine),
                                    "total_us_per_step": tot_us, "alg_bytes_per_launch": nb / len(mine),
                                    "GBps": nb / (tot_us * 1e-6) / 1e9}
        dom = max(per_kernel, key=lambda k: per_kernel[k]["total_us_per_step"])
        traffic = None
        try:
            with open(args.traffic_json) as fh:
                traffic = json.load(fh).get(f"{wl.name}:{args.mode}:{dom}")
        except (OSError, ValueError):
            pass
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(per_kernel[dom]["GBps"], 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(per_kernel[dom]["GBps"] / HBM_PEAK_GBPS, 4),
                    "traffic": traffic, "avg_launch_us": round(per_kernel[dom]["avg_us"], 2),
                    "alg_bytes_per_launch": per_kernel[dom]["alg_bytes_per_launch"]}
        for k, v in per_kernel.items():
            log(f"[bench] kernel {k}: avg {v['avg_us']:.2f} us/launch, {v['GBps']:.1f} GB/s algorithmic")

    # ---- the CPU oracle on the host cores, same three operations, bounded sample
    cpu = None
    if not args.no_cpu_baseline and not args.raf:      # the oracle leg times the one-unshard step only
        cpu = cpu_baseline(states, wl, pre, post, rank, hp, torch)

    out = {
        "metric": "effective HBM GB/s per FSDP unit pass: unshard + reduce-scatter + Adam",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "units": len(states), "world_size": wl.world_size,
                   "grad_dtype": wl.grad_dtype, "unshard_dtype": "bf16", "rank": rank, "mode": args.mode,
                   "reshard_after_forward": bool(args.raf),
                   "prefetch_depth": args.depth if batched else (1 if args.mode == "prefetch" else 0),
                   "hip_graph": use_graph, "launches_per_step": len(launches), "alg_bytes_per_step": step_bytes,
                   "touched_bytes_per_step": touched},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "roofline": roofline, "cpu_baseline": cpu, "kernels": per_kernel,
    }
    print(json.dumps(out), flush=True)


def next_rows(args, wl, F, torch, workloads):
    """Hybrid-sharding reduction (Sec. 3.2.2) and gradient accumulation
    (Sec. 3.3.4) on the largest unit of the workload: one kernel each, timed
    back to back over rotating buffer sets between one pair of HIP events."""
    unit = max(wl.units, key=lambda u: sum(workloads.numel(s) for s in u.shapes))
    W = wl.world_size
    gdt = torch.float32 if wl.grad_dtype == "f32" else torch.bfloat16
    gb = 4 if wl.grad_dtype == "f32" else 2
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    G = 2 if 2 * W <= 64 else 1
    nsets = max(1, min(3, int(100e9 // (W * G * P * gb + 2 * W * P + 18 * P))))   # rotate buffer sets while HBM allows
    pre, post = F.fsdp_default_divide_factors(W * G)
    pre_w, post_w = F.fsdp_default_divide_factors(W)
    sets = []
    for i in range(nsets):
        grads = [workloads.gen_rank_grad(P, N, w, i, wl.grad_dtype, device="cuda") for w in range(W * G)]
        d = {"grads": F.PtrArray(grads), "flat": F.PtrArray(grads[:W]),
             "out": torch.zeros(S, device="cuda"), "acc": torch.zeros(P, device="cuda")}
        # FP16 path (Sec. 4.4): fp16 gradient buffers of the W ranks, fp32 shards, an fp16 flat buffer, the scaler flag
        d["g16"] = F.PtrArray([g.to(torch.float16) for g in grads[:W]])
        d["shards"] = F.PtrArray([torch.randn(S, device="cuda") * 0.02 for _ in range(W)])
        d["flat16"] = torch.empty(P, dtype=torch.float16, device="cuda")
        d["flat32"] = torch.empty(P, dtype=torch.float32, device="cuda")
        d["flag"] = torch.zeros(1, device="cuda")
        sets.append(d)
    rows = {
        "reduce_scatter_hybrid": (lambda d: F.fsdp_reduce_scatter_hybrid(lay, d["grads"], G, 0, pre, post, d["out"]),
                                  gb * S * W * G + 4 * S),
        "reduce_scatter_accumulate": (lambda d: F.fsdp_reduce_scatter_accumulate(lay, d["flat"], 0, pre, post, d["out"]),
                                      gb * P + 8 * S),
        "grad_accumulate": (lambda d: F.fsdp_grad_accumulate(lay, d["acc"], d["flat"].tensors[0]), (8 + gb) * P),
        "unshard_fp16": (lambda d: F.fsdp_unshard(lay, d["shards"], d["flat16"]), 6 * P),
        "unshard_fp32": (lambda d: F.fsdp_unshard(lay, d["shards"], d["flat32"]), 8 * P),
        "reduce_scatter_unscale_fp16": (lambda d: F.fsdp_reduce_scatter_unscale(
            lay, d["g16"], 0, pre_w, post_w, 1.0 / 1024.0, d["out"], d["flag"]), 2 * P + 4 * S),
    }
    out = {}
    reps = 30
    for name, (fn, nbytes) in rows.items():
        for d in sets:
            fn(d)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(reps):
            fn(sets[i % nsets])
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / reps
        out[name] = {"avg_us": round(us, 2), "alg_bytes": nbytes, "GBps": round(nbytes / us / 1e3, 1),
                     "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
        log(f"[bench] {name}: {us:.2f} us, {nbytes / us / 1e3:.1f} GB/s")
    print(json.dumps({"metric": "effective HBM GB/s of the rows beyond the hot path", "unit": "GB/s",
                      "config": {"workload": wl.name, "unit": unit.name, "world_size": W, "hybrid_groups": G,
                                 "grad_dtype": wl.grad_dtype}, "rows": out}), flush=True)


def probe_copy(n, torch, fbuild):
    """N launches of a plain copy of 256 MiB (reads 256 MiB, writes 256 MiB)."""
    import ctypes
    lib = ctypes.CDLL(fbuild.build_probe(force=False))
    lib.fsdp_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    nbytes = 256 << 20
    bufs = [(torch.ones(nbytes // 4, dtype=torch.float32, device="cuda"),
             torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")) for _ in range(3)]
    torch.cuda.synchronize()
    st = torch.cuda.current_stream().cuda_stream
    for i in range(n):
        src, dst = bufs[i % len(bufs)]
        rc = lib.fsdp_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, st)
        assert rc == 0, rc
    torch.cuda.synchronize()
    assert bool((bufs[0][1] == 1).all())
    print(json.dumps({"probe": "copy", "launches": n, "bytes_read_per_launch": nbytes,
                      "bytes_written_per_launch": nbytes}), flush=True)


def cpu_baseline(states, wl, pre, post, rank, hp, torch):
    """Time the oracle (as it stands) on the host: unshard + rank share of the
    reduce-scatter + Adam for a bounded sample of the workload's units."""
    import numpy as np
    import oracle
    budget_s = 10.0
    done_bytes = 0
    spent = 0.0
    n_units = 0
    host = []
    for s in states:
        S = s.S
        if wl.grad_dtype == "f32":
            h_slices = [g[rank * S:(rank + 1) * S].cpu().numpy() for g in s.grads]
        else:
            h_slices = [g[rank * S:(rank + 1) * S].cpu().view(torch.int16).numpy().view(np.uint16) for g in s.grads]
        host.append(([x.cpu().numpy() for x in s.shards], h_slices, s.m.cpu().numpy(), s.v.cpu().numpy(), s.b_total))
    def one_pass():
        nonlocal done_bytes, spent, n_units
        for h_shards, h_slices, h_m, h_v, nbytes in host:
            t0 = time.perf_counter()
            oracle.unshard_bf16(h_shards)
            g = oracle.reduce_slices(h_slices, pre, post)
            oracle.adam_f32(h_shards[rank], g, h_m, h_v, 1, *hp)
            spent += time.perf_counter() - t0
            done_bytes += nbytes
            n_units += 1

    passes = 0
    while spent < budget_s:
        one_pass()
        passes += 1
    out = {"value": round(done_bytes / spent / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(),
           "kind": "oracle", "sample": f"{passes} passes over all {len(states)} units of {wl.name} "
                                       f"({n_units} unit passes), {spent:.2f} s of oracle time"}
    # the same on one host thread, a shorter sample (reported beside the all-cores figure)
    threads = oracle.num_threads()
    oracle.set_num_threads(1)
    try:
        done_bytes, spent, n_units = 0, 0.0, 0
        while spent < 3.0:
            one_pass()
        out["value_1_thread"] = round(done_bytes / spent / 1e9, 3)
    finally:
        oracle.set_num_threads(threads)
    return out


if __name__ == "__main__":
    main()
