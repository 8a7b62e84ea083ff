#!/usr/bin/env python3
"""Benchmark of the FlatParameter data path on one MI355X.

A step is one pass of the hot path over every FSDP unit of a workload, in
order: unshard (fp32 shards -> bf16 flat buffer, all W ranks' shards), then the
rank-0 share of the reduce-scatter over W simulated ranks' gradient buffers and
the sharded Adam step.  Inputs are synthetic, seeded, and resident in HBM before
the timed region starts.

Without --config all five configurations are timed in one run.  The headline
(`value`, `config.workload`, `roofline`, `cpu_baseline`) is the largest one, a
GPT-3-175B block over 16 ranks (18.1 GB per pass); the others are listed under
`configs`.  Prints ONE JSON line: metric = effective HBM GB/s (algorithmic bytes
of unshard + reduce-scatter + Adam, summed over the units, per second).
"""
from __future__ import annotations

import argparse
import ctypes
import gc
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GRAPH_MIN_LAUNCHES = 16      # steps with more launches than this are captured in a HIP graph by default
HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, published
HEADLINE_CONFIG = 4          # the largest single-GPU configuration
COLD_REPLICAS = 6            # configuration 0 rotates over this many copies of its unit (see run_config)
PROBE_SRC = os.path.join(ROOT, "bench_probe.hip")
PROBE_LIB = os.path.join(ROOT, "libbench_probe.so")


VERBOSE = False


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def vlog(*a):
    if VERBOSE:
        log(*a)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=None,
                    help="time one workload only: 0 one GPT-2-small block, 1 full GPT-2-small, 2 1.3B blocks W=12, "
                         "3 Llama-7B blocks W=64, 4 one GPT-3-175B block W=16 (default: all five, headline = 4)")
    ap.add_argument("--max-units", type=int, default=0, help="limit the number of units (0 = all)")
    ap.add_argument("--depth", type=int, default=0,
                    help="units per batch in --mode batch (prefetch depth); 0 = 6 when the units are small enough to "
                         "share grids (launch-bound), 1 when they are not (then only the pairing of unit i's update "
                         "with unit i+1's unshard matters)")
    ap.add_argument("--mode", choices=["batch", "fused", "separate", "lp", "batch-lp"], default="batch",
                    help="batch: the updates of `depth` units and the prefetched unshards of the next `depth` units "
                         "are independent and are recorded as one batch (fsdp_batch_*), which the library issues in "
                         "as few grids as it can; fused: reduce-scatter + Adam in one launch, unshard in another; "
                         "separate: the three required entry points, one launch each; lp: every rank keeps a bf16 "
                         "copy of its shard (written by the fused Adam), the unshard gathers bf16 (Sec. 4.4); "
                         "batch-lp: the same hand-off issued as batches (moves 4P instead of 6P per unshard; the "
                         "metric's numerator stays the fixed 6P)")
    ap.add_argument("--graph", action="store_true", help="always replay the step as a HIP graph")
    ap.add_argument("--no-graph", action="store_true", help="always launch eagerly")
    ap.add_argument("--replicas", type=int, default=0,
                    help="rotate the steps over this many copies of the workload's buffers (cold caches); 0 = "
                         f"{COLD_REPLICAS} for configuration 0, whose single unit would otherwise stay in the 256 MB "
                         "Infinity Cache, 1 for the others (their steps already cycle through far more than that)")
    ap.add_argument("--probe-copy", type=int, default=0, metavar="N",
                    help="run only N launches of a plain 256 MiB copy kernel (calibrates rocprofv3 --pmc byte counters)")
    ap.add_argument("--probe-mix", action="store_true",
                    help="run only the read / write mix probe: 16 streams of a GPT-3-175B block's rank slice read in "
                         "lock step as the reduce-scatter reads them, with and without the fp32 result written")
    ap.add_argument("--probe-update", action="store_true",
                    help="run only the update probe: the library's fused reduce-scatter + Adam and a plain kernel with "
                         "the same memory traffic, on the same buffers (--config 3 or 4: 16-bit gradients)")
    ap.add_argument("--probe-small", action="store_true",
                    help="run only the small-launch probe: plain kernels carrying the traffic of configuration 0's two "
                         "launches, over rotating (cold) buffers")
    ap.add_argument("--next-rows", action="store_true",
                    help="measure the kernels beyond the hot path (hybrid-sharding reduce, gradient accumulation, "
                         "fp16 / fp32 unshard, unscale) on the workload's largest unit and print their own JSON line")
    ap.add_argument("--unit-scale", type=int, default=1,
                    help="size study: every unit holds this many copies of its parameter list")
    ap.add_argument("--raf", action="store_true",
                    help="reshard after forward (Sec. 3, Sec. 4.4): every unit is unsharded twice per step, once for "
                         "the forward pass and once before its backward; the metric's bytes count both")
    ap.add_argument("--grad-dtype", choices=["f32", "bf16"], default=None,
                    help="override the workload's gradient dtype (the fp32 / bf16 variants of every configuration)")
    ap.add_argument("--rank", type=int, default=0,
                    help="the rank whose share of the reduce-scatter and of the optimizer step is timed (default 0; "
                         "with a shard size that is not a multiple of 4, other ranks' gradient slices are not "
                         "16-byte aligned)")
    ap.add_argument("--walk", choices=["auto", "wide", "deep", "half"], default="auto",
                    help="rank walk of the stand-alone reduce-scatter kernels (the layouts' fsdp_layout_init_ex hint)")
    ap.add_argument("--grad-sets", type=int, default=0,
                    help="cap the number of distinct sets of gradient buffers per unit shape (0 = as many as fit)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (timing and parity)")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the plain copy / read / write kernels")
    ap.add_argument("--detail-json", default=os.path.join(ROOT, "bench_detail.json"),
                    help="file that receives every figure of the run (the line on stdout is a compact view); '' = none")
    ap.add_argument("--verbose", action="store_true", help="log per-kernel and per-unit lines as they are measured")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="HBM bytes per launch by `workload:kernel`, from rocprofv3 --pmc runs (see profiles/)")
    return ap.parse_args()


# ---------------------------------------------------------------------------
# measurement support: plain streaming kernels (bench_probe.hip)
# ---------------------------------------------------------------------------
def build_probe(force: bool = False) -> str:
    """Compile bench_probe.hip next to this file (hipcc, gfx950)."""
    if not force and os.path.exists(PROBE_LIB) and os.path.getmtime(PROBE_LIB) >= os.path.getmtime(PROBE_SRC):
        return PROBE_LIB
    tmp = PROBE_LIB + f".tmp{os.getpid()}"
    hipcc = os.environ.get("HIPCC") or ("/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else "hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang",
                           "-target-feature", "-Xclang", "-packed-fp32-ops", "-x", "hip", PROBE_SRC, "-o", tmp])
    os.replace(tmp, PROBE_LIB)
    return PROBE_LIB


def load_probe():
    lib = ctypes.CDLL(build_probe(force=False))
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    lib.fsdp_probe_copy.argtypes = [vp, vp, i64, ctypes.c_int, vp]
    lib.fsdp_probe_memcpy.argtypes = [vp, vp, i64, vp]
    lib.fsdp_probe_cast.argtypes = [vp, vp, i64, ctypes.c_int, vp]
    lib.fsdp_probe_read.argtypes = [vp, i64, vp, ctypes.c_int, vp]
    lib.fsdp_probe_write.argtypes = [vp, i64, ctypes.c_float, ctypes.c_int, vp]
    lib.fsdp_probe_streams.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, ctypes.c_int, vp, vp]
    lib.fsdp_probe_update.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, vp, vp, vp, vp]
    return lib


def measure_ceilings(torch):
    """Plain copy, read-only and write-only streaming kernels over 1 GiB
    buffers (four in rotation, far beyond the 256 MB Infinity Cache), timed
    with HIP events on the launch stream: what this machine gives a kernel that
    does nothing but stream."""
    lib = load_probe()
    nbytes = 1 << 30
    bufs = [torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda") for _ in range(4)]
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    reps = 24

    def timed(fn, moved):
        for i in range(4):
            fn(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return round(moved * reps / (a.elapsed_time(b) * 1e-3) / 1e9, 1)

    def chk(rc):
        assert rc == 0, f"probe kernel launch failed: hipError_t {rc}"

    # Workgroup size per kernel: what measured fastest for its shape on MI355X (copy and cast: single-wave
    # workgroups, 2-7 % above 256 lanes; the one-sided kernels need 256 lanes: 6.9 against 4.8 TB/s).
    LANES, ONE_SIDED = 64, 256
    out = {
        "copy_GBps": timed(lambda i: chk(lib.fsdp_probe_copy(bufs[(i + 1) % 4].data_ptr(), bufs[i % 4].data_ptr(), nbytes,
                                                             LANES, st)), 2 * nbytes),
        "read_GBps": timed(lambda i: chk(lib.fsdp_probe_read(bufs[i % 4].data_ptr(), nbytes, sink.data_ptr(), ONE_SIDED, st)),
                           nbytes),
        "write_GBps": timed(lambda i: chk(lib.fsdp_probe_write(bufs[i % 4].data_ptr(), nbytes, 0.0, ONE_SIDED, st)), nbytes),
        "cast_GBps": timed(lambda i: chk(lib.fsdp_probe_cast(bufs[(i + 1) % 4].data_ptr(), bufs[i % 4].data_ptr(), nbytes // 2,
                                                             LANES, st)), nbytes + nbytes // 2),
        "copy_256_lane_workgroups_GBps": timed(lambda i: chk(lib.fsdp_probe_copy(
            bufs[(i + 1) % 4].data_ptr(), bufs[i % 4].data_ptr(), nbytes, 256, st)), 2 * nbytes),
        "hipMemcpyAsync_d2d_GBps": timed(lambda i: chk(lib.fsdp_probe_memcpy(bufs[(i + 1) % 4].data_ptr(), bufs[i % 4].data_ptr(),
                                                                             nbytes, st)), 2 * nbytes),
        "buffer_bytes": nbytes,
        "note": "plain nontemporal streaming kernels of bench_probe.hip (copy and cast in single-wave workgroups, read-only "
                "and write-only in 256-lane ones: the fastest shape of each) and the runtime's own device-to-device copy, "
                "same run, HIP events; copy and cast count bytes read + bytes written",
    }
    assert float(sink.item()) == 0.0
    del bufs
    torch.cuda.empty_cache()
    return out


def probe_copy(n, torch):
    """N launches of a plain copy of 256 MiB (reads 256 MiB, writes 256 MiB)."""
    lib = load_probe()
    nbytes = 256 << 20
    bufs = [(torch.ones(nbytes // 4, dtype=torch.float32, device="cuda"),
             torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")) for _ in range(3)]
    torch.cuda.synchronize()
    st = torch.cuda.current_stream().cuda_stream
    for i in range(n):
        src, dst = bufs[i % len(bufs)]
        rc = lib.fsdp_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, 256, st)
        assert rc == 0, rc
    torch.cuda.synchronize()
    assert bool((bufs[0][1] == 1).all())
    print(json.dumps({"probe": "copy", "launches": n, "bytes_read_per_launch": nbytes,
                      "bytes_written_per_launch": nbytes}), flush=True)


def probe_mix(torch):
    """What a small write stream costs next to many read streams.  The rank
    walk of the reduce-scatter on the GPT-3-175B block reads the rank's slice
    (113,256,192 bf16 = 226.5 MB) of 16 gradient buffers and writes 453 MB of
    fp32 sums.  Timed here with almost no arithmetic: the reads alone, the
    reads plus the write, and the write alone; a half-duplex memory would take
    t(reads) + t(write) for the mix."""
    lib = load_probe()
    nbytes = 226512384
    st = torch.cuda.current_stream().cuda_stream
    out = torch.zeros(nbytes // 2, dtype=torch.float32, device="cuda")
    res = {}
    for n in (1, 2, 4, 8, 16):
        bufs = [torch.zeros(nbytes // 2, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
        tab = (ctypes.c_void_p * n)(*[b.data_ptr() for b in bufs])

        def timed(fn):
            for _ in range(2):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for _ in range(6):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e3 / 6

        def run(store):
            rc = lib.fsdp_probe_streams(tab, n, nbytes, store, out.data_ptr(), st)
            assert rc == 0, rc

        def write_only():
            rc = lib.fsdp_probe_write(out.data_ptr(), 2 * nbytes, 0.0, 256, st)
            assert rc == 0, rc

        t_r, t_rw, t_rw2, t_w = timed(lambda: run(0)), timed(lambda: run(1)), timed(lambda: run(2)), timed(write_only)
        res[f"{n}_streams"] = {
            "read_bytes": n * nbytes, "write_bytes": 2 * nbytes, "reads_only_us": round(t_r, 1),
            "reads_and_write_us": round(t_rw, 1), "reads_and_strided_write_us": round(t_rw2, 1),
            "write_only_us": round(t_w, 1),
            "reads_only_GBps": round(n * nbytes / t_r / 1e3, 1),
            "mix_GBps": round((n + 2) * nbytes / t_rw / 1e3, 1),
            "half_duplex_model_us": round(t_r + t_w, 1),
        }
        log(f"[probe-mix] {n} streams: reads alone {t_r:.1f} us ({n * nbytes / t_r / 1e3:.0f} GB/s), with the write "
            f"{t_rw:.1f} us ({(n + 2) * nbytes / t_rw / 1e3:.0f} GB/s; stores of 32 bytes per lane: {t_rw2:.1f} us), "
            f"write alone {t_w:.1f} us")
        del bufs
        torch.cuda.empty_cache()
    print(json.dumps({"probe": "read/write mix", "stream_bytes": nbytes, "results": res}), flush=True)


def probe_update(cfg, F, torch, workloads):
    """The fused reduce-scatter + Adam of a configuration's largest unit next
    to a plain kernel that moves the same bytes through the same buffers (W
    rank slices of 16-bit gradients read; p, m, v read and written in place)
    with almost no arithmetic: what the memory system gives this traffic,
    whatever the kernel.  The two are timed alternately, three rounds."""
    lib = load_probe()
    wl = workloads.config(cfg)
    assert wl.grad_dtype == "bf16", "the update probe reads 16-bit gradient streams: --config 3 or 4"
    W = wl.world_size
    unit = max(wl.units, key=lambda u: sum(workloads.numel(x) for x in u.shapes))
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P = lay.shard, lay.padded
    assert (2 * S) % 16 == 0
    pre, post = F.fsdp_default_divide_factors(W)
    hp = (wl.lr, wl.beta1, wl.beta2, wl.eps)
    st = torch.cuda.current_stream().cuda_stream
    touched = 2 * W * S + 24 * S
    nsets = max(1, min(8, int(2e9 // touched) + 1))          # rotate while one launch moves less than 2 GB
    sets = []
    for i in range(nsets):
        grads = [workloads.gen_rank_grad(P, lay.numel, w, i, "bf16", device="cuda") for w in range(W)]
        state = [torch.empty(S, device="cuda").normal_(0, 0.02), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")]
        tab = (ctypes.c_void_p * W)(*[g.data_ptr() for g in grads])          # rank 0's slices start at the buffers' bases
        sets.append((F.PtrArray(grads), state, tab))

    walks = {"auto": F.FSDP_WALK_AUTO, "wide": F.FSDP_WALK_WIDE, "deep": F.FSDP_WALK_DEEP, "half": F.FSDP_WALK_HALF}
    lays = {name: F.fsdp_layout_init(unit.shapes, W, reduce_walk=hint) for name, hint in walks.items()}

    def library(name):
        def fn(i):
            tabs, (p, m, v), _ = sets[i % nsets]
            F.fsdp_reduce_scatter_adam_fused(lays[name], tabs, 0, pre, post, None, p, m, v, 2, *hp, None)
        return fn

    def plain(i):
        _, (p, m, v), tab = sets[i % nsets]
        rc = lib.fsdp_probe_update(tab, W, 2 * S, p.data_ptr(), m.data_ptr(), v.data_ptr(), st)
        assert rc == 0, rc

    reps = max(6, min(60, int(20e9 // touched)))

    def timed(fn):
        for i in range(nsets + 1):
            fn(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    rounds = []
    for _ in range(3):
        r = {f"library_{name}_us": round(timed(library(name)), 1) for name in walks}
        r["plain_us"] = round(timed(plain), 1)
        rounds.append(r)
        log(f"[probe-update] {wl.name}: " + ", ".join(f"{k[:-3]} {v:.1f} us ({touched / v / 1e3:.0f} GB/s)" for k, v in r.items()))
    print(json.dumps({"probe": "fused update (the library's choice of rank walk and each walk forced) against a plain kernel "
                               "with the same traffic", "workload": wl.name,
                      "unit": unit.name, "world_size": W, "touched_bytes": touched, "rotating_sets": nsets,
                      "rounds": rounds}), flush=True)


def probe_small(torch):
    """What plain streaming kernels take for the traffic of configuration 0's
    two launches (one GPT-2-small block over 8 ranks: the unshard reads 28.4 MB
    and writes 14.2 MB, the fused update reads 39.0 MB and writes 10.6 MB),
    launched back to back over 12 rotating sets of buffers like the timed
    steps: the floor that launch ramp and drain leave at this size."""
    lib = load_probe()
    st = torch.cuda.current_stream().cuda_stream
    R = 12

    def timed(fn, reps=300):
        for i in range(2 * R):
            fn(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    res = {}

    def streams(tag, n, nbytes, store):
        sets = []
        for _ in range(R):
            srcs = [torch.zeros(nbytes // 2, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
            out = torch.zeros(nbytes // 2, dtype=torch.float32, device="cuda")
            sets.append((srcs, out, (ctypes.c_void_p * n)(*[x.data_ptr() for x in srcs])))

        def fn(i):
            rc = lib.fsdp_probe_streams(sets[i % R][2], n, nbytes, store, sets[i % R][1].data_ptr(), st)
            assert rc == 0, rc

        us = timed(fn)
        moved = n * nbytes + (2 * nbytes if store else 0)
        res[tag] = {"streams": n, "read_bytes": n * nbytes, "written_bytes": 2 * nbytes if store else 0,
                    "us": round(us, 2), "GBps": round(moved / us / 1e3, 1)}
        log(f"[probe-small] {tag}: {us:.2f} us, {moved / 1e6:.1f} MB, {moved / us / 1e3:.0f} GB/s")

    def copy(tag, nbytes):
        bufs = [(torch.zeros(nbytes // 4, device="cuda"), torch.zeros(nbytes // 4, device="cuda")) for _ in range(R)]

        def fn(i):
            rc = lib.fsdp_probe_copy(bufs[i % R][1].data_ptr(), bufs[i % R][0].data_ptr(), nbytes, 64, st)
            assert rc == 0, rc

        us = timed(fn)
        res[tag] = {"read_bytes": nbytes, "written_bytes": nbytes, "us": round(us, 2), "GBps": round(2 * nbytes / us / 1e3, 1)}
        log(f"[probe-small] {tag}: {us:.2f} us, {2 * nbytes / 1e6:.1f} MB, {2 * nbytes / us / 1e3:.0f} GB/s")

    copy("empty_launch", 16)
    streams("unshard_traffic_4_streams_28.4MB_read_14.2MB_written", 4, 7087872, 1)
    copy("copy_of_the_same_total_21.3MB_each_way", 21263616)
    streams("update_traffic_11_streams_39.0MB_read_7.1MB_written", 11, 3543936, 1)
    copy("copy_of_the_same_total_23.0MB_each_way", 23035584)
    print(json.dumps({"probe": "small launches", "rotating_sets": R, "results": res}), flush=True)


# ---------------------------------------------------------------------------
# one workload
# ---------------------------------------------------------------------------
class UnitState:
    """Device buffers of one FSDP unit (caller-owned, as the library expects)."""

    def __init__(self, F, wl, unit, index, torch, workloads, share_grads_with=None, walk=0):
        W = wl.world_size
        self.name = unit.name
        self.index = index
        self.lay = F.fsdp_layout_init(unit.shapes, W, reduce_walk=walk)
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
        self.grad_tab = F.PtrArray(self.grads)
        self.lp_shards = self.lp_tab = None
        # algorithmic bytes (fixed numerators, whatever the kernels really touch)
        self.b_unshard = 6 * P
        self.b_reduce = self.gbytes * P + 4 * S
        self.b_adam = 28 * S
        self.b_total = self.b_unshard + self.b_reduce + self.b_adam

    def make_lp_shards(self, F, torch):
        """The ranks' bf16 copies of their shards (Sec. 4.4 hand-off modes only)."""
        W, S = self.W, self.S
        self.lp_base = torch.empty(W * S, dtype=torch.bfloat16, device="cuda")
        self.lp_shards = [self.lp_base[w * S:(w + 1) * S] for w in range(W)]
        for w in range(W):
            F.fsdp_cast_shard(self.lay, self.shards[w], self.lp_shards[w])
        self.lp_tab = F.PtrArray(self.lp_shards)


def make_states(F, wl, units, args, torch, workloads):
    states = []
    grad_budget = 160e9          # bytes of HBM given to the simulated ranks' gradient buffers
    used = 0.0
    walk = {"auto": F.FSDP_WALK_AUTO, "wide": F.FSDP_WALK_WIDE, "deep": F.FSDP_WALK_DEEP, "half": F.FSDP_WALK_HALF}[args.walk]
    for i, u in enumerate(units):
        share = None
        need = wl.world_size * sum(workloads.numel(s) for s in u.shapes) * (4 if wl.grad_dtype == "f32" else 2)
        same = [s for s in states if s.unit_shapes == u.shapes and s.owns_grads]
        if used + need > grad_budget or (args.grad_sets and len(same) >= args.grad_sets):
            share = same[len(states) % len(same)] if same else None
        st = UnitState(F, wl, u, i, torch, workloads, share_grads_with=share, walk=walk)
        st.unit_shapes, st.owns_grads = u.shapes, share is None
        used += need if share is None else 0
        states.append(st)
    return states


def build_launches(F, states, flats, args, depth, rank, pre, post, hp):
    """One step as a list of launches, each exactly one kernel of the library:
    (kernel name, callable(t), algorithmic bytes, bytes the kernel touches)."""
    mode = args.mode
    lp_handoff = mode in ("lp", "batch-lp")
    nflat = len(flats)
    n = len(states)
    launches = []

    def touched_update(s):
        return s.gbytes * s.P + (26 if lp_handoff else 24) * s.S      # fused: the gradient shard stays in registers

    def touched_unshard(s):
        return (4 if lp_handoff else 6) * s.P

    def batch_items(ops):
        """ops: [("update" | "unshard", unit index)] in issue order.  One batch when the library issues it as one
        grid; otherwise one batch per operation, in the same order, so that every item is one kernel."""
        def record(sub):
            b = F.Batch()
            for kind, i in sub:
                s = states[i]
                if kind == "update":
                    b.add_reduce_scatter_adam(s.lay, s.grad_tab, rank, pre, post, None, s.shards[rank], s.m, s.v, *hp,
                                              s.lp_shards[rank] if lp_handoff else None)
                elif lp_handoff:
                    b.add_unshard_lp(s.lay, s.lp_tab, flats[i % nflat][:s.P])
                else:
                    b.add_unshard(s.lay, s.shard_tab, flats[i % nflat][:s.P])
            return b

        def item(b, sub, plan):
            alg = sum(states[i].b_reduce + states[i].b_adam if k == "update" else states[i].b_unshard for k, i in sub)
            tch = sum(touched_update(states[i]) if k == "update" else touched_unshard(states[i]) for k, i in sub)
            return (plan["kernel"], (lambda t, b=b: b.launch(t)), alg, tch)

        b = record(ops)
        plan = b.launches()
        if len(plan) == 1:
            return [item(b, ops, plan[0])]
        b.close()
        out = []
        for op in ops:
            b1 = record([op])
            p1 = b1.launches()
            assert len(p1) == 1, f"{op}: {p1}"
            out.append(item(b1, [op], p1[0]))
        return out

    if mode in ("batch", "batch-lp"):
        groups = [list(range(i, min(i + depth, n))) for i in range(0, n, depth)]

        def ops_of(red, uns):
            # updates and unshards alternate, so that the library can pair a large update with a large unshard
            ops = []
            for j in range(max(len(red), len(uns))):
                if j < len(red):
                    ops.append(("update", red[j]))
                if j < len(uns):
                    ops.append(("unshard", uns[j]))
            return ops

        if args.raf:      # forward pass: the unshards alone, in forward order (the rest then plays the backward pass)
            for grp in groups:
                launches += batch_items(ops_of([], grp))
        launches += batch_items(ops_of([], groups[0]))
        for j, grp in enumerate(groups):
            launches += batch_items(ops_of(grp, groups[j + 1] if j + 1 < len(groups) else []))
        return launches

    def unshard_item(i, s):
        buf = flats[i % 2]
        if mode == "lp":
            return ("gather_lp_kernel", (lambda t, s=s, buf=buf: F.fsdp_unshard_lp(s.lay, s.lp_tab, buf[:s.P])),
                    s.b_unshard, touched_unshard(s))
        probe = F.Batch()          # a one-member batch goes out through the same entry point: its plan names the kernel
        probe.add_unshard(s.lay, s.shard_tab, buf[:s.P])
        name = probe.launches()[0]["kernel"]
        probe.close()
        return (name, (lambda t, s=s, buf=buf: F.fsdp_unshard(s.lay, s.shard_tab, buf[:s.P])),
                s.b_unshard, touched_unshard(s))

    assert all(s.W <= 64 for s in states), "these modes name one kernel per entry point, which holds up to 64 ranks"
    if args.raf:
        launches += [unshard_item(i, s) for i, s in enumerate(states)]
    for i, s in enumerate(states):
        launches.append(unshard_item(i, s))
        if mode in ("fused", "lp"):
            launches.append(("reduce_kernel", (lambda t, s=s: F.fsdp_reduce_scatter_adam_fused(
                s.lay, s.grad_tab, rank, pre, post, None, s.shards[rank], s.m, s.v, t, *hp,
                s.lp_shards[rank] if mode == "lp" else None)), s.b_reduce + s.b_adam, touched_update(s)))
        else:
            launches.append(("reduce_kernel", (lambda t, s=s: F.fsdp_reduce_scatter_local(
                s.lay, s.grad_tab, rank, pre, post, s.gshard)), s.b_reduce, s.b_reduce))
            launches.append(("adam_kernel", (lambda t, s=s: F.fsdp_shard_adam_step(
                s.lay, s.shards[rank], s.gshard, s.m, s.v, t, *hp)), s.b_adam, s.b_adam))
    return launches


def run_config(cfg, args, F, torch, workloads, headline, traffic_table):
    """Set up one workload, time `steps` steps after `warmup`, then the kernels
    one kind at a time.  Returns (record for the JSON line, cpu_baseline or None)."""
    wl = workloads.config(cfg)
    if args.grad_dtype:
        import dataclasses
        wl = dataclasses.replace(wl, grad_dtype=args.grad_dtype)
    units = list(wl.units)
    if args.max_units:
        units = units[:args.max_units]
    if args.unit_scale > 1:
        units = [workloads.Unit(f"{u.name}x{args.unit_scale}", tuple(u.shapes) * args.unit_scale) for u in units]
    pre, post = F.fsdp_default_divide_factors(wl.world_size)
    hp = (wl.lr, wl.beta1, wl.beta2, wl.eps)
    rank = args.rank
    if not 0 <= rank < wl.world_size:
        raise SystemExit(f"bench.py: --rank {rank} is outside 0..{wl.world_size - 1} of {wl.name}")
    batched = args.mode in ("batch", "batch-lp")
    lp_handoff = args.mode in ("lp", "batch-lp")
    # Configuration 0 is one 99 MB unit: run over and over it would stay in the
    # 256 MB Infinity Cache, so its steps rotate over copies of the unit (cold),
    # and the figure with one copy (warm) is reported beside it.
    replicas = args.replicas or (COLD_REPLICAS if cfg == 0 else 1)

    t0 = time.time()
    reps_states, reps_launches = [], []
    depth = args.depth
    for _ in range(replicas):
        states = make_states(F, wl, units, args, torch, workloads)
        if lp_handoff:
            for s in states:
                s.make_lp_shards(F, torch)
        if depth <= 0:
            small = sorted(s.b_unshard for s in states)[len(states) // 2] <= (128 << 20)
            depth = 6 if small else 1
        # The unsharded flat parameter is transient (Sec. 3.2.1: peak memory is the largest unit);
        # as many buffers rotate as unshards can be in flight.
        nflat = 2 * depth if batched else 2
        flats = [torch.empty(max(s.P for s in states), dtype=torch.bfloat16, device="cuda") for _ in range(nflat)]
        reps_states.append(states)
        reps_launches.append(build_launches(F, states, flats, args, depth, rank, pre, post, hp))
    states, launches = reps_states[0], reps_launches[0]
    torch.cuda.synchronize()
    vlog(f"[bench] {wl.name}: {len(states)} units, W={wl.world_size}, grads {wl.grad_dtype}, mode {args.mode}, "
        f"{len(launches)} launches per step, setup {time.time() - t0:.1f}s, HBM in use "
        f"{torch.cuda.memory_allocated() / 2**30:.2f} GiB")

    # ---- parity of the first step against the oracle, and the oracle's own timing (headline only)
    first = None
    if headline and not args.no_cpu_baseline and not args.raf and args.mode == "batch":
        first = FirstStepCheck(states, wl, rank, torch)

    main_s = torch.cuda.Stream()

    def step_of(ls):
        def step(t):
            for _kind, fn, _a, _b in ls:
                fn(t)
        return step

    steps_fns = [step_of(ls) for ls in reps_launches]
    # A graph replay costs a fixed 6-10 us per step on this machine, which a step of a few
    # long launches does not win back; steps of many launches replay a graph.
    use_graph = (args.graph or (not args.no_graph and len(launches) > GRAPH_MIN_LAUNCHES)) and replicas == 1
    rec = {}
    with torch.cuda.stream(main_s):
        for fn in steps_fns:
            fn(1)                      # first touch / module load outside any capture
        torch.cuda.synchronize()
        if first is not None:
            first.fetch_gpu(states, rank)
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=main_s):
                steps_fns[0](2)
            run = lambda t: graph.replay()                                   # noqa: E731
        else:
            run = lambda t: steps_fns[t % replicas](t)                       # noqa: E731

        def timed_pass(run_fn, per_step_events):
            for i in range(args.warmup):
                run_fn(3 + i)
            torch.cuda.synchronize()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)] if per_step_events else None
            tb = time.perf_counter()
            if evs:
                evs[0].record()
            for i in range(args.steps):
                run_fn(3 + args.warmup + i)
                if evs:
                    evs[i + 1].record()
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - tb) * 1e3
            if not evs:
                return wall_ms, None
            return wall_ms, sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(args.steps))

        # the figure: exactly `steps` steps between two synchronisations, wall clock
        wall_ms, _ = timed_pass(run, False)
        # the same again with a HIP event after every step: minimum and median step time
        _, per_step = timed_pass(run, True)
        ms_per_step = wall_ms / args.steps
        warm = None
        if replicas > 1:               # the same steps on one copy of the buffers: what the Infinity Cache adds
            _w_ms, w_steps = timed_pass(lambda t: steps_fns[0](t), True)
            warm = {"us_per_step_median": round(w_steps[len(w_steps) // 2], 2), "us_per_step_min": round(w_steps[0], 2)}

    step_bytes = sum(s.b_total for s in states) + (sum(s.b_unshard for s in states) if args.raf else 0)
    touched = sum(b for _k, _f, _a, b in launches)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    log(f"[bench] {wl.name}: {args.steps} steps, {ms_per_step * 1e3:.1f} us/step (min {per_step[0]:.1f}, median "
        f"{per_step[len(per_step) // 2]:.1f}), {value:.1f} GB/s effective ({100 * value / HBM_PEAK_GBPS:.1f}% of peak)")
    rec.update({
        "workload": wl.name, "units": len(states), "world_size": wl.world_size, "grad_dtype": wl.grad_dtype,
        "unshard_dtype": "bf16", "rank": rank, "mode": args.mode, "reshard_after_forward": bool(args.raf),
        "prefetch_depth": depth if batched else 0, "hip_graph": use_graph, "launches_per_step": len(launches),
        "buffer_replicas": replicas, "alg_bytes_per_step": step_bytes, "touched_bytes_per_step": touched,
        "us_per_step": round(ms_per_step * 1e3, 2), "us_per_step_min": round(per_step[0], 2),
        "us_per_step_median": round(per_step[len(per_step) // 2], 2),
        "GBps": round(value, 1), "GBps_touched": round(touched / (ms_per_step * 1e-3) / 1e9, 1),
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
    })
    if warm:
        warm["GBps"] = round(step_bytes / (warm["us_per_step_median"] * 1e-6) / 1e9, 1)
        rec["warm_one_replica"] = warm
    if cfg == 0:
        rec["note"] = ("99 MB in two dependent launches of ~8 us each: launch ramp and drain, not HBM, bound this "
                       "configuration; it stays below the 70 % target")

    # ---- per-kernel durations (HIP events on the launch stream)
    per_kernel = {}
    if not args.no_kernel_timing:
        # Each kernel alone: its launches of one step (of every replica), in order, the
        # sequence repeated, between one pair of HIP events on the launch stream: average
        # duration per launch with the same cold-cache rotation over the units' buffers
        # as in the timed steps.
        reps = max(5, min(200, int(25.0 / max(ms_per_step * replicas, 1e-3))))      # about 25 ms of launches per kernel
        names = []
        for k, _f, _a, _b in launches:
            if k not in names:
                names.append(k)
        with torch.cuda.stream(main_s):
            for name in names:
                mine = [(fn, a, b) for ls in reps_launches for k, fn, a, b in ls if k == name]
                for fn, _a, _b in mine:
                    fn(2)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(reps):
                    for fn, _a, _b in mine:
                        fn(2)
                e1.record()
                torch.cuda.synchronize()
                avg_us = e0.elapsed_time(e1) * 1e3 / reps / len(mine)
                alg = sum(a for _f, a, _b in mine) / len(mine)
                tch = sum(b for _f, _a, b in mine) / len(mine)
                per_step_launches = len(mine) // replicas
                per_kernel[name] = {
                    "launches_per_step": per_step_launches, "avg_us": round(avg_us, 2),
                    "total_us_per_step": round(avg_us * per_step_launches, 2), "alg_bytes_per_launch": round(alg),
                    "touched_bytes_per_launch": round(tch), "GBps": round(alg / (avg_us * 1e-6) / 1e9, 1),
                    "GBps_touched": round(tch / (avg_us * 1e-6) / 1e9, 1),
                    "hbm_bytes_per_launch": traffic_table.get(f"{wl.name}:{name}") if args.mode == "batch" else None,
                }
                vlog(f"[bench] {wl.name} kernel {name}: {per_step_launches} per step, avg {avg_us:.2f} us, "
                    f"{alg / avg_us / 1e3:.1f} GB/s algorithmic, {tch / avg_us / 1e3:.1f} GB/s touched")
    rec["kernels"] = per_kernel

    # ---- per FSDP unit: each distinct unit shape alone, as two launches (unshard, then the fused
    # reduce-scatter + Adam through their own entry points), over all units of that shape in order
    per_unit = []
    if not args.no_kernel_timing and not lp_handoff and all(s.W <= 64 for s in states):
        flat0 = torch.empty(max(s.P for s in states), dtype=torch.bfloat16, device="cuda")
        with torch.cuda.stream(main_s):
            seen = []
            for s0 in states:
                if s0.unit_shapes in seen:
                    continue
                seen.append(s0.unit_shapes)
                same = [s for sts in reps_states for s in sts if s.unit_shapes == s0.unit_shapes]

                def unit_pass(s):
                    F.fsdp_unshard(s.lay, s.shard_tab, flat0[:s.P])
                    F.fsdp_reduce_scatter_adam_fused(s.lay, s.grad_tab, rank, pre, post, None, s.shards[rank], s.m, s.v, 2,
                                                     *hp, None)

                for s in same:
                    unit_pass(s)
                n_rep = max(3, min(100, int(25e3 / max(1.0, len(same) * s0.b_total / 6e6))))    # about 25 ms
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(n_rep):
                    for s in same:
                        unit_pass(s)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / n_rep / len(same)
                per_unit.append({"unit": s0.name, "count": len([s for s in states if s.unit_shapes == s0.unit_shapes]),
                                 "bytes_algorithmic": s0.b_total, "gpu_ms": round(us / 1e3, 5),
                                 "gpu_GBps": round(s0.b_total / us / 1e3, 1),
                                 "pct_of_8TBps": round(100 * s0.b_total / us / 1e3 / HBM_PEAK_GBPS, 2),
                                 "launches": 2})
                vlog(f"[bench] {wl.name} unit {s0.name} alone (2 launches): {us:.1f} us, {s0.b_total / us / 1e3:.1f} GB/s")
        del flat0
    rec["units_alone"] = per_unit

    cpu = None
    if first is not None:
        cpu = first.oracle_leg(wl, pre, post, rank, hp)
    # free this workload's HBM before the next one
    del reps_states, reps_launches, states, launches, steps_fns
    gc.collect()
    torch.cuda.empty_cache()
    return rec, cpu


class FirstStepCheck:
    """Headline workload only: keeps the inputs of the first step on the host,
    fetches what the GPU made of them, then times the oracle on the same
    inputs (the `cpu_baseline`) and compares its results with the GPU's."""

    def __init__(self, states, wl, rank, torch):
        import numpy as np
        self.torch, self.np = torch, np
        self.units = []
        for s in states:
            S = s.S
            if wl.grad_dtype == "f32":
                sl = [g[rank * S:(rank + 1) * S].cpu().numpy() for g in s.grads]
            else:
                sl = [g[rank * S:(rank + 1) * S].cpu().view(torch.int16).numpy().view(np.uint16) for g in s.grads]
            self.units.append({"name": s.name, "shards": [x.cpu().numpy() for x in s.shards], "slices": sl,
                               "m": s.m.cpu().numpy(), "v": s.v.cpu().numpy(), "bytes": s.b_total})
        self.gpu = None

    def fetch_gpu(self, states, rank):
        """After step 1 from the initial state: unit 0's updated rank shard and optimizer state."""
        s = states[0]
        self.gpu = {"p": s.shards[rank].cpu().numpy(), "m": s.m.cpu().numpy(), "v": s.v.cpu().numpy()}

    def _pass(self, oracle, u, rank, pre, post, hp):
        t0 = time.perf_counter()
        flat = oracle.unshard_bf16(u["shards"])
        g = oracle.reduce_slices(u["slices"], pre, post)
        res = oracle.adam_f32(u["shards"][rank], g, u["m"], u["v"], 1, *hp)
        dt = time.perf_counter() - t0
        del flat, g
        return dt, res

    def oracle_leg(self, wl, pre, post, rank, hp):
        import oracle
        np = self.np
        budget_s = 12.0
        done, spent, passes = 0, 0.0, 0
        per_unit_ms = []
        ref0 = None
        while spent < budget_s:
            for i, u in enumerate(self.units):
                dt, res = self._pass(oracle, u, rank, pre, post, hp)
                spent += dt
                done += u["bytes"]
                if passes == 0:
                    per_unit_ms.append(round(dt * 1e3, 1))
                    if i == 0:
                        ref0 = res
                del res
            passes += 1
        out = {"value": round(done / spent / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{passes} passes over the {len(self.units)} unit(s) of {wl.name}, {spent:.1f} s",
               "oracle_ms_all_cores": per_unit_ms}
        # the same on one host thread: units in order until about 8 s are spent (reported beside the all-cores figure)
        threads = oracle.num_threads()
        oracle.set_num_threads(1)
        try:
            done, spent, one_thread_ms = 0, 0.0, []
            for u in self.units:
                dt, _res = self._pass(oracle, u, rank, pre, post, hp)
                spent += dt
                done += u["bytes"]
                one_thread_ms.append(round(dt * 1e3, 1))
                if spent > 8.0:
                    break
            out["value_1_thread"] = round(done / spent / 1e9, 3)
            out["oracle_ms_1_core"] = one_thread_ms
        finally:
            oracle.set_num_threads(threads)
        # parity of the GPU's first step (unit 0, the timed rank) with the oracle's first pass
        if self.gpu is not None and ref0 is not None:
            same = all(np.array_equal(np.ascontiguousarray(a).view(np.uint32), np.ascontiguousarray(b).view(np.uint32))
                       for a, b in zip((self.gpu["p"], self.gpu["m"], self.gpu["v"]), ref0))
            out["parity_first_step"] = {"unit": self.units[0]["name"], "rank": rank,
                                        "reduce_scatter+adam": "bit-identical to the oracle" if same else "MISMATCH"}
            assert same, "bench: the first step's update differs from the oracle's"
        return out


def next_rows(args, wl, F, torch, workloads):
    """Hybrid-sharding reduction (Sec. 3.2.2), gradient accumulation
    (Sec. 3.3.4), fp16 / fp32 unshard and the unscaling reduce (Sec. 4.4) on the
    largest unit of the workload: one kernel each, timed back to back over
    rotating buffer sets between one pair of HIP events."""
    unit = max(wl.units, key=lambda u: sum(workloads.numel(s) for s in u.shapes))
    W = wl.world_size
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
        d["p"], d["m"], d["v"] = (torch.zeros(S, device="cuda") for _ in range(3))
        sets.append(d)
    rows = {
        "reduce_scatter_hybrid": (lambda d: F.fsdp_reduce_scatter_hybrid(lay, d["grads"], G, 0, pre, post, d["out"]),
                                  gb * S * W * G + 4 * S),
        "reduce_scatter_hybrid_adam_fused": (lambda d: F.fsdp_reduce_scatter_hybrid_adam_fused(
            lay, d["grads"], G, 0, pre, post, None, d["p"], d["m"], d["v"], 2, wl.lr, wl.beta1, wl.beta2, wl.eps, None),
                                             gb * S * W * G + 4 * S + 28 * S),
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


def main():
    global VERBOSE
    args = parse_args()
    VERBOSE = args.verbose or args.config is not None
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
        probe_copy(args.probe_copy, torch)
        return
    if args.probe_mix:
        probe_mix(torch)
        return
    if args.probe_small:
        probe_small(torch)
        return
    if args.probe_update:
        probe_update(4 if args.config is None else args.config, F, torch, workloads)
        return
    if args.next_rows:
        wl = workloads.config(1 if args.config is None else args.config)
        if args.grad_dtype:
            import dataclasses
            wl = dataclasses.replace(wl, grad_dtype=args.grad_dtype)
        next_rows(args, wl, F, torch, workloads)
        return
    try:
        with open(args.traffic_json) as fh:
            traffic_table = json.load(fh)
    except (OSError, ValueError):
        traffic_table = {}

    cfgs = [args.config] if args.config is not None else list(range(workloads.NUM_CONFIGS))
    head_cfg = args.config if args.config is not None else HEADLINE_CONFIG
    records, cpu = [], None
    for c in cfgs:
        rec, cpu_c = run_config(c, args, F, torch, workloads, c == head_cfg, traffic_table)
        records.append(rec)
        cpu = cpu_c if c == head_cfg else cpu
    ceilings = None if args.no_ceilings else measure_ceilings(torch)
    if ceilings:
        log(f"[bench] ceilings of this box: copy {ceilings['copy_GBps']} GB/s, read-only {ceilings['read_GBps']} GB/s, "
            f"write-only {ceilings['write_GBps']} GB/s, cast (2 bytes read per byte written) {ceilings['cast_GBps']} GB/s; hipMemcpyAsync device-to-device {ceilings['hipMemcpyAsync_d2d_GBps']} GB/s")

    head = next(r for r in records if r["workload"] == workloads.config(head_cfg).name)
    roofline = None
    if head["kernels"]:
        # the kernel with the largest total time per step of the headline workload, under the name rocprofv3 shows
        dom = max(head["kernels"], key=lambda k: head["kernels"][k]["total_us_per_step"])
        k = head["kernels"][dom]
        roofline = {"bound": "hbm", "kernel": dom, "achieved": k["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(k["GBps"] / HBM_PEAK_GBPS, 4), "traffic": k["hbm_bytes_per_launch"],
                    "avg_launch_us": k["avg_us"], "alg_bytes_per_launch": k["alg_bytes_per_launch"],
                    "launches_per_step": k["launches_per_step"],
                    "frac_of_measured_copy": round(k["GBps_touched"] / ceilings["copy_GBps"], 4) if ceilings else None,
                    "frac_of_measured_plain_cast": round(k["GBps_touched"] / ceilings["cast_GBps"], 4) if ceilings else None}
    # per-unit record of the headline workload when it is a single unit (the batch grids of the
    # multi-unit workloads mix units, so only their per-configuration figures exist)
    units_table = None
    if head["units"] == 1:
        hbm = [k["hbm_bytes_per_launch"] for k in head["kernels"].values()]
        units_table = [{
            "unit": workloads.config(head_cfg).units[0].name, "bytes_algorithmic": head["alg_bytes_per_step"],
            "gpu_ms": round(head["us_per_step"] / 1e3, 4), "gpu_GBps": head["GBps"], "pct_of_8TBps": head["pct_of_hbm_peak"],
            "rocprof_bytes": sum(hbm) if hbm and all(h is not None for h in hbm) else None,
            "oracle_ms_all_cores": cpu["oracle_ms_all_cores"][0] if cpu else None,
            "oracle_ms_1_core": cpu["oracle_ms_1_core"][0] if cpu and cpu.get("oracle_ms_1_core") else None,
            "host_cores": cpu["cores"] if cpu else None,
            "parity": cpu.get("parity_first_step") if cpu else None,
        }]
    out = {
        "metric": "effective HBM GB/s (and % of peak) per FSDP unit: unshard + reduce-scatter + Adam",
        "value": head["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["us_per_step"] / 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "units", "world_size", "grad_dtype", "unshard_dtype", "rank", "mode",
                                        "reshard_after_forward", "prefetch_depth", "hip_graph", "launches_per_step",
                                        "buffer_replicas", "alg_bytes_per_step", "touched_bytes_per_step")},
        "pct_of_hbm_peak": head["pct_of_hbm_peak"],
        "ms_per_step_min": round(head["us_per_step_min"] / 1e3, 5),
        "ms_per_step_median": round(head["us_per_step_median"] / 1e3, 5),
        "roofline": roofline, "cpu_baseline": cpu, "measured_ceilings": ceilings, "units_table": units_table,
        "kernels": head["kernels"], "configs": records,
    }
    # Everything measured goes to a file; the ONE line on stdout is a compact view of it (harnesses keep
    # only the tail of a run's output).
    if args.detail_json:
        try:
            os.makedirs(os.path.dirname(os.path.abspath(args.detail_json)), exist_ok=True)
            with open(args.detail_json, "w") as fh:
                json.dump(out, fh, indent=1)
        except OSError as e:
            log(f"[bench] could not write {args.detail_json}: {e}")
    print(json.dumps(compact(out), separators=(",", ":")), flush=True)


def compact(out):
    """The JSON line: the contract's keys in full, per-kernel and per-configuration records reduced to their figures."""
    def kern(ks):
        return {k: {"n": v["launches_per_step"], "avg_us": v["avg_us"], "GBps": v["GBps"], "GBps_touched": v["GBps_touched"],
                    "hbm_bytes": v["hbm_bytes_per_launch"]} for k, v in ks.items()}
    line = dict(out)
    line["config"] = {k: out["config"][k] for k in ("workload", "units", "world_size", "grad_dtype", "mode",
                                                    "launches_per_step", "alg_bytes_per_step", "touched_bytes_per_step")}
    if out["measured_ceilings"]:
        line["measured_ceilings"] = {k: out["measured_ceilings"][k] for k in ("copy_GBps", "read_GBps", "write_GBps", "cast_GBps",
                                                                                 "hipMemcpyAsync_d2d_GBps")}
    line["kernels"] = kern(out["kernels"])
    if out["units_table"]:
        line["units_table"] = [{k: (v["reduce_scatter+adam"] if k == "parity" and isinstance(v, dict) else v)
                                for k, v in u.items()} for u in out["units_table"]]
    line["configs"] = []
    for c in out["configs"]:
        r = {"workload": c["workload"], "us_per_step": c["us_per_step"], "us_min": c["us_per_step_min"],
             "us_median": c["us_per_step_median"], "GBps": c["GBps"], "pct_of_hbm_peak": c["pct_of_hbm_peak"],
             "launches": c["launches_per_step"], "kernel_us": {k: v["avg_us"] for k, v in c["kernels"].items()}}
        if c.get("warm_one_replica"):
            r["cold_replicas"] = c["buffer_replicas"]
            r["warm_us_median"] = c["warm_one_replica"]["us_per_step_median"]
        if c.get("note"):
            r["note"] = "launch-bound (two dependent launches)"
        line["configs"].append(r)
    return line


if __name__ == "__main__":
    main()
