"""GPU parity at the benchmark's full sizes: each distinct unit shape of the
five configurations, through the same entry points and launch configuration
bench.py times, compared element by element with the CPU oracle.

Inputs are generated once on the device from the seeded workload module and
copied to the host bit for bit; for the two largest configurations the host
receives only the rank's slice of every rank's gradient buffer, which is all
the reduce-scatter's rank share reads."""
import gc

import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import assert_adam_parity, first_diff, load_product, np_bits, np_f32, same_bits

pytestmark = pytest.mark.gpu

BENCH_RANK = 0      # the rank bench.py times
BENCH_DEPTH = 6     # bench.py's default --depth

CASES = [(c, u) for c in range(workloads.NUM_CONFIGS) for u in workloads.config(c).distinct_units]


def _ranks(cfg, W):
    return list(range(W)) if cfg <= 2 else [0, 1, W - 1]


@pytest.fixture(scope="module")
def F():
    assert torch.cuda.is_available()
    return load_product()


@pytest.mark.parametrize("cfg,unit_index", CASES, ids=[f"cfg{c}-unit{u}" for c, u in CASES])
def test_config_unit_matches_oracle(F, cfg, unit_index):
    wl = workloads.config(cfg)
    unit = wl.units[unit_index]
    W = wl.world_size
    hp = (wl.lr, wl.beta1, wl.beta2, wl.eps)
    print(f"\n[case] {wl.name} unit {unit.name} W={W}", flush=True)
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    off_ref, N_ref, S_ref, P_ref, pad_ref = oracle.layout(unit.shapes, W)
    assert (N, S, P, lay.pad) == (N_ref, S_ref, P_ref, pad_ref)

    # ---- flatten + pad + shard (contiguous shards: base + w*S, as bench.py lays them out)
    params = workloads.gen_params(unit, unit_index, device="cuda")
    base = torch.empty(W * S, dtype=torch.float32, device="cuda")
    base.view(torch.int32).fill_(0x7FC00001)
    shards = [base[w * S:(w + 1) * S] for w in range(W)]
    F.fsdp_flatten_shard(lay, params, shards)
    torch.cuda.synchronize()
    h_params = [np_f32(p) for p in params]
    del params
    h_shards, _ = oracle.flatten_shard(h_params, W)
    del h_params
    got = np_bits(base)
    ref = np.concatenate(h_shards).view(np.uint32)
    assert same_bits(got, ref), "flatten_shard: " + first_diff(got, ref)
    del got, ref
    print("[step] flatten_shard bit-exact", flush=True)

    # ---- unshard: cast + gather into the bf16 flat buffer, and the views
    flat = torch.empty(P, dtype=torch.bfloat16, device="cuda")
    flat.view(torch.int16).fill_(0x7FCD)
    F.fsdp_unshard(lay, shards, flat)
    torch.cuda.synchronize()
    ref = oracle.unshard_bf16(h_shards)
    got = np_bits(flat)
    assert same_bits(got, ref), "unshard: " + first_diff(got, ref)
    views = F.fsdp_views(lay, flat)
    assert [tuple(v.shape) for v in views] == [tuple(s) for s in unit.shapes]
    for i, v in enumerate(views):
        assert v.data_ptr() == flat.data_ptr() + 2 * off_ref[i]
    del got, ref, views, flat
    print("[step] unshard bit-exact", flush=True)

    # ---- gradients of the W simulated ranks
    gdt = torch.float32 if wl.grad_dtype == "f32" else torch.bfloat16
    grads = []
    for w in range(W):
        g = torch.empty(P, dtype=gdt, device="cuda")
        workloads.gen_rank_grad(P, N, w, unit_index, wl.grad_dtype, device="cuda", outlier_frac=wl.outlier_frac,
                                outlier_scale=wl.outlier_scale, out=g)
        grads.append(g)
    torch.cuda.synchronize()

    gs = torch.empty(S, dtype=torch.float32, device="cuda")
    for r in _ranks(cfg, W):
        if gdt == torch.float32:
            h_slices = [np_f32(g[r * S:(r + 1) * S]) for g in grads]
        else:
            h_slices = [np_bits(g[r * S:(r + 1) * S]) for g in grads]
        ref_g = oracle.reduce_slices(h_slices, pre, post)
        del h_slices
        gs.view(torch.int32).fill_(0x7FC00001)
        F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, gs)
        torch.cuda.synchronize()
        got = np_bits(gs)
        assert same_bits(got, ref_g.view(np.uint32)), f"reduce-scatter rank {r}: " + first_diff(got, ref_g.view(np.uint32))

        # Adam on this rank's shard, first step from zero state; then the fused call from the same start
        p = shards[r].clone()
        m = torch.zeros(S, device="cuda")
        v = torch.zeros(S, device="cuda")
        F.fsdp_shard_adam_step(lay, p, gs, m, v, 1, *hp)
        p2 = shards[r].clone()
        m2 = torch.zeros(S, device="cuda")
        v2 = torch.zeros(S, device="cuda")
        F.fsdp_reduce_scatter_adam_fused(lay, grads, r, pre, post, None, p2, m2, v2, 1, *hp, None)
        torch.cuda.synchronize()
        z = np.zeros(S, np.float32)
        gp, gm, gv = np_f32(p), np_f32(m), np_f32(v)
        rp, rm, rv = assert_adam_parity(gp, gm, gv, h_shards[r], ref_g, z, z, 1, hp, f"Adam rank {r}")
        for a, b, n in ((p, p2, "p"), (m, m2, "m"), (v, v2, "v")):
            assert same_bits(np_bits(a), np_bits(b)), f"fused {n} differs from the two-call path at rank {r}"
        if lay.pad and r == W - 1:
            assert not np_bits(p)[S - lay.pad:].any()
        if r == BENCH_RANK:
            bench_ref = (rp.copy(), rm.copy(), rv.copy(), np_bits(p2).copy(), np_bits(m2).copy(), np_bits(v2).copy())
            # both rank walks forced through the layout (one of them is the library's own choice): same bits
            for walk in (F.FSDP_WALK_WIDE, F.FSDP_WALK_DEEP, F.FSDP_WALK_HALF):
                lay_w = F.fsdp_layout_init(unit.shapes, W, reduce_walk=walk)
                p3, m3, v3 = shards[r].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
                F.fsdp_reduce_scatter_adam_fused(lay_w, grads, r, pre, post, None, p3, m3, v3, 1, *hp, None)
                torch.cuda.synchronize()
                for a, b, n in ((p3, p2, "p"), (m3, m2, "m"), (v3, v2, "v")):
                    assert same_bits(np_bits(a), np_bits(b)), f"{n}: rank walk {walk} differs at rank {r}"
                del p3, m3, v3
        print(f"[step] rank {r}: reduce-scatter bit-exact, Adam bit-identical to the fp32 oracle and within 1e-6 of "
              f"the fp64 one, fused == two calls", flush=True)
        del p, m, v, p2, m2, v2, rp, rm, rv, gp, gm, gv, ref_g

    # ---- the launch configuration bench.py times by default: one batch holding the fused
    # reduce-scatter + Adam of `depth` units and the unshards of `depth` units (here: copies of this unit)
    rp, rm, rv, p2b, m2b, v2b = bench_ref
    ref_flat = oracle.unshard_bf16(h_shards)
    batch = F.Batch()
    outs = []
    for _ in range(BENCH_DEPTH):
        pb, mb, vb = shards[BENCH_RANK].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
        batch.add_reduce_scatter_adam(lay, grads, BENCH_RANK, pre, post, None, pb, mb, vb, *hp, None)
        outs.append((pb, mb, vb))
    flats = []
    for _ in range(BENCH_DEPTH):
        fb = torch.empty(P, dtype=torch.bfloat16, device="cuda")
        fb.view(torch.int16).fill_(0x7FCD)
        batch.add_unshard(lay, shards, fb)
        flats.append(fb)
    batch.launch(1)
    torch.cuda.synchronize()
    for j, (pb, mb, vb) in enumerate(outs):
        for a, b, n in ((pb, rp, "p"), (mb, rm, "m"), (vb, rv, "v")):
            assert same_bits(np_bits(a), b.view(np.uint32)), f"batch update {j}: {n} differs from the fp32 oracle"
        for a, b, n in ((pb, p2b, "p"), (mb, m2b, "m"), (vb, v2b, "v")):
            assert same_bits(np_bits(a), b), f"batch update {j}: {n} differs from the fused call"
    for j, fb in enumerate(flats):
        got = np_bits(fb)
        assert same_bits(got, ref_flat), f"batch unshard {j}: " + first_diff(got, ref_flat)
    print(f"[step] batch of {BENCH_DEPTH}+{BENCH_DEPTH} operations: updates bit-identical to the fp32 oracle and to "
          "the fused call, unshards bit-exact", flush=True)
    batch.close()
    del outs, flats, batch, ref_flat, bench_ref
    del grads, shards, base, h_shards
    gc.collect()
    torch.cuda.empty_cache()


def _poisoned(n, dtype):
    t = torch.empty(n, dtype=dtype, device="cuda")
    t.view(torch.int16 if dtype in (torch.bfloat16, torch.float16) else torch.int32).fill_(
        0x7FCD if dtype in (torch.bfloat16, torch.float16) else 0x7FC00001)
    return t


@pytest.mark.parametrize("cfg,unit_index", CASES, ids=[f"cfg{c}-unit{u}" for c, u in CASES])
def test_config_unit_variants_match_oracle(F, cfg, unit_index):
    """The variants of the path that bench.py also times, at the unit's full
    size: the other gradient dtype (under the rank walk the library chooses at
    that size), the fp32 and fp16 unshard (Sec. 3.2.1, 4.4), the bf16 shard
    hand-off as batch members (Sec. 4.4), and the hybrid (Sec. 3.2.2),
    accumulate (Sec. 3.3.4) and unscale (Sec. 4.4) forms of the reduce-scatter."""
    wl = workloads.config(cfg)
    unit = wl.units[unit_index]
    W = wl.world_size
    hp = (wl.lr, wl.beta1, wl.beta2, wl.eps)
    r = BENCH_RANK
    print(f"\n[case] variants of {wl.name} unit {unit.name} W={W}", flush=True)
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    params = workloads.gen_params(unit, unit_index, device="cuda")
    base = torch.empty(W * S, dtype=torch.float32, device="cuda")
    shards = [base[w * S:(w + 1) * S] for w in range(W)]
    F.fsdp_flatten_shard(lay, params, shards)
    torch.cuda.synchronize()
    del params
    h_shards = [np_f32(s) for s in shards]          # flatten_shard itself is compared with the oracle in the test above

    # ---- unshard to fp32 and to fp16
    for dt, ref_fn in ((torch.float32, oracle.unshard_f32), (torch.float16, oracle.unshard_f16)):
        flat = _poisoned(P, dt)
        F.fsdp_unshard(lay, shards, flat)
        torch.cuda.synchronize()
        ref = ref_fn(h_shards)
        got = np_bits(flat)
        ref = ref.view(np.uint32) if ref.dtype == np.float32 else ref
        assert same_bits(got, ref), f"unshard to {dt}: " + first_diff(got, ref)
        del flat, got, ref
    print("[step] unshard to fp32 and fp16 bit-exact", flush=True)

    # ---- the other gradient dtype: fused reduce-scatter + Adam with both optional outputs, rank 0
    other = "bf16" if wl.grad_dtype == "f32" else "f32"
    odt = torch.bfloat16 if other == "bf16" else torch.float32
    grads = []
    for w in range(W):
        g = torch.empty(P, dtype=odt, device="cuda")
        workloads.gen_rank_grad(P, N, w, unit_index, other, device="cuda", outlier_frac=wl.outlier_frac,
                                outlier_scale=wl.outlier_scale, out=g)
        grads.append(g)
    torch.cuda.synchronize()
    h_slices = [(np_f32 if other == "f32" else np_bits)(g[r * S:(r + 1) * S]) for g in grads]
    ref_g = oracle.reduce_slices(h_slices, pre, post)
    p, m, v = shards[r].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
    g_out, lp_out = _poisoned(S, torch.float32), _poisoned(S, torch.bfloat16)
    F.fsdp_reduce_scatter_adam_fused(lay, grads, r, pre, post, g_out, p, m, v, 1, *hp, lp_out)
    torch.cuda.synchronize()
    got = np_bits(g_out)
    assert same_bits(got, ref_g.view(np.uint32)), f"{other} gradients, reduce-scatter: " + first_diff(got, ref_g.view(np.uint32))
    z = np.zeros(S, np.float32)
    rp, _, _ = assert_adam_parity(np_f32(p), np_f32(m), np_f32(v), h_shards[r], ref_g, z, z, 1, hp, f"{other} gradients")
    assert same_bits(np_bits(lp_out), oracle.cast_bf16(rp)), "bf16 copy of the updated shard"
    for walk in (F.FSDP_WALK_WIDE, F.FSDP_WALK_DEEP, F.FSDP_WALK_HALF):
        lay_w = F.fsdp_layout_init(unit.shapes, W, reduce_walk=walk)
        p3, m3, v3 = shards[r].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
        F.fsdp_reduce_scatter_adam_fused(lay_w, grads, r, pre, post, None, p3, m3, v3, 1, *hp, None)
        torch.cuda.synchronize()
        for a, b, n in ((p3, p, "p"), (m3, m, "m"), (v3, v, "v")):
            assert same_bits(np_bits(a), np_bits(b)), f"{other} gradients, {n}: rank walk {walk} differs"
        del p3, m3, v3
    print(f"[step] {other} gradients: reduce-scatter bit-exact, Adam bit-identical (both rank walks), bf16 copy of the "
          "new shard bit-exact", flush=True)

    # ---- the same update and the gather of the ranks' bf16 shards as members of one batch (bench.py --mode batch-lp)
    lp_base = _poisoned(W * S, torch.bfloat16)
    lps = [lp_base[w * S:(w + 1) * S] for w in range(W)]
    for w in range(W):
        F.fsdp_cast_shard(lay, shards[w], lps[w])
    torch.cuda.synchronize()
    h_lps = [oracle.cast_bf16(h) for h in h_shards]
    assert same_bits(np_bits(lp_base), np.concatenate(h_lps)), "cast_shard"
    p2, m2, v2 = shards[r].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
    flat = _poisoned(P, torch.bfloat16)
    b_upd, b_gather = F.Batch(), F.Batch()
    b_upd.add_reduce_scatter_adam(lay, grads, r, pre, post, None, p2, m2, v2, *hp, lps[r])
    b_gather.add_unshard_lp(lay, lps, flat)
    b_upd.launch(1)
    b_gather.launch(1)
    torch.cuda.synchronize()
    for a, b, n in ((p2, p, "p"), (m2, m, "m"), (v2, v, "v")):
        assert same_bits(np_bits(a), np_bits(b)), f"batch member: {n} differs from the fused call"
    h_lps[r] = oracle.cast_bf16(rp)
    ref = oracle.gather_lp(h_lps)
    got = np_bits(flat)
    assert same_bits(got, ref), "gather of the bf16 shards after the update: " + first_diff(got, ref)
    b_upd.close()
    b_gather.close()
    del flat, lp_base, lps, h_lps, p2, m2, v2, got, ref
    print("[step] bf16 shard hand-off as batch members bit-exact", flush=True)

    # ---- accumulate (out += reduce-scatter) and unscale (+ the non-finite flag) on the same gradients
    acc0 = torch.empty(S, device="cuda").normal_(0.0, 1e-3, generator=torch.Generator(device="cuda").manual_seed(7))
    h_acc0 = np_f32(acc0).copy()
    F.fsdp_reduce_scatter_accumulate(lay, grads, r, pre, post, acc0)
    torch.cuda.synchronize()
    ref = oracle.accumulate(h_acc0, ref_g)
    assert same_bits(np_bits(acc0), ref.view(np.uint32)), "accumulate: " + first_diff(np_bits(acc0), ref.view(np.uint32))
    flag = torch.zeros(1, device="cuda")
    out = _poisoned(S, torch.float32)
    inv_scale = 1.0 / 1024.0
    F.fsdp_reduce_scatter_unscale(lay, grads, r, pre, post, inv_scale, out, flag)
    torch.cuda.synchronize()
    ref, ref_flag = oracle.unscale_check(ref_g, inv_scale)
    assert same_bits(np_bits(out), ref.view(np.uint32)) and float(flag.item()) == ref_flag == 0.0, "unscale"
    # one Inf in the last element of one rank's slice: the flag must come up
    k = r * S + S - 1
    saved = grads[W // 2][k].clone()
    grads[W // 2][k] = float("inf")
    F.fsdp_reduce_scatter_unscale(lay, grads, r, pre, post, inv_scale, out, flag)
    torch.cuda.synchronize()
    grads[W // 2][k] = saved
    assert float(flag.item()) == 1.0, "a non-finite sum in the last element must set the flag"
    # the last micro-batch of an accumulation: accumulate and step in one launch
    acc1 = torch.from_numpy(h_acc0).cuda()
    p4, m4, v4 = shards[r].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
    F.fsdp_reduce_scatter_accumulate_adam_fused(lay, grads, r, pre, post, acc1, p4, m4, v4, 1, *hp, None)
    torch.cuda.synchronize()
    ref_acc = oracle.accumulate(h_acc0, ref_g)
    assert same_bits(np_bits(acc1), ref_acc.view(np.uint32)), "accumulate + Adam: the accumulated gradient"
    assert_adam_parity(np_f32(p4), np_f32(m4), np_f32(v4), h_shards[r], ref_acc, z, z, 1, hp, "accumulate + Adam")
    del acc0, acc1, p4, m4, v4, out, ref, ref_acc
    print("[step] accumulate (also fused with Adam) and unscale bit-exact", flush=True)

    # ---- hybrid sharding: two sharded groups of W ranks (more than 64 ranks in all go out as one launch
    # per group); the second group holds the same buffers in reverse rank order, so the inner sums differ
    # between the groups
    table = list(grads) + list(reversed(grads))
    pre_h, post_h = F.fsdp_default_divide_factors(2 * W)
    out = _poisoned(S, torch.float32)
    F.fsdp_reduce_scatter_hybrid(lay, table, 2, r, pre_h, post_h, out)
    torch.cuda.synchronize()
    sl = h_slices + h_slices[::-1]
    ref = oracle.reduce_slices_hybrid(sl, 2, W, pre_h, post_h)
    assert same_bits(np_bits(out), ref.view(np.uint32)), "hybrid: " + first_diff(np_bits(out), ref.view(np.uint32))
    # the same reduction with the Adam step in the launch
    p5, m5, v5 = shards[r].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
    out2 = _poisoned(S, torch.float32)
    F.fsdp_reduce_scatter_hybrid_adam_fused(lay, table, 2, r, pre_h, post_h, out2, p5, m5, v5, 1, *hp, None)
    torch.cuda.synchronize()
    assert same_bits(np_bits(out2), ref.view(np.uint32)), "hybrid + Adam: the reduced gradient"
    assert_adam_parity(np_f32(p5), np_f32(m5), np_f32(v5), h_shards[r], ref, z, z, 1, hp, "hybrid + Adam")
    print(f"[step] hybrid reduce-scatter (2 groups of {W}), alone and fused with Adam, bit-exact", flush=True)
    del p5, m5, v5, out2
    del grads, table, sl, out, ref, shards, base, h_shards, h_slices
    gc.collect()
    torch.cuda.empty_cache()


def test_unit_with_more_than_2_31_elements(F):
    """Maximum-size edge: element indices and byte offsets beyond 32 bits in
    every kernel (N = 2^31 + 12345 over two ranks, odd N so the last rank holds
    one pad element and rank 1's shard is only 4-byte aligned)."""
    W = 2
    shapes = [(1 << 31,), (12345,)]
    lay = F.fsdp_layout_init(shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    off_ref, N_ref, S_ref, P_ref, pad_ref = oracle.layout(shapes, W)
    assert (N, S, P, lay.pad) == (N_ref, S_ref, P_ref, pad_ref) == ((1 << 31) + 12345, (1 << 30) + 6173, (1 << 31) + 12346, 1)
    print(f"\n[case] 2^31+12345 elements, W={W}, S={S}", flush=True)

    gen = torch.Generator(device="cuda")
    gen.manual_seed(workloads.BASE_SEED)
    params = [torch.empty(s, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=gen) for s in shapes]
    base = torch.empty(P, dtype=torch.float32, device="cuda")
    base.view(torch.int32).fill_(0x7FC00001)
    shards = [base[w * S:(w + 1) * S] for w in range(W)]
    F.fsdp_flatten_shard(lay, params, shards)
    torch.cuda.synchronize()
    h_params = [np_f32(p) for p in params]
    del params
    h_shards, _ = oracle.flatten_shard(h_params, W)
    del h_params
    for w in range(W):
        got = np_bits(shards[w])
        assert same_bits(got, h_shards[w].view(np.uint32)), f"flatten_shard rank {w}: " + first_diff(got, h_shards[w].view(np.uint32))
    print("[step] flatten_shard bit-exact", flush=True)

    flat = torch.empty(P, dtype=torch.bfloat16, device="cuda")
    flat.view(torch.int16).fill_(0x7FCD)
    F.fsdp_unshard(lay, shards, flat)
    torch.cuda.synchronize()
    ref = oracle.unshard_bf16(h_shards)
    got = np_bits(flat)
    assert same_bits(got, ref), "unshard: " + first_diff(got, ref)
    views = F.fsdp_views(lay, flat)
    assert views[1].data_ptr() == flat.data_ptr() + 2 * (1 << 31) and tuple(views[1].shape) == (12345,)
    del got, ref, flat, views
    print("[step] unshard bit-exact", flush=True)

    grads = [workloads.gen_rank_grad(P, N, w, 0, "bf16", device="cuda") for w in range(W)]
    pre, post = F.fsdp_default_divide_factors(W)
    hp = (1e-4, 0.9, 0.999, 1e-8)
    r = W - 1                                  # the slice that starts beyond 2^30 elements and ends with the pad
    h_slices = [np_bits(g[r * S:(r + 1) * S]) for g in grads]
    ref_g = oracle.reduce_slices(h_slices, pre, post)
    del h_slices
    gs = torch.empty(S, dtype=torch.float32, device="cuda")
    gs.view(torch.int32).fill_(0x7FC00001)
    F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, gs)
    p2, m2, v2 = shards[r].clone(), torch.zeros(S, device="cuda"), torch.zeros(S, device="cuda")
    F.fsdp_reduce_scatter_adam_fused(lay, grads, r, pre, post, None, p2, m2, v2, 1, *hp, None)
    torch.cuda.synchronize()
    got = np_bits(gs)
    assert same_bits(got, ref_g.view(np.uint32)), "reduce-scatter: " + first_diff(got, ref_g.view(np.uint32))
    del got, gs, grads
    z = np.zeros(S, np.float32)
    assert_adam_parity(np_f32(p2), np_f32(m2), np_f32(v2), h_shards[r], ref_g, z, z, 1, hp, "fused update")
    assert not np_bits(p2)[S - 1:].any(), "the pad element must stay zero"
    print("[step] reduce-scatter bit-exact, fused update bit-identical to the fp32 oracle", flush=True)
    del p2, m2, v2, shards, base, h_shards
    gc.collect()
    torch.cuda.empty_cache()
