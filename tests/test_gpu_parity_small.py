"""GPU parity, small and ragged cases: the HIP path (through the C ABI) against
the CPU oracle, element by element, on sizes that span several tiles and a
ragged tail.  Bit-exact for pack / gather / cast / reduce; Adam within 1e-6."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import (POISON16, POISON32, assert_adam_bits, assert_adam_parity, carve, first_diff, load_product, np_bits, np_f32, np_grad,
                         same_bits)

pytestmark = pytest.mark.gpu

LR, B1, B2, EPS = 1e-4, 0.9, 0.999, 1e-8

EDGE_BITS = [0x00000000, 0x80000000, 0x3F800000, 0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x7F7F8000,
             0x7F7F7FFF, 0xFF7F8000, 0x00008000, 0x00018000, 0x00008001, 0x00000001, 0x807FFFFF, 0x7F800000,
             0xFF800000, 0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF80FFFF, 0x7FA00000, 0x7FFFFFFF]


@pytest.fixture(scope="module")
def F():
    assert torch.cuda.is_available()
    return load_product()


def big_unit():
    """Several tiles per shard, a ragged tail, more than one pack-launch worth of
    parameters, and edge-value content."""
    shapes = [(len(EDGE_BITS),), (257, 129), (1,), (), (0, 3), (100003,), (64, 64), (7,)]
    shapes += [(i + 1,) for i in range(40)] + [(333, 77), (5, 5, 5), (20011,)]
    return workloads.Unit("big_ragged", tuple(shapes))


def make_params(unit, seed, misalign):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    out = []
    for i, shp in enumerate(unit.shapes):
        n = workloads.numel(shp)
        t = carve(n, torch.float32, (i % 4) if misalign else 0)
        if n:
            t.normal_(0.0, 0.02, generator=g)
        out.append(t.view(shp) if n else torch.empty(shp, dtype=torch.float32, device="cuda"))
    if unit.shapes[0] == (len(EDGE_BITS),):
        out[0].copy_(torch.tensor(np.array(EDGE_BITS, dtype=np.uint32).view(np.float32)))
    return out


def alloc_shards(W, S, mode):
    """mode: 'separate' (each its own allocation), 'contig' (base + w*S),
    'contig_odd' (base + 1 + w*S: only element-aligned)."""
    if mode == "separate":
        return [carve(S, torch.float32, 0, fill=POISON32) for _ in range(W)], None
    off = 1 if mode == "contig_odd" else 0
    base = carve(W * S, torch.float32, off, fill=POISON32)
    return [base[w * S:(w + 1) * S] for w in range(W)], base


@pytest.mark.parametrize("W", [1, 2, 3, 7, 8, 12, 64, 100])
@pytest.mark.parametrize("mode", ["separate", "contig", "contig_odd"])
def test_flatten_shard_and_unshard(F, W, mode):
    unit = big_unit() if W <= 12 else workloads.ragged_unit()
    params = make_params(unit, 1234 + W, misalign=(mode != "separate"))
    lay = F.fsdp_layout_init(unit.shapes, W)
    shards, _ = alloc_shards(W, lay.shard, mode)
    F.fsdp_flatten_shard(lay, params, shards)
    torch.cuda.synchronize()
    ref_shards, (off, N, S, P, pad) = oracle.flatten_shard([np_f32(p) for p in params], W)
    assert (lay.numel, lay.shard, lay.padded, lay.pad) == (N, S, P, pad)
    for w in range(W):
        got = np_bits(shards[w])
        assert same_bits(got, ref_shards[w].view(np.uint32)), f"shard {w}: {first_diff(got, ref_shards[w].view(np.uint32))}"

    # unshard, bf16 (cast + gather) and fp32 (gather), destination aligned and not
    for dst_off in (0, 1, 3):
        flat_lp = carve(P, torch.bfloat16, dst_off, fill=POISON16)
        F.fsdp_unshard(lay, shards, flat_lp)
        flat_fp = carve(P, torch.float32, dst_off, fill=POISON32)
        F.fsdp_unshard(lay, shards, flat_fp)
        torch.cuda.synchronize()
        ref_lp = oracle.unshard_bf16(ref_shards)
        ref_fp = oracle.unshard_f32(ref_shards)
        assert same_bits(np_bits(flat_lp), ref_lp), first_diff(np_bits(flat_lp), ref_lp)
        assert same_bits(np_bits(flat_fp), ref_fp.view(np.uint32)), first_diff(np_bits(flat_fp), ref_fp.view(np.uint32))

    # views (Sec. 3.2.3): zero copy, original shapes, flatten o unflatten = identity
    views_fp = F.fsdp_views(lay, flat_fp)
    views_lp = F.fsdp_views(lay, flat_lp)
    for i, (v, p) in enumerate(zip(views_fp, params)):
        assert tuple(v.shape) == tuple(p.shape)
        if v.numel():
            assert v.data_ptr() == flat_fp.data_ptr() + 4 * off[i]
            assert views_lp[i].data_ptr() == flat_lp.data_ptr() + 2 * off[i]
        assert same_bits(np_bits(v), np_bits(p))
        assert same_bits(np_bits(views_lp[i]).reshape(-1), oracle.cast_bf16(np_f32(p)).reshape(-1))


def make_grads(W, P, N, dtype, seed, outliers=False, elem_offset=0):
    grads = []
    for w in range(W):
        t = carve(P, dtype, elem_offset)
        workloads.gen_rank_grad(P, N, w, 0, "bf16" if dtype == torch.bfloat16 else "f32", device="cuda", seed=seed,
                                outlier_frac=0.01 if outliers else 0.0, outlier_scale=1e3, out=t)
        grads.append(t)
    return grads


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("W,pre,post", [(1, 1.0, 1.0), (2, 2.0, 1.0), (3, 1.0, 3.0), (3, 3.0, 1.0), (8, 4.0, 2.0),
                                        (12, 4.0, 3.0), (16, 4.0, 4.0), (64, 8.0, 8.0), (70, 2.0, 35.0),
                                        (130, 1.0, 130.0), (5, 2.5, 2.0)])
def test_reduce_scatter_bit_exact(F, gdt, W, pre, post):
    unit = workloads.ragged_unit() if W > 16 else big_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    grads = make_grads(W, P, N, gdt, 99 + W, outliers=True, elem_offset=(1 if W % 2 else 0))
    # special values in rank 0 / all ranks: signed zeros, a denormal, a large value
    for w, g in enumerate(grads):
        g[:4] = torch.tensor([-0.0, -0.0 if w != 1 else 0.0, 1e-40, 3e38 if w < 2 else 0.0], dtype=gdt)
    host = [np_grad(g) for g in grads]
    ranks = range(W) if W <= 16 else (0, 1, W // 2, W - 1)
    for r in ranks:
        out = carve(S, torch.float32, r % 3, fill=POISON32)
        F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, out)
        torch.cuda.synchronize()
        ref = oracle.reduce_scatter(host, r, pre, post)
        got = np_bits(out)
        assert same_bits(got, ref.view(np.uint32)), f"rank {r}: {first_diff(got, ref.view(np.uint32))}"


def test_reduce_order_witness_on_gpu(F):
    """((1e8 + 1) - 1e8) + 1 = 1 only in strict rank order."""
    lay = F.fsdp_layout_init([(4000,)], 4)
    vals = [1e8, 1.0, -1e8, 1.0]
    grads = [torch.full((lay.padded,), v, dtype=torch.float32, device="cuda") for v in vals]
    out = torch.empty(lay.shard, dtype=torch.float32, device="cuda")
    F.fsdp_reduce_scatter_local(lay, grads, 2, 1.0, 1.0, out)
    torch.cuda.synchronize()
    assert bool((out == 1.0).all())


def _adam_state(S, t, seed, offs=(0, 0, 0, 0)):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    p = carve(S, torch.float32, offs[0]).normal_(0, 0.02, generator=g)
    gr = carve(S, torch.float32, offs[1]).normal_(0, 1e-3, generator=g)
    m = carve(S, torch.float32, offs[2])
    v = carve(S, torch.float32, offs[3])
    if t > 1:
        m.normal_(0, 1e-3, generator=g)
        v.uniform_(0, 1e-6, generator=g)
    else:
        m.zero_()
        v.zero_()
    return p, gr, m, v


@pytest.mark.parametrize("t", [1, 2, 7, 1000])
@pytest.mark.parametrize("S,offs", [(1, (0, 0, 0, 0)), (5, (1, 2, 3, 0)), (4099, (0, 0, 0, 0)), (100003, (3, 1, 0, 2)),
                                    (262144, (0, 0, 0, 0))])
def test_adam_step(F, t, S, offs):
    lay = F.fsdp_layout_init([(S,)], 1)
    p, g, m, v = _adam_state(S, t, 5 + t + S, offs)
    g[:1] = 0.0
    # a quarter of the shard starts at p = 0 and another at |p| <= lr: there the tolerance is a bound on the
    # update itself (2e-6 of it), which tells the Adam reading taken from its neighbours
    p[S // 4: S // 2] = 0.0
    p[S // 2: 3 * S // 4] *= 5e-3
    hp, hg, hm, hv = (np_f32(x).copy() for x in (p, g, m, v))
    F.fsdp_shard_adam_step(lay, p, g, m, v, t, LR, B1, B2, EPS)
    torch.cuda.synchronize()
    assert_adam_parity(np_f32(p), np_f32(m), np_f32(v), hp, hg, hm, hv, t, (LR, B1, B2, EPS), "adam_step")
    assert same_bits(np_bits(g), hg.view(np.uint32))            # the gradient is not modified


def test_adam_pad_stays_zero_and_is_deterministic(F):
    S = 10007
    lay = F.fsdp_layout_init([(S,)], 1)
    p, g, m, v = _adam_state(S, 1, 77)
    p[-5:] = 0.0
    g[-5:] = 0.0
    snap = [x.clone() for x in (p, g, m, v)]
    F.fsdp_shard_adam_step(lay, p, g, m, v, 1, LR, B1, B2, EPS)
    torch.cuda.synchronize()
    assert not np_bits(p)[-5:].any() and not np_bits(m)[-5:].any() and not np_bits(v)[-5:].any()
    p2, g2, m2, v2 = snap
    F.fsdp_shard_adam_step(lay, p2, g2, m2, v2, 1, LR, B1, B2, EPS)
    torch.cuda.synchronize()
    assert same_bits(np_bits(p), np_bits(p2)) and same_bits(np_bits(m), np_bits(m2)) and same_bits(np_bits(v), np_bits(v2))


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("W", [3, 8, 70])
@pytest.mark.parametrize("with_outputs", [True, False])
def test_fused_reduce_scatter_adam_equals_two_calls(F, gdt, W, with_outputs):
    unit = big_unit() if W <= 8 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    grads = make_grads(W, P, N, gdt, 300 + W)
    r = W - 1
    t = 3
    p, _, m, v = _adam_state(S, t, 17, (1, 0, 2, 3))
    p2, m2, v2 = p.clone(), m.clone(), v.clone()
    hp, hm, hv = (np_f32(x).copy() for x in (p, m, v))
    # two calls
    gs = torch.empty(S, dtype=torch.float32, device="cuda")
    F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, gs)
    F.fsdp_shard_adam_step(lay, p, gs, m, v, t, LR, B1, B2, EPS)
    # fused
    need_g = with_outputs or W > 64
    gs2 = carve(S, torch.float32, 1, fill=POISON32) if need_g else None
    lp = carve(S, torch.bfloat16, 1, fill=POISON16) if with_outputs else None
    F.fsdp_reduce_scatter_adam_fused(lay, grads, r, pre, post, gs2, p2, m2, v2, t, LR, B1, B2, EPS, lp)
    torch.cuda.synchronize()
    for a, b in ((p, p2), (m, m2), (v, v2)):
        assert same_bits(np_bits(a), np_bits(b)), first_diff(np_bits(a), np_bits(b))
    if need_g:
        assert same_bits(np_bits(gs), np_bits(gs2))
    if with_outputs:
        assert same_bits(np_bits(lp), oracle.cast_bf16(np_f32(p2)))
    # and against the oracle
    ref_g = oracle.reduce_scatter([np_grad(g) for g in grads], r, pre, post)
    assert same_bits(np_bits(gs), ref_g.view(np.uint32))
    assert_adam_parity(np_f32(p2), np_f32(m2), np_f32(v2), hp, ref_g, hm, hv, t, (LR, B1, B2, EPS), "fused")


def test_whole_path_two_iterations_pad_stays_zero(F):
    """flatten -> [unshard -> reduce-scatter -> Adam] x 2 for every rank of a
    W = 12 unit with a pad; checks the unsharded bf16 buffer after the updates
    and that the pad never leaves zero (state is caller-owned: resume = same buffers)."""
    unit = workloads.Unit("u", ((1001, 7), (13,), (2048,)))
    W = 12
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    assert lay.pad > 0
    params = workloads.gen_params(unit, 0, device="cuda")
    shards = [torch.empty(S, dtype=torch.float32, device="cuda") for _ in range(W)]
    F.fsdp_flatten_shard(lay, params, shards)
    ms = [torch.zeros(S, device="cuda") for _ in range(W)]
    vs = [torch.zeros(S, device="cuda") for _ in range(W)]
    h_shards, _ = oracle.flatten_shard([np_f32(p) for p in params], W)
    h_m = [np.zeros(S, np.float32) for _ in range(W)]
    h_v = [np.zeros(S, np.float32) for _ in range(W)]
    pre, post = F.fsdp_default_divide_factors(W)
    flat = torch.empty(P, dtype=torch.bfloat16, device="cuda")
    gs = torch.empty(S, dtype=torch.float32, device="cuda")
    for t in (1, 2):
        F.fsdp_unshard(lay, shards, flat)
        torch.cuda.synchronize()
        assert same_bits(np_bits(flat), oracle.unshard_bf16(h_shards))
        grads = [workloads.gen_rank_grad(P, N, w, t, "f32", device="cuda") for w in range(W)]
        h_grads = [np_f32(g) for g in grads]
        for r in range(W):
            F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, gs)
            F.fsdp_shard_adam_step(lay, shards[r], gs, ms[r], vs[r], t, LR, B1, B2, EPS)
            torch.cuda.synchronize()
            ref_g = oracle.reduce_scatter(h_grads, r, pre, post)
            assert same_bits(np_bits(gs), ref_g.view(np.uint32))
            old = h_shards[r]
            h_shards[r], h_m[r], h_v[r] = oracle.adam_f32(old, ref_g, h_m[r], h_v[r], t, LR, B1, B2, EPS)
            assert_adam_bits(np_f32(shards[r]), np_f32(ms[r]), np_f32(vs[r]), h_shards[r], h_m[r], h_v[r])
            # keep both sides on identical state so that later steps stay comparable
            shards[r].copy_(torch.from_numpy(h_shards[r]))
            ms[r].copy_(torch.from_numpy(h_m[r]))
            vs[r].copy_(torch.from_numpy(h_v[r]))
        assert not np_bits(shards[W - 1])[S - lay.pad:].any()
    views = F.fsdp_views(lay, flat)
    assert [tuple(v.shape) for v in views] == [tuple(s) for s in unit.shapes]


def test_hip_graph_replay_matches_eager(F):
    """The entry points allocate and synchronise nothing, so a caller may
    capture them; every replay must reproduce the eager result."""
    unit = workloads.Unit("u", ((513, 33), (77,), (4096,)))
    W = 8
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    params = workloads.gen_params(unit, 3, device="cuda")
    shards = [torch.empty(S, dtype=torch.float32, device="cuda") for _ in range(W)]
    F.fsdp_flatten_shard(lay, params, shards)
    grads = [workloads.gen_rank_grad(P, N, w, 0, "f32", device="cuda") for w in range(W)]
    flat = torch.empty(P, dtype=torch.bfloat16, device="cuda")
    gs = torch.empty(S, dtype=torch.float32, device="cuda")
    p0 = shards[0].clone()
    m = torch.zeros(S, device="cuda")
    v = torch.zeros(S, device="cuda")

    # a second unit, updated and unsharded through the one-launch forms inside the same graph
    unit2 = workloads.Unit("u2", ((300, 41), (19,)))
    lay2 = F.fsdp_layout_init(unit2.shapes, W)
    params2 = workloads.gen_params(unit2, 4, device="cuda")
    shards2 = [torch.empty(lay2.shard, dtype=torch.float32, device="cuda") for _ in range(W)]
    F.fsdp_flatten_shard(lay2, params2, shards2)
    grads2 = [workloads.gen_rank_grad(lay2.padded, lay2.numel, w, 1, "f32", device="cuda") for w in range(W)]
    flat2 = torch.empty(lay2.padded, dtype=torch.bfloat16, device="cuda")
    flat2b = torch.empty(lay2.padded, dtype=torch.bfloat16, device="cuda")
    p2_0 = shards2[1].clone()
    m2 = torch.zeros(lay2.shard, device="cuda")
    v2 = torch.zeros(lay2.shard, device="cuda")
    batch = F.Batch()
    batch.add_reduce_scatter_adam(lay2, grads2, 1, pre, post, None, shards2[1], m2, v2, LR, B1, B2, EPS, None)
    batch.add_unshard(lay, shards, flat)

    def step():
        F.fsdp_unshard(lay, shards, flat)
        F.fsdp_unshard(lay2, shards2, flat2)
        F.fsdp_reduce_scatter_local(lay, grads, 0, pre, post, gs)
        F.fsdp_shard_adam_step(lay, shards[0], gs, m, v, 1, LR, B1, B2, EPS)
        batch.launch(1)                       # update of unit 2 + unshard of unit 1 (after its update) in one grid
        F.fsdp_reduce_scatter_adam_prefetch_unshard(lay2, grads2, 1, pre, post, None, shards2[1], m2, v2, 2, LR, B1, B2,
                                                    EPS, None, lay2, shards2[:1] + shards2[:1] * (W - 1), flat2b)

    step()
    torch.cuda.synchronize()
    outputs = (flat, gs, shards[0], m, v, flat2, flat2b, shards2[1], m2, v2)
    eager = [x.clone() for x in outputs]

    def reset():
        shards[0].copy_(p0)
        shards2[1].copy_(p2_0)
        for x in (m, v, flat, gs, m2, v2, flat2, flat2b):
            x.fill_(0.0)

    reset()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    for _ in range(3):
        reset()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, outputs):
            assert same_bits(np_bits(a), np_bits(b))


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("W,W_next,out_dt", [(8, 8, torch.bfloat16), (3, 12, torch.bfloat16), (12, 1, torch.bfloat16),
                                             (70, 8, torch.bfloat16), (8, 100, torch.bfloat16),
                                             (8, 8, torch.float32)])
def test_prefetch_launch_equals_separate_calls(F, gdt, W, W_next, out_dt):
    """Reduce-scatter + Adam of one unit and the unshard of another in one
    launch (backward prefetching) must give exactly what the separate entry
    points give, and match the oracle; W > 64 or an fp32 unshard fall back to
    two launches with the same results."""
    unit_a = big_unit() if W <= 12 else workloads.ragged_unit()
    unit_b = workloads.Unit("next", ((1023, 65), (7,), (30001,), (3, 3)))
    la = F.fsdp_layout_init(unit_a.shapes, W)
    lb = F.fsdp_layout_init(unit_b.shapes, W_next)
    pre, post = F.fsdp_default_divide_factors(W)
    grads = make_grads(W, la.padded, la.numel, gdt, 500 + W)
    r = W // 2
    t = 4
    p, _, m, v = _adam_state(la.shard, t, 23, (0, 0, 1, 2))
    p2, m2, v2 = p.clone(), m.clone(), v.clone()
    params_b = make_params(unit_b, 77, misalign=True)
    shards_b, _ = alloc_shards(W_next, lb.shard, "contig_odd")
    F.fsdp_flatten_shard(lb, params_b, shards_b)
    poison = POISON16 if out_dt == torch.bfloat16 else POISON32
    flat1 = carve(lb.padded, out_dt, 1, fill=poison)
    flat2 = carve(lb.padded, out_dt, 1, fill=poison)
    gs1 = carve(la.shard, torch.float32, 0, fill=POISON32)
    gs2 = carve(la.shard, torch.float32, 0, fill=POISON32)
    # separate calls
    F.fsdp_reduce_scatter_adam_fused(la, grads, r, pre, post, gs1, p, m, v, t, LR, B1, B2, EPS, None)
    F.fsdp_unshard(lb, shards_b, flat1)
    # one launch
    F.fsdp_reduce_scatter_adam_prefetch_unshard(la, grads, r, pre, post, gs2, p2, m2, v2, t, LR, B1, B2, EPS, None,
                                                lb, shards_b, flat2)
    torch.cuda.synchronize()
    for a, b, name in ((p, p2, "p"), (m, m2, "m"), (v, v2, "v"), (gs1, gs2, "g"), (flat1, flat2, "flat")):
        assert same_bits(np_bits(a), np_bits(b)), f"{name}: {first_diff(np_bits(a), np_bits(b))}"
    ref_g = oracle.reduce_scatter([np_grad(g) for g in grads], r, pre, post)
    assert same_bits(np_bits(gs2), ref_g.view(np.uint32))
    h_sh = [np_f32(x) for x in shards_b]
    ref_flat = oracle.unshard_bf16(h_sh) if out_dt == torch.bfloat16 else oracle.unshard_f32(h_sh).view(np.uint32)
    assert same_bits(np_bits(flat2), ref_flat)


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
def test_batch_of_independent_operations_equals_single_calls(F, gdt):
    """Four updates (W = 3, 8, 12 and 70, which is launched on its own; one with
    extra outputs) and four unshards (one W = 100 and one fp32 output, which
    cannot share a grid) in one batch: bit-identical to the single entry points, and the batch can be
    launched again with another step count."""
    specs = [(big_unit(), 3), (workloads.ragged_unit(), 8), (big_unit(), 12), (workloads.ragged_unit(), 70)]
    reds = []
    for i, (unit, W) in enumerate(specs):
        lay = F.fsdp_layout_init(unit.shapes, W)
        grads = make_grads(W, lay.padded, lay.numel, gdt, 800 + i)
        p, _, m, v = _adam_state(lay.shard, 3, 31 + i, (i % 2, 0, 1, 0))
        reds.append({"lay": lay, "grads": grads, "W": W, "r": W - 1, "p": p, "m": m, "v": v,
                     "g": carve(lay.shard, torch.float32, 0, fill=POISON32) if i in (1, 3) else None,   # W > 64 needs it
                     "lp": carve(lay.shard, torch.bfloat16, 1, fill=POISON16) if i == 1 else None})
    uns = []
    for i, (W, dt) in enumerate([(8, torch.bfloat16), (100, torch.bfloat16), (5, torch.float32), (12, torch.bfloat16)]):
        unit = workloads.Unit(f"u{i}", ((513 + i, 65), (7,), (20001,), (3, 3)))
        lay = F.fsdp_layout_init(unit.shapes, W)
        params = make_params(unit, 90 + i, misalign=True)
        shards, _ = alloc_shards(W, lay.shard, "contig_odd")
        F.fsdp_flatten_shard(lay, params, shards)
        uns.append({"lay": lay, "shards": shards, "dt": dt})
    batch = F.Batch()
    flats_b, flats_s = [], []
    for u in uns:
        poison = POISON16 if u["dt"] == torch.bfloat16 else POISON32
        flats_b.append(carve(u["lay"].padded, u["dt"], 1, fill=poison))
        flats_s.append(carve(u["lay"].padded, u["dt"], 1, fill=poison))
    order = [("u", 0), ("r", 0), ("u", 1), ("r", 1), ("r", 3), ("r", 2), ("u", 2), ("u", 3)]
    for kind, i in order:
        if kind == "u":
            batch.add_unshard(uns[i]["lay"], uns[i]["shards"], flats_b[i])
        else:
            d = reds[i]
            pre, post = F.fsdp_default_divide_factors(d["W"])
            batch.add_reduce_scatter_adam(d["lay"], d["grads"], d["r"], pre, post, d["g"], d["p"], d["m"], d["v"],
                                          LR, B1, B2, EPS, d["lp"])
    for step in (3, 4):
        snap = [(d["p"].clone(), d["m"].clone(), d["v"].clone()) for d in reds]
        batch.launch(step)
        torch.cuda.synchronize()
        for d, (p0, m0, v0) in zip(reds, snap):
            pre, post = F.fsdp_default_divide_factors(d["W"])
            gs = torch.empty(d["lay"].shard, dtype=torch.float32, device="cuda")
            F.fsdp_reduce_scatter_adam_fused(d["lay"], d["grads"], d["r"], pre, post, gs, p0, m0, v0, step, LR, B1, B2,
                                             EPS, None)
            torch.cuda.synchronize()
            for a, b, name in ((d["p"], p0, "p"), (d["m"], m0, "m"), (d["v"], v0, "v")):
                assert same_bits(np_bits(a), np_bits(b)), f"step {step} {name}: {first_diff(np_bits(a), np_bits(b))}"
            if d["g"] is not None:
                assert same_bits(np_bits(d["g"]), np_bits(gs))
            if d["lp"] is not None:
                assert same_bits(np_bits(d["lp"]), oracle.cast_bf16(np_f32(d["p"])))
            ref_g = oracle.reduce_scatter([np_grad(g) for g in d["grads"]], d["r"], pre, post)
            assert same_bits(np_bits(gs), ref_g.view(np.uint32))
        for u, fb, fs in zip(uns, flats_b, flats_s):
            F.fsdp_unshard(u["lay"], u["shards"], fs)
            torch.cuda.synchronize()
            assert same_bits(np_bits(fb), np_bits(fs))
            h = [np_f32(x) for x in u["shards"]]
            ref = oracle.unshard_bf16(h) if u["dt"] == torch.bfloat16 else oracle.unshard_f32(h).view(np.uint32)
            assert same_bits(np_bits(fb), ref)
    batch.close()


@pytest.mark.parametrize("lp_dt", [torch.bfloat16, torch.float16])
def test_batch_with_low_precision_hand_off(F, lp_dt):
    """Sec. 4.4 hand-off in batches: updates that write the rank's 16-bit shard,
    then gathers of 16-bit shards (one with W = 100, which is launched on its
    own) next to a cast + gather member, against the oracle."""
    specs = [(big_unit(), 3), (workloads.ragged_unit(), 8), (workloads.ragged_unit(), 100)]
    units = []
    for i, (unit, W) in enumerate(specs):
        lay = F.fsdp_layout_init(unit.shapes, W)
        params = make_params(unit, 70 + i, misalign=True)
        shards, _ = alloc_shards(W, lay.shard, "contig_odd")
        F.fsdp_flatten_shard(lay, params, shards)
        lps = [carve(lay.shard, lp_dt, (w + i) % 8, fill=POISON16) for w in range(W)]
        for w in range(W):
            F.fsdp_cast_shard(lay, shards[w], lps[w])
        units.append({"lay": lay, "W": W, "shards": shards, "lps": lps,
                      "flat": carve(lay.padded, lp_dt, 3, fill=POISON16)})
    torch.cuda.synchronize()
    batch = F.Batch()
    batch.add_unshard_lp(units[0]["lay"], units[0]["lps"], units[0]["flat"])
    extra = carve(units[1]["lay"].padded, torch.bfloat16, 1, fill=POISON16)
    batch.add_unshard(units[1]["lay"], units[1]["shards"], extra)              # cast + gather member in the same grid
    batch.add_unshard_lp(units[1]["lay"], units[1]["lps"], units[1]["flat"])
    batch.add_unshard_lp(units[2]["lay"], units[2]["lps"], units[2]["flat"])
    batch.launch(1)
    torch.cuda.synchronize()
    for u in units:
        h = [np_f32(x) for x in u["shards"]]
        ref = oracle.unshard_bf16(h) if lp_dt == torch.bfloat16 else oracle.unshard_f16(h)
        assert same_bits(np_bits(u["flat"]), ref), first_diff(np_bits(u["flat"]), ref)
        assert same_bits(np_bits(u["flat"]), oracle.gather_lp([np_bits(x) for x in u["lps"]]))
    assert same_bits(np_bits(extra), oracle.unshard_bf16([np_f32(x) for x in units[1]["shards"]]))
    batch.close()

    if lp_dt != torch.bfloat16:
        return      # the Adam epilogue writes bf16 copies only
    # one iteration of the hand-off: the update of rank r writes its bf16 shard, the next gather reads it
    u = units[1]
    lay, W, r = u["lay"], u["W"], 5
    grads = make_grads(W, lay.padded, lay.numel, torch.bfloat16, 4242)
    pre, post = F.fsdp_default_divide_factors(W)
    m, v = torch.zeros(lay.shard, device="cuda"), torch.zeros(lay.shard, device="cuda")
    p0 = np_f32(u["shards"][r]).copy()
    b1, b2 = F.Batch(), F.Batch()
    b1.add_reduce_scatter_adam(lay, grads, r, pre, post, None, u["shards"][r], m, v, LR, B1, B2, EPS, u["lps"][r])
    b2.add_unshard_lp(lay, u["lps"], u["flat"])
    b1.launch(1)
    b2.launch(1)
    torch.cuda.synchronize()
    ref_g = oracle.reduce_scatter([np_grad(g) for g in grads], r, pre, post)
    z = np.zeros(lay.shard, np.float32)
    rp, rm, rv = oracle.adam_f32(p0, ref_g, z, z, 1, LR, B1, B2, EPS)
    assert_adam_bits(np_f32(u["shards"][r]), np_f32(m), np_f32(v), rp, rm, rv)
    ref = oracle.unshard_bf16([np_f32(x) for x in u["shards"]])      # the other ranks' shards are unchanged
    assert same_bits(np_bits(u["flat"]), ref), first_diff(np_bits(u["flat"]), ref)
    b1.close()
    b2.close()


def test_resume_from_copied_state_is_bit_identical(F):
    """The state is caller-owned (p, m, v, step count): two steps in place equal
    one step, a copy of the state to other buffers, and one more step there."""
    unit, W, r = big_unit(), 8, 3
    lay = F.fsdp_layout_init(unit.shapes, W)
    S = lay.shard
    pre, post = F.fsdp_default_divide_factors(W)
    g1 = make_grads(W, lay.padded, lay.numel, torch.float32, 611)
    g2 = make_grads(W, lay.padded, lay.numel, torch.float32, 612)
    p, _, m, v = _adam_state(S, 1, 77)
    h0 = np_f32(p).copy()
    F.fsdp_reduce_scatter_adam_fused(lay, g1, r, pre, post, None, p, m, v, 1, LR, B1, B2, EPS, None)
    torch.cuda.synchronize()
    saved = [np_f32(x).copy() for x in (p, m, v)]                      # "checkpoint" on the host
    F.fsdp_reduce_scatter_adam_fused(lay, g2, r, pre, post, None, p, m, v, 2, LR, B1, B2, EPS, None)
    p2, m2, v2 = (carve(S, torch.float32, off) for off in (1, 2, 3))   # restore into other, misaligned buffers
    for dst, src in zip((p2, m2, v2), saved):
        dst.copy_(torch.from_numpy(src))
    F.fsdp_reduce_scatter_adam_fused(lay, g2, r, pre, post, None, p2, m2, v2, 2, LR, B1, B2, EPS, None)
    torch.cuda.synchronize()
    for a, b, n in ((p, p2, "p"), (m, m2, "m"), (v, v2, "v")):
        assert same_bits(np_bits(a), np_bits(b)), n
    # and the chain equals the oracle's
    z = np.zeros(S, np.float32)
    r1 = oracle.reduce_scatter([np_grad(g) for g in g1], r, pre, post)
    r2 = oracle.reduce_scatter([np_grad(g) for g in g2], r, pre, post)
    op, om, ov = oracle.adam_f32(h0, r1, z, z, 1, LR, B1, B2, EPS)
    op2, om2, ov2 = oracle.adam_f32(op, r2, om, ov, 2, LR, B1, B2, EPS)
    assert_adam_bits(np_f32(p), np_f32(m), np_f32(v), op2, om2, ov2)


def test_fig3_worked_example_on_gpu(F):
    """Sec. 3.2.1 / Fig. 3: a 4x3 Linear (12 weights + 3 biases) over 16 ranks:
    one element per rank, the last rank holds the pad.  The whole path at S = 1."""
    W = 16
    shapes = [(3, 4), (3,)]
    lay = F.fsdp_layout_init(shapes, W)
    assert (lay.numel, lay.shard, lay.padded, lay.pad) == (15, 1, 16, 1)
    w = torch.arange(1, 13, dtype=torch.float32, device="cuda").view(3, 4)
    b = torch.arange(13, 16, dtype=torch.float32, device="cuda")
    base = carve(W, torch.float32, 1, fill=POISON32)
    shards = [base[i:i + 1] for i in range(W)]
    F.fsdp_flatten_shard(lay, [w, b], shards)
    torch.cuda.synchronize()
    assert base.tolist() == [float(i) for i in range(1, 16)] + [0.0]
    assert np_bits(shards[15])[0] == 0                                  # the pad is +0.0f on the last rank
    flat = carve(16, torch.bfloat16, 3, fill=POISON16)
    F.fsdp_unshard(lay, shards, flat)
    grads = [torch.full((16,), float(r + 1), device="cuda") for r in range(W)]
    for g in grads:
        g[15] = 0.0                                                     # nothing is ever written to the pad's gradient
    h_shards = [np_f32(s) for s in shards]
    for r in range(W):
        gs = torch.empty(1, device="cuda")
        F.fsdp_reduce_scatter_local(lay, grads, r, 4.0, 4.0, gs)
        m = torch.zeros(1, device="cuda")
        v = torch.zeros(1, device="cuda")
        F.fsdp_shard_adam_step(lay, shards[r], gs, m, v, 1, LR, B1, B2, EPS)
        torch.cuda.synchronize()
        ref_g = oracle.reduce_scatter([np_f32(g) for g in grads], r, 4.0, 4.0)
        assert same_bits(np_bits(gs), ref_g.view(np.uint32))
        assert float(gs[0]) == (8.5 if r < 15 else 0.0)                 # mean of 1..16
        z = np.zeros(1, np.float32)
        rp, rm, rv = oracle.adam_f32(h_shards[r], ref_g, z, z, 1, LR, B1, B2, EPS)
        assert_adam_bits(np_f32(shards[r]), np_f32(m), np_f32(v), rp, rm, rv)
    torch.cuda.synchronize()
    assert same_bits(np_bits(flat), oracle.unshard_bf16(h_shards))
    assert float(shards[15][0]) == 0.0                                  # the pad stays zero through Adam
    views = F.fsdp_views(lay, flat)
    assert tuple(views[0].shape) == (3, 4) and tuple(views[1].shape) == (3,)
    assert views[0].float().flatten().tolist() == [float(i) for i in range(1, 13)]


def test_readme_usage_block_runs_and_matches_oracle(F):
    """The usage example printed in README.md, executed as it stands."""
    import os
    import re
    text = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "README.md")).read()
    blocks = re.findall(r"```python\n(.*?)```", text, flags=re.S)
    assert len(blocks) == 1
    torch.manual_seed(11)
    ns = {}
    exec(compile(blocks[0], "README.md", "exec"), ns)
    torch.cuda.synchronize()
    lay, W, rank = ns["lay"], ns["W"], ns["rank"]
    S = lay.shard
    # the views show the bf16 cast of the parameters as they were before the update
    for view, param in zip(ns["views"], ns["params"]):
        assert view.shape == param.shape
        assert same_bits(np_bits(view.contiguous()).ravel(), oracle.cast_bf16(np_f32(param).ravel()))
    # the rank's shard after step 1 from zero state
    flat32 = np.concatenate([np_f32(p).ravel() for p in ns["params"]] + [np.zeros(lay.pad, np.float32)])
    g = oracle.reduce_scatter([np_f32(x) for x in ns["grads"]], rank, ns["pre"], ns["post"])
    z = np.zeros(S, np.float32)
    rp, rm, rv = oracle.adam_f32(flat32[rank * S:(rank + 1) * S], g, z, z, 1, 1e-4, 0.9, 0.999, 1e-8)
    assert_adam_bits(np_f32(ns["shards"][rank]), np_f32(ns["m"]), np_f32(ns["v"]), rp, rm, rv)


def test_host_threads_share_a_layout_and_a_batch(F):
    """Calls that share a layout (and launches of an unmodified batch) are
    independent across host threads and streams: four threads, each on its own
    stream with its own outputs and optimizer state, give the bits of the same
    calls issued one after the other from one thread."""
    import threading
    W, r, iters, nthreads = 8, 5, 40, 4
    unit = big_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    params = make_params(unit, 77, misalign=False)
    shards, _ = alloc_shards(W, S, "contig_odd")
    F.fsdp_flatten_shard(lay, params, shards)
    shard_tab = F.PtrArray(shards)
    grad_tab = F.PtrArray(make_grads(W, P, N, torch.bfloat16, 4100))
    batch = F.Batch()
    batch_flat = carve(P, torch.bfloat16, 0, fill=POISON16)
    batch.add_unshard(lay, shard_tab, batch_flat)
    torch.cuda.synchronize()

    def fresh_state():
        g = torch.Generator(device="cuda")
        g.manual_seed(4200)
        return (torch.empty(S, device="cuda").normal_(0, 0.02, generator=g), torch.zeros(S, device="cuda"),
                torch.zeros(S, device="cuda"), carve(P, torch.bfloat16, 1, fill=POISON16))

    def work(state, stream):
        p, m, v, flat = state
        for t in range(1, iters + 1):
            F.fsdp_unshard(lay, shard_tab, flat, stream=stream)
            batch.launch(t, stream=stream)
            F.fsdp_reduce_scatter_adam_fused(lay, grad_tab, r, pre, post, None, p, m, v, t, LR, B1, B2, EPS, None,
                                             stream=stream)

    ref = fresh_state()
    work(ref, None)
    torch.cuda.synchronize()
    states = [fresh_state() for _ in range(nthreads)]
    streams = [torch.cuda.Stream() for _ in range(nthreads)]
    torch.cuda.synchronize()
    errors = []

    def body(i):
        try:
            work(states[i], streams[i])
        except Exception as e:       # surfaced below: an exception in a thread must fail the test
            errors.append(e)

    threads = [threading.Thread(target=body, args=(i,)) for i in range(nthreads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i, st in enumerate(states):
        for got, want, name in zip(st, ref, ("p", "m", "v", "flat")):
            assert same_bits(np_bits(got), np_bits(want)), f"thread {i} {name}: {first_diff(np_bits(got), np_bits(want))}"
    assert same_bits(np_bits(batch_flat), np_bits(ref[3]))
    assert same_bits(np_bits(ref[3]), oracle.unshard_bf16([np_f32(s) for s in shards]))
    batch.close()
