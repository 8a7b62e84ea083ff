"""GPU parity for the rows after the hot path: hybrid-sharding reduction
(Sec. 3.2.2) and gradient accumulation with and without communication
(Sec. 3.3.4).  Bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import POISON32, carve, first_diff, load_product, np_bits, np_f32, np_grad, same_bits
from test_gpu_parity_small import big_unit, make_grads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    assert torch.cuda.is_available()
    return load_product()


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("G,Fs,pre,post", [(1, 8, 4.0, 2.0), (2, 8, 4.0, 4.0), (4, 2, 2.0, 4.0), (3, 4, 4.0, 3.0),
                                           (8, 8, 8.0, 8.0), (2, 3, 1.0, 6.0), (5, 1, 1.0, 5.0), (16, 4, 8.0, 8.0),
                                           # more than 64 ranks: several launches of whole groups
                                           (16, 8, 16.0, 8.0), (3, 40, 8.0, 15.0), (2, 64, 8.0, 16.0), (70, 1, 7.0, 10.0),
                                           (9, 12, 4.0, 27.0)])
def test_hybrid_reduce_scatter_bit_exact(F, gdt, G, Fs, pre, post):
    unit = big_unit() if G * Fs <= 16 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, Fs)            # sharding factor F, world = G * F ranks
    S, P, N = lay.shard, lay.padded, lay.numel
    grads = make_grads(G * Fs, P, N, gdt, 700 + G * Fs, outliers=True, elem_offset=1)
    host = [np_grad(g) for g in grads]
    for r in sorted({0, Fs // 2, Fs - 1}):
        out = carve(S, torch.float32, r % 3, fill=POISON32)
        F.fsdp_reduce_scatter_hybrid(lay, grads, G, r, pre, post, out)
        torch.cuda.synchronize()
        ref = oracle.reduce_slices_hybrid([h[r * S:(r + 1) * S] for h in host], G, Fs, pre, post)
        got = np_bits(out)
        assert same_bits(got, ref.view(np.uint32)), f"rank {r}: {first_diff(got, ref.view(np.uint32))}"
        if G == 1:
            flat = torch.empty(S, dtype=torch.float32, device="cuda")
            F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, flat)
            torch.cuda.synchronize()
            assert same_bits(np_bits(flat), got)


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("G,Fs,pre,post,with_outputs", [(2, 8, 4.0, 4.0, True), (4, 4, 4.0, 4.0, False), (3, 5, 1.0, 15.0, True),
                                                        (16, 8, 16.0, 8.0, True), (3, 40, 8.0, 15.0, True)])
def test_hybrid_reduce_scatter_fused_with_adam(F, gdt, G, Fs, pre, post, with_outputs):
    """Sec. 3.2.2 reduction with the Adam step applied in the same launch: the
    bits of fsdp_reduce_scatter_hybrid followed by fsdp_shard_adam_step, and of
    the oracle's two steps, at t = 3 from non-zero state."""
    from gpu_helpers import POISON16, assert_adam_bits
    unit = big_unit() if G * Fs <= 16 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, Fs)
    S, P, N = lay.shard, lay.padded, lay.numel
    grads = make_grads(G * Fs, P, N, gdt, 2300 + G * Fs, elem_offset=1)
    host = [np_grad(g) for g in grads]
    hp = (1e-4, 0.9, 0.999, 1e-8)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(61)
    for r in sorted({0, Fs - 1}):
        p = carve(S, torch.float32, 0)
        p.normal_(0, 0.02, generator=gen)
        m = carve(S, torch.float32, 1)
        m.normal_(0, 1e-3, generator=gen)
        v = carve(S, torch.float32, 3)
        v.uniform_(0, 1e-6, generator=gen)
        p2, m2, v2 = p.clone(), m.clone(), v.clone()
        h_p, h_m, h_v = np_f32(p).copy(), np_f32(m).copy(), np_f32(v).copy()
        g_out = carve(S, torch.float32, 2, fill=POISON32) if with_outputs else None
        lp_out = carve(S, torch.bfloat16, 1, fill=POISON16) if with_outputs else None
        F.fsdp_reduce_scatter_hybrid_adam_fused(lay, grads, G, r, pre, post, g_out, p, m, v, 3, *hp, lp_out)
        gs = torch.empty(S, device="cuda")
        F.fsdp_reduce_scatter_hybrid(lay, grads, G, r, pre, post, gs)
        F.fsdp_shard_adam_step(lay, p2, gs, m2, v2, 3, *hp)
        torch.cuda.synchronize()
        for a, b, name in ((p, p2, "p"), (m, m2, "m"), (v, v2, "v")):
            assert same_bits(np_bits(a), np_bits(b)), f"rank {r} {name}: {first_diff(np_bits(a), np_bits(b))}"
        ref_g = oracle.reduce_slices_hybrid([h[r * S:(r + 1) * S] for h in host], G, Fs, pre, post)
        rp, rm, rv = oracle.adam_f32(h_p, ref_g, h_m, h_v, 3, *hp)
        assert_adam_bits(np_f32(p), np_f32(m), np_f32(v), rp, rm, rv)
        if with_outputs:
            assert same_bits(np_bits(g_out), ref_g.view(np.uint32))
            assert same_bits(np_bits(lp_out), oracle.cast_bf16(np_f32(p)))


def test_hybrid_fused_needs_the_gradient_shard_beyond_one_launch(F):
    lay = F.fsdp_layout_init([(100,)], 8)
    grads = [torch.zeros(lay.padded, device="cuda") for _ in range(72)]
    p, m, v = (torch.zeros(lay.shard, device="cuda") for _ in range(3))
    with pytest.raises(F.FsdpError) as e:
        F.fsdp_reduce_scatter_hybrid_adam_fused(lay, grads, 9, 0, 1.0, 1.0, None, p, m, v, 1, 1e-4, 0.9, 0.999, 1e-8, None)
    assert e.value.status == -2


def test_hybrid_order_witness_on_gpu(F):
    """(1e8, 1 | -1e8, 1): group sums first gives 0, flat rank order gives 1."""
    lay = F.fsdp_layout_init([(3000,)], 2)
    grads = [torch.full((lay.padded,), v, dtype=torch.float32, device="cuda") for v in (1e8, 1.0, -1e8, 1.0)]
    out = torch.empty(lay.shard, dtype=torch.float32, device="cuda")
    F.fsdp_reduce_scatter_hybrid(lay, grads, 2, 1, 1.0, 1.0, out)
    torch.cuda.synchronize()
    assert bool((out == 0.0).all())


def test_hybrid_rejects_a_group_larger_than_one_launch(F):
    lay = F.fsdp_layout_init([(100,)], 65)
    grads = [torch.zeros(lay.padded, device="cuda") for _ in range(130)]
    out = torch.empty(lay.shard, device="cuda")
    with pytest.raises(F.FsdpError) as e:
        F.fsdp_reduce_scatter_hybrid(lay, grads, 2, 0, 1.0, 1.0, out)
    assert e.value.status == -1


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("W", [1, 3, 8, 12, 64])
def test_gradient_accumulation_with_communication(F, gdt, W):
    """Three micro-batches, each reduce-scattered into the running sharded gradient."""
    unit = big_unit() if W <= 12 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    r = W - 1
    acc = carve(S, torch.float32, 1)
    acc.zero_()
    h_acc = np.zeros(S, np.float32)
    for mb in range(3):
        grads = make_grads(W, P, N, gdt, 900 + 10 * mb + W)
        F.fsdp_reduce_scatter_accumulate(lay, grads, r, pre, post, acc)
        torch.cuda.synchronize()
        h_acc = oracle.accumulate(h_acc, oracle.reduce_scatter([np_grad(g) for g in grads], r, pre, post))
        assert same_bits(np_bits(acc), h_acc.view(np.uint32)), f"micro-batch {mb}: {first_diff(np_bits(acc), h_acc.view(np.uint32))}"


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("off", [0, 1, 3])
def test_gradient_accumulation_without_communication(F, gdt, off):
    """Unsharded local accumulation over P elements, then one reduce-scatter."""
    unit = big_unit()
    W = 4
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    accs = [carve(P, torch.float32, off) for _ in range(W)]
    for a in accs:
        a.zero_()
    h_accs = [np.zeros(P, np.float32) for _ in range(W)]
    for mb in range(3):
        grads = make_grads(W, P, N, gdt, 1200 + 10 * mb, elem_offset=(off + 1) % 2)
        for w in range(W):
            F.fsdp_grad_accumulate(lay, accs[w], grads[w])
            h_accs[w] = oracle.accumulate(h_accs[w], np_grad(grads[w]))
        torch.cuda.synchronize()
        for w in range(W):
            assert same_bits(np_bits(accs[w]), h_accs[w].view(np.uint32)), (mb, w)
    out = torch.empty(S, dtype=torch.float32, device="cuda")
    F.fsdp_reduce_scatter_local(lay, accs, 2, 2.0, 2.0, out)
    torch.cuda.synchronize()
    assert same_bits(np_bits(out), oracle.reduce_scatter(h_accs, 2, 2.0, 2.0).view(np.uint32))


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("W", [1, 3, 8, 12, 64])
def test_last_micro_batch_accumulates_and_steps_in_one_launch(F, gdt, W):
    """Two micro-batches accumulated, the third accumulated and followed by the
    Adam step inside the same launch: the bits of the separate calls and of the
    oracle's chain, at t = 2 from non-zero state."""
    from gpu_helpers import POISON16, assert_adam_bits
    unit = big_unit() if W <= 12 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    hp = (1e-4, 0.9, 0.999, 1e-8)
    r = W // 2
    gen = torch.Generator(device="cuda")
    gen.manual_seed(71 + W)
    p = carve(S, torch.float32, 0)
    p.normal_(0, 0.02, generator=gen)
    m = carve(S, torch.float32, 1)
    m.normal_(0, 1e-3, generator=gen)
    v = carve(S, torch.float32, 2)
    v.uniform_(0, 1e-6, generator=gen)
    p2, m2, v2 = p.clone(), m.clone(), v.clone()
    h_p, h_m, h_v = np_f32(p).copy(), np_f32(m).copy(), np_f32(v).copy()
    acc = carve(S, torch.float32, 3)
    acc.zero_()
    acc2 = torch.zeros(S, device="cuda")
    lp = carve(S, torch.bfloat16, 1, fill=POISON16)
    h_acc = np.zeros(S, np.float32)
    for mb in range(3):
        grads = make_grads(W, P, N, gdt, 2600 + 10 * mb + W)
        if mb < 2:
            F.fsdp_reduce_scatter_accumulate(lay, grads, r, pre, post, acc)
        else:
            F.fsdp_reduce_scatter_accumulate_adam_fused(lay, grads, r, pre, post, acc, p, m, v, 2, *hp, lp)
        F.fsdp_reduce_scatter_accumulate(lay, grads, r, pre, post, acc2)
        torch.cuda.synchronize()
        h_acc = oracle.accumulate(h_acc, oracle.reduce_scatter([np_grad(g) for g in grads], r, pre, post))
    F.fsdp_shard_adam_step(lay, p2, acc2, m2, v2, 2, *hp)
    torch.cuda.synchronize()
    assert same_bits(np_bits(acc), h_acc.view(np.uint32)), first_diff(np_bits(acc), h_acc.view(np.uint32))
    assert same_bits(np_bits(acc), np_bits(acc2))
    for a, b, name in ((p, p2, "p"), (m, m2, "m"), (v, v2, "v")):
        assert same_bits(np_bits(a), np_bits(b)), f"{name}: {first_diff(np_bits(a), np_bits(b))}"
    rp, rm, rv = oracle.adam_f32(h_p, h_acc, h_m, h_v, 2, *hp)
    assert_adam_bits(np_f32(p), np_f32(m), np_f32(v), rp, rm, rv)
    assert same_bits(np_bits(lp), oracle.cast_bf16(np_f32(p)))


def test_accumulate_then_fused_adam_equals_oracle_chain(F):
    """Two accumulated micro-batches followed by the optimizer step at t = 2 from non-zero state."""
    unit = big_unit()
    W = 8
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    r = 3
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    p = torch.empty(S, device="cuda").normal_(0, 0.02, generator=g)
    m = torch.empty(S, device="cuda").normal_(0, 1e-3, generator=g)
    v = torch.empty(S, device="cuda").uniform_(0, 1e-6, generator=g)
    hp, hm, hv = np_f32(p).copy(), np_f32(m).copy(), np_f32(v).copy()
    acc = torch.zeros(S, device="cuda")
    h_acc = np.zeros(S, np.float32)
    for mb in range(2):
        grads = make_grads(W, P, N, torch.float32, 1500 + mb)
        F.fsdp_reduce_scatter_accumulate(lay, grads, r, pre, post, acc)
        h_acc = oracle.accumulate(h_acc, oracle.reduce_scatter([np_f32(x) for x in grads], r, pre, post))
    F.fsdp_shard_adam_step(lay, p, acc, m, v, 2, 1e-4, 0.9, 0.999, 1e-8)
    torch.cuda.synchronize()
    rp, rm, rv = oracle.adam_f32(hp, h_acc, hm, hv, 2, 1e-4, 0.9, 0.999, 1e-8)
    from gpu_helpers import assert_adam_bits
    assert_adam_bits(np_f32(p), np_f32(m), np_f32(v), rp, rm, rv)


@pytest.mark.parametrize("W", [1, 3, 8, 12, 100])
@pytest.mark.parametrize("mode", ["separate", "contig_odd"])
def test_low_precision_shard_handoff(F, W, mode):
    """Each rank casts its own shard once (or Adam writes the bf16 copy), the
    unshard gathers bf16: same flat buffer as the fused cast+gather."""
    from test_gpu_parity_small import alloc_shards, make_params
    from gpu_helpers import POISON16
    unit = big_unit() if W <= 12 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P = lay.shard, lay.padded
    params = make_params(unit, 40 + W, misalign=False)
    shards, _ = alloc_shards(W, S, mode)
    F.fsdp_flatten_shard(lay, params, shards)
    if mode == "separate":
        lps = [carve(S, torch.bfloat16, w % 3, fill=POISON16) for w in range(W)]
    else:
        base = carve(W * S, torch.bfloat16, 1, fill=POISON16)
        lps = [base[w * S:(w + 1) * S] for w in range(W)]
    for w in range(W):
        F.fsdp_cast_shard(lay, shards[w], lps[w])
    flat = carve(P, torch.bfloat16, 1, fill=POISON16)
    F.fsdp_unshard_lp(lay, lps, flat)
    ref_flat = torch.empty(P, dtype=torch.bfloat16, device="cuda")
    F.fsdp_unshard(lay, shards, ref_flat)
    torch.cuda.synchronize()
    h_shards = [np_f32(s) for s in shards]
    for w in range(W):
        assert same_bits(np_bits(lps[w]), oracle.cast_bf16(h_shards[w])), f"cast of shard {w}"
    ref = oracle.gather_lp([np_bits(x) for x in lps])
    assert same_bits(np_bits(flat), ref), first_diff(np_bits(flat), ref)
    assert same_bits(np_bits(flat), np_bits(ref_flat))
    assert same_bits(np_bits(flat), oracle.unshard_bf16(h_shards))
