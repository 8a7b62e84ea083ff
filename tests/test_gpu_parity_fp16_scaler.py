"""GPU parity for the FP16 path and the sharded gradient scaler (Sec. 4.4):
fp16 cast in the unshard, fp16 gradients in the reduce-scatter, the fused
non-finite check + unscale, the cross-rank flag combine, the guarded optimizer
step and the scale update.  Bit-exact against the oracle (Adam within 1e-6)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import (POISON16, POISON32, assert_adam_bits, assert_adam_parity, carve, first_diff, load_product, np_bits, np_f32, same_bits)
from test_gpu_parity_small import EDGE_BITS, alloc_shards, big_unit, make_params

pytestmark = pytest.mark.gpu

F16_EDGES = [0x477FE000, 0x477FF000, 0x477FEFFF, 0x47800000, 0x33800000, 0x33000000, 0x33000001, 0x38800000,
             0x387FE000, 0x387FC000, 0x3F801000, 0x3F803000, 0x3F801001, 0xC7FFFFFF, 0x337FFFFF, 0x38000000,
             0x387FFFFF, 0x33C00000, 0x34400000]


@pytest.fixture(scope="module")
def F():
    assert torch.cuda.is_available()
    return load_product()


@pytest.mark.parametrize("W", [1, 3, 8, 12, 100])
def test_unshard_fp16(F, W):
    unit = big_unit() if W <= 12 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    params = make_params(unit, 60 + W, misalign=True)
    if W <= 12:   # second parameter: values around the fp16 rounding / overflow / subnormal edges
        edge = np.array(F16_EDGES + EDGE_BITS, dtype=np.uint32).view(np.float32)
        params[1].view(-1)[:edge.size].copy_(torch.tensor(edge))
        params[1].view(-1)[edge.size:edge.size + 4096].mul_(3e6)       # some overflow to Inf
        params[1].view(-1)[edge.size + 4096:edge.size + 8192].mul_(1e-6)  # some land on the subnormal grid
    shards, _ = alloc_shards(W, lay.shard, "contig_odd")
    F.fsdp_flatten_shard(lay, params, shards)
    flat = carve(lay.padded, torch.float16, 1, fill=POISON16)
    F.fsdp_unshard(lay, shards, flat)
    lps = [carve(lay.shard, torch.float16, w % 2, fill=POISON16) for w in range(W)]
    for w in range(W):
        F.fsdp_cast_shard(lay, shards[w], lps[w])
    flat2 = carve(lay.padded, torch.float16, 0, fill=POISON16)
    F.fsdp_unshard_lp(lay, lps, flat2)
    torch.cuda.synchronize()
    ref = oracle.unshard_f16([np_f32(s) for s in shards])
    assert same_bits(np_bits(flat), ref), first_diff(np_bits(flat), ref)
    assert same_bits(np_bits(flat2), ref)
    views = F.fsdp_views(lay, flat)
    assert [tuple(v.shape) for v in views] == [tuple(s) for s in unit.shapes]


def make_f16_grads(W, P, N, seed, scale=1.0):
    grads = []
    for w in range(W):
        g32 = workloads.gen_rank_grad(P, N, w, 0, "f32", device="cuda", seed=seed, std=1e-3 * scale)
        t = carve(P, torch.float16, w % 2)
        t.copy_(g32)            # input preparation: torch's own cast, the bytes are what both sides read
        grads.append(t)
    return grads


@pytest.mark.parametrize("W,pre,post", [(1, 1.0, 1.0), (3, 1.0, 3.0), (8, 4.0, 2.0), (12, 4.0, 3.0), (64, 8.0, 8.0),
                                        (70, 2.0, 35.0)])
def test_reduce_scatter_fp16_grads(F, W, pre, post):
    unit = big_unit() if W <= 12 else workloads.ragged_unit()
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    grads = make_f16_grads(W, P, N, 70 + W)
    for w, g in enumerate(grads):     # fp16 subnormals, signed zero, the largest finite value
        g.view(torch.int16)[:6] = torch.tensor([0x0001, -0x7FFF - 1, 0x03FF, 0x7BFF if w == 0 else 0x0400, 0x0000,
                                                0x8001 - 0x10000], dtype=torch.int16)
    host = [np_bits(g) for g in grads]
    for r in sorted({0, W // 2, W - 1}):
        out = carve(S, torch.float32, r % 3, fill=POISON32)
        F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, out)
        torch.cuda.synchronize()
        ref = oracle.reduce_slices_f16([h[r * S:(r + 1) * S] for h in host], pre, post)
        assert same_bits(np_bits(out), ref.view(np.uint32)), f"rank {r}: {first_diff(np_bits(out), ref.view(np.uint32))}"


@pytest.mark.parametrize("bad", [None, "inf", "nan", "overflow_in_sum"])
def test_reduce_scatter_unscale_and_sharded_flag(F, bad):
    """Scaled fp16 gradients on W = 8 ranks; one non-finite value sits in rank
    5's shard only.  Every rank's shard is unscaled and checked; the combined
    flag makes every rank skip the step."""
    unit = big_unit()
    W = 8
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = F.fsdp_default_divide_factors(W)
    scale = 1024.0
    inv = float(np.float32(1.0 / scale))
    grads = make_f16_grads(W, P, N, 90, scale=scale)
    spot = 5 * S + 17
    if bad == "inf":
        grads[2][spot] = float("inf")
    elif bad == "nan":
        grads[6][spot] = float("nan")
    elif bad == "overflow_in_sum":
        for g in grads:
            g[spot] = 65504.0
        pre, post = 1.0, 8.0           # the fp32 sum of eight 65504 is finite: no flag expected from it
    host = [np_bits(g) for g in grads]
    flags = [torch.zeros(1, device="cuda") for _ in range(W)]
    outs = [carve(S, torch.float32, 0, fill=POISON32) for _ in range(W)]
    for r in range(W):
        F.fsdp_reduce_scatter_unscale(lay, grads, r, pre, post, inv, outs[r], flags[r])
    torch.cuda.synchronize()
    ref_flags = []
    for r in range(W):
        red = oracle.reduce_slices_f16([h[r * S:(r + 1) * S] for h in host], pre, post)
        ref_g, ref_f = oracle.unscale_check(red, inv)
        ref_flags.append(ref_f)
        got = np_bits(outs[r])
        fin = np.isfinite(ref_g)
        assert same_bits(got[fin], ref_g.view(np.uint32)[fin]), f"rank {r}: {first_diff(got[fin], ref_g.view(np.uint32)[fin])}"
        assert np.array_equal(np.isnan(np_f32(outs[r])), np.isnan(ref_g))
        assert float(flags[r].item()) == ref_f, (r, bad)
    expect_any = 1.0 if bad in ("inf", "nan") else 0.0
    assert max(ref_flags) == expect_any
    if bad in ("inf", "nan"):
        assert ref_flags == [0.0] * 5 + [1.0] + [0.0] * 2      # only rank 5 sees it locally
    F.fsdp_found_inf_combine(flags)
    torch.cuda.synchronize()
    combined = oracle.found_inf_combine(ref_flags)
    assert [float(f.item()) for f in flags] == [combined] * W

    # guarded optimizer step on rank 0's shard: skipped exactly when the combined flag is set
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    p = torch.empty(S, device="cuda").normal_(0, 0.02, generator=g)
    m = torch.zeros(S, device="cuda")
    v = torch.zeros(S, device="cuda")
    hp = np_f32(p).copy()
    F.fsdp_shard_adam_step_guarded(lay, p, outs[0], m, v, 1, 1e-4, 0.9, 0.999, 1e-8, flags[0])
    torch.cuda.synchronize()
    if combined:
        assert same_bits(np_bits(p), hp.view(np.uint32)) and not np_bits(m).any() and not np_bits(v).any()
    else:
        z = np.zeros(S, np.float32)
        rp, rm, rv = oracle.adam_f32(hp, np_f32(outs[0]), z, z, 1, 1e-4, 0.9, 0.999, 1e-8)
        assert_adam_bits(np_f32(p), np_f32(m), np_f32(v), rp, rm, rv)


@pytest.mark.parametrize("gdt", ["f16", "bf16"])
def test_reduce_scatter_unscale_over_more_ranks_than_one_launch(F, gdt):
    """W = 100: the sum is carried over two launches and the check and the
    unscaling act on the finished sum.  An Inf sits in rank 80's buffer inside
    rank 3's slice; with bf16 gradients ranks 10 and 88 hold 3e38 at one
    position of rank 99's slice, so the fp32 sum overflows in the second launch."""
    unit = workloads.ragged_unit()
    W = 100
    lay = F.fsdp_layout_init(unit.shapes, W)
    S, P, N = lay.shard, lay.padded, lay.numel
    pre, post = 1.0, 100.0
    inv = float(np.float32(1.0 / 512.0))
    if gdt == "f16":
        grads = make_f16_grads(W, P, N, 190, scale=512.0)
    else:
        grads = [workloads.gen_rank_grad(P, N, w, 3, "bf16", device="cuda", std=0.5) for w in range(W)]
    grads[80][3 * S + min(5, S - 1)] = float("inf")
    if gdt == "bf16":
        for w in (10, 88):
            grads[w][99 * S] = 3.0e38
    host = [np_bits(g) for g in grads]
    reduce_slices = oracle.reduce_slices_f16 if gdt == "f16" else oracle.reduce_slices
    seen = []
    for r in (0, 3, 99):
        out = carve(S, torch.float32, r % 3, fill=POISON32)
        flag = torch.zeros(1, device="cuda")
        F.fsdp_reduce_scatter_unscale(lay, grads, r, pre, post, inv, out, flag)
        torch.cuda.synchronize()
        red = reduce_slices([h[r * S:(r + 1) * S] for h in host], pre, post)
        ref_g, ref_f = oracle.unscale_check(red, inv)
        got = np_bits(out)
        fin = np.isfinite(ref_g)
        assert same_bits(got[fin], ref_g.view(np.uint32)[fin]), f"rank {r}: {first_diff(got[fin], ref_g.view(np.uint32)[fin])}"
        assert np.array_equal(np_f32(out)[~fin], ref_g[~fin], equal_nan=True)
        assert float(flag.item()) == ref_f, r
        seen.append(ref_f)
    assert seen == ([0.0, 1.0, 0.0] if gdt == "f16" else [0.0, 1.0, 1.0])


@pytest.mark.parametrize("n,set_at", [(150, [140]), (150, [3]), (150, []), (64, [63]), (65, [64]), (127, [0, 126]), (1, [0])])
def test_found_inf_combine_over_any_number_of_ranks(F, n, set_at):
    """The all-reduce of the ranks' flags, also for more flags than one launch takes."""
    flags = [torch.zeros(1, device="cuda") for _ in range(n)]
    for i in set_at:
        flags[i].fill_(1.0)
    F.fsdp_found_inf_combine(flags)
    torch.cuda.synchronize()
    want = oracle.found_inf_combine([1.0 if i in set_at else 0.0 for i in range(n)])
    assert want == (1.0 if set_at else 0.0)
    assert [float(f.item()) for f in flags] == [want] * n


def test_grad_scaler_update_sequence(F):
    rng = np.random.default_rng(3)
    scale = torch.tensor([65536.0], device="cuda")
    tracker = torch.zeros(1, dtype=torch.int32, device="cuda")
    flag = torch.zeros(1, device="cuda")
    s_ref, t_ref = 65536.0, 0
    for i in range(60):
        found = float(rng.random() < 0.2)
        flag.fill_(found)
        F.fsdp_grad_scaler_update(scale, tracker, flag, 2.0, 0.5, 4)
        s_ref, t_ref = oracle.scaler_update(s_ref, t_ref, found, 2.0, 0.5, 4)
        torch.cuda.synchronize()
        assert float(scale.item()) == s_ref and int(tracker.item()) == t_ref, i


def test_gradient_accumulation_fp16_microbatches(F):
    unit = big_unit()
    lay = F.fsdp_layout_init(unit.shapes, 4)
    P, N = lay.padded, lay.numel
    acc = torch.zeros(P, device="cuda")
    h_acc = np.zeros(P, np.float32)
    for mb in range(2):
        g = make_f16_grads(1, P, N, 200 + mb)[0]
        F.fsdp_grad_accumulate(lay, acc, g)
        h_acc = h_acc + oracle.upcast_f16(np_bits(g))
        torch.cuda.synchronize()
        assert same_bits(np_bits(acc), h_acc.view(np.uint32))
