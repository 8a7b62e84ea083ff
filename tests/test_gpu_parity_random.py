"""GPU parity on seeded random cases: world size, ragged parameter shapes,
gradient dtype, rank, buffer misalignment, divide factors, rank walk and the
operation are drawn together, so that combinations the hand-written cases do
not list (a split W with a misaligned bf16 slice under the deep walk, hybrid
groups with fp16 gradients, ...) are compared with the oracle too.  The draws
come from numpy's seeded generator: every run sees the same cases."""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_helpers import POISON16, POISON32, assert_adam_parity, carve, first_diff, load_product, np_bits, np_f32, same_bits

pytestmark = pytest.mark.gpu

HP = (1e-4, 0.9, 0.999, 1e-8)
TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


@pytest.fixture(scope="module")
def F():
    assert torch.cuda.is_available()
    return load_product()


def _shapes(rng, target):
    """Ragged parameter list with about `target` elements: scalars, empties, odd vectors, small matrices."""
    shapes, n = [], 0
    while n < target:
        kind = rng.integers(0, 6)
        if kind == 0:
            s = ()
        elif kind == 1:
            s = (0, int(rng.integers(1, 5)))
        elif kind == 2:
            s = (int(rng.integers(1, 40)),)
        elif kind == 3:
            s = (int(rng.integers(1, max(2, target // 2))),)
        elif kind == 4:
            s = (int(rng.integers(1, 70)), int(rng.integers(1, 70)))
        else:
            s = (int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 9)))
        shapes.append(s)
        n += workloads.numel(s)
    return shapes


def _grads(rng, nbuf, P, N, kind, seed):
    """nbuf gradient buffers of P elements (pad zero) at random element offsets; returns (device, host)."""
    dev, host = [], []
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    for _ in range(nbuf):
        x = torch.zeros(P, dtype=torch.float32, device="cuda")
        x[:N].normal_(0.0, 1e-3, generator=g)
        t = carve(P, TORCH_DT[kind], int(rng.integers(0, 8)))
        t.copy_(x)
        dev.append(t)
        host.append(np_f32(t) if kind == "f32" else np_bits(t))
    return dev, host


def _oracle_reduce(host, kind, r, S, pre, post):
    sl = [h[r * S:(r + 1) * S] for h in host]
    return oracle.reduce_slices_f16(sl, pre, post) if kind == "f16" else oracle.reduce_slices(sl, pre, post)


def _factors(rng, F, W):
    pick = rng.integers(0, 4)
    if pick == 0:
        return F.fsdp_default_divide_factors(W)
    if pick == 1:
        return 1.0, float(W)
    if pick == 2:
        return float(W), 1.0
    return 3.0, float(W) / 3.0 if W % 3 == 0 else float(W)     # non-power-of-two pre: true divisions


# FSDP_RANDOM_CASES=<n> widens the sweep for an occasional longer run, FSDP_RANDOM_SCALE=<k> multiplies the unit sizes
CASES = list(range(int(os.environ.get("FSDP_RANDOM_CASES", "600"))))
SCALE = int(os.environ.get("FSDP_RANDOM_SCALE", "1"))


@pytest.mark.parametrize("case", CASES)
def test_random_case(F, case):
    rng = np.random.default_rng(20230411 + case)
    op = ["flatten_unshard", "reduce", "fused", "hybrid", "accumulate", "unscale", "unshard_lp", "prefetch",
          "batch"][case % 9]
    W = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 31, 33, 64, 65, 100, 130]))
    if op in ("hybrid", "accumulate", "unscale"):
        W = min(W, 64)
    if op in ("prefetch", "batch"):
        W = min(W, 65)
    target = int(rng.choice([1, 50, 3000, 40000, 300000])) * SCALE
    shapes = _shapes(rng, target)
    kind = str(rng.choice(["f32", "bf16", "f16"]))
    walk = F.FSDP_WALK_DEEP if rng.integers(0, 2) else F.FSDP_WALK_AUTO
    lay = F.fsdp_layout_init(shapes, W, reduce_walk=walk)
    S, P, N = lay.shard, lay.padded, lay.numel
    r = int(rng.integers(0, W))
    pre, post = _factors(rng, F, W)
    print(f"\n[case {case}] {op} W={W} N={N} S={S} grads={kind} rank={r} pre={pre} post={post} walk={walk}", flush=True)
    if op == "flatten_unshard":
        gen = torch.Generator(device="cuda")
        gen.manual_seed(case)
        params = []
        for i, shp in enumerate(shapes):
            n = workloads.numel(shp)
            t = carve(n, torch.float32, int(rng.integers(0, 4)))
            if n:
                t.normal_(0.0, 0.02, generator=gen)
            params.append(t.view(shp) if n else torch.empty(shp, dtype=torch.float32, device="cuda"))
        off = int(rng.integers(0, 4))
        base = carve(W * S, torch.float32, off, fill=POISON32)
        shards = [base[w * S:(w + 1) * S] for w in range(W)]
        F.fsdp_flatten_shard(lay, params, shards)
        out_kind = str(rng.choice(["f32", "bf16", "f16"]))
        flat = carve(P, TORCH_DT[out_kind], int(rng.integers(0, 8)), fill=POISON32 if out_kind == "f32" else POISON16)
        F.fsdp_unshard(lay, shards, flat)
        torch.cuda.synchronize()
        h_shards, _ = oracle.flatten_shard([np_f32(p) for p in params], W)
        ref = np.concatenate(h_shards).view(np.uint32)
        assert same_bits(np_bits(base), ref), "flatten_shard: " + first_diff(np_bits(base), ref)
        ref = {"f32": lambda: oracle.unshard_f32(h_shards).view(np.uint32), "bf16": lambda: oracle.unshard_bf16(h_shards),
               "f16": lambda: oracle.unshard_f16(h_shards)}[out_kind]()
        assert same_bits(np_bits(flat), ref), f"unshard {out_kind}: " + first_diff(np_bits(flat), ref)
        return

    if op == "unshard_lp":
        lp_kind = "bf16" if kind == "f32" else kind
        gen = torch.Generator(device="cuda")
        gen.manual_seed(case)
        shards = [carve(S, torch.float32, int(rng.integers(0, 4))).normal_(0.0, 0.02, generator=gen) for _ in range(W)]
        lps = [carve(S, TORCH_DT[lp_kind], int(rng.integers(0, 8)), fill=POISON16) for _ in range(W)]
        for w in range(W):
            F.fsdp_cast_shard(lay, shards[w], lps[w])
        flat = carve(P, TORCH_DT[lp_kind], int(rng.integers(0, 8)), fill=POISON16)
        F.fsdp_unshard_lp(lay, lps, flat)
        torch.cuda.synchronize()
        hs = [np_f32(s) for s in shards]
        ref = oracle.unshard_bf16(hs) if lp_kind == "bf16" else oracle.unshard_f16(hs)
        assert same_bits(np_bits(flat), ref), "cast_shard + unshard_lp: " + first_diff(np_bits(flat), ref)
        return

    G = int(rng.choice([g for g in (1, 2, 3, 4, 8) if g * W <= 64])) if op == "hybrid" else 1
    if op == "hybrid":
        pre, post = F.fsdp_default_divide_factors(W * G)
    grads, host = _grads(rng, W * G, P, N, kind, 1000 + case)
    out = carve(S, torch.float32, int(rng.integers(0, 4)), fill=POISON32)

    if op == "reduce":
        F.fsdp_reduce_scatter_local(lay, grads, r, pre, post, out)
        torch.cuda.synchronize()
        ref = _oracle_reduce(host, kind, r, S, pre, post)
        assert same_bits(np_bits(out), ref.view(np.uint32)), first_diff(np_bits(out), ref.view(np.uint32))
    elif op == "hybrid":
        F.fsdp_reduce_scatter_hybrid(lay, grads, G, r, pre, post, out)
        torch.cuda.synchronize()
        sl = [h[r * S:(r + 1) * S] for h in host]
        if kind == "f16":
            sl = [oracle.upcast_f16(x) for x in sl]      # exact: the two-level sum then runs on fp32 inputs
        ref = oracle.reduce_slices_hybrid(sl, G, W, pre, post)
        assert same_bits(np_bits(out), ref.view(np.uint32)), first_diff(np_bits(out), ref.view(np.uint32))
    elif op == "accumulate":
        out.normal_(0.0, 1e-3)
        h_acc = np_f32(out).copy()
        F.fsdp_reduce_scatter_accumulate(lay, grads, r, pre, post, out)
        torch.cuda.synchronize()
        ref = oracle.accumulate(h_acc, _oracle_reduce(host, kind, r, S, pre, post))
        assert same_bits(np_bits(out), ref.view(np.uint32)), first_diff(np_bits(out), ref.view(np.uint32))
    elif op == "unscale":
        plant = rng.integers(0, 3)
        if plant and N:
            j = int(rng.integers(0, N))
            grads[int(rng.integers(0, W))][j] = float("inf") if plant == 1 else float("nan")
            host = [np_f32(g) if kind == "f32" else np_bits(g) for g in grads]
        flag = torch.zeros(1, device="cuda")
        inv = 1.0 / 1024.0
        F.fsdp_reduce_scatter_unscale(lay, grads, r, pre, post, inv, out, flag)
        torch.cuda.synchronize()
        ref, found = oracle.unscale_check(_oracle_reduce(host, kind, r, S, pre, post), inv)
        assert same_bits(np_bits(out), ref.view(np.uint32)), first_diff(np_bits(out), ref.view(np.uint32))
        assert float(flag.item()) == float(found)
    else:       # fused / prefetch / batch: Adam at a random step from a random state
        t = int(rng.choice([1, 2, 9, 300]))
        gen = torch.Generator(device="cuda")
        gen.manual_seed(5000 + case)
        p = carve(S, torch.float32, int(rng.integers(0, 4))).normal_(0.0, 0.02, generator=gen)
        m = carve(S, torch.float32, int(rng.integers(0, 4))).normal_(0.0, 1e-3, generator=gen)
        v = carve(S, torch.float32, int(rng.integers(0, 4))).uniform_(0.0, 1e-6, generator=gen)
        if t == 1:
            m.zero_()
            v.zero_()
        hp0, hm0, hv0 = np_f32(p).copy(), np_f32(m).copy(), np_f32(v).copy()
        want_out = bool(rng.integers(0, 2)) or W > 64
        want_lp = bool(rng.integers(0, 2))
        lp = carve(S, torch.bfloat16, int(rng.integers(0, 8)), fill=POISON16) if want_lp else None
        g_out = out if want_out else None
        # an unshard of another unit rides along in the prefetch and batch forms
        W2 = int(rng.choice([1, 3, 8, 12, 40]))
        lay2 = F.fsdp_layout_init(_shapes(rng, int(rng.choice([10, 5000, 90000]))), W2)
        shards2 = [carve(lay2.shard, torch.float32, int(rng.integers(0, 4))).normal_(0.0, 0.02, generator=gen)
                   for _ in range(W2)]
        flat2 = carve(lay2.padded, torch.bfloat16, int(rng.integers(0, 8)), fill=POISON16)
        if op == "fused":
            F.fsdp_reduce_scatter_adam_fused(lay, grads, r, pre, post, g_out, p, m, v, t, *HP, lp)
        elif op == "prefetch":
            F.fsdp_reduce_scatter_adam_prefetch_unshard(lay, grads, r, pre, post, g_out, p, m, v, t, *HP, lp, lay2,
                                                        shards2, flat2)
        else:
            b = F.Batch()
            b.add_unshard(lay2, shards2, flat2)
            b.add_reduce_scatter_adam(lay, grads, r, pre, post, g_out, p, m, v, *HP, lp)
            b.launch(t)
            torch.cuda.synchronize()
            b.close()
        torch.cuda.synchronize()
        ref_g = _oracle_reduce(host, kind, r, S, pre, post)
        if want_out:
            assert same_bits(np_bits(out), ref_g.view(np.uint32)), first_diff(np_bits(out), ref_g.view(np.uint32))
        assert_adam_parity(np_f32(p), np_f32(m), np_f32(v), hp0, ref_g, hm0, hv0, t, HP, "Adam")
        if want_lp:
            ref_lp = oracle.cast_bf16(np_f32(p))
            assert same_bits(np_bits(lp), ref_lp), "bf16 copy of the updated shard"
        if op != "fused":
            ref2 = oracle.unshard_bf16([np_f32(s) for s in shards2])
            assert same_bits(np_bits(flat2), ref2), "rider unshard: " + first_diff(np_bits(flat2), ref2)
