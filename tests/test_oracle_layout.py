"""Pins for the oracle's layout, flatten/pad/chunk, unshard and views
(Sec. 3.2.1, Sec. 3.2.3).  CPU only."""
import os

import numpy as np
import pytest

import oracle
import workloads


def _read_golden(path):
    kv = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            kv[k] = [int(x) for x in v]
    return kv


def test_fig3_worked_example(golden_dir):
    """Sec. 3.2.1 / Fig. 3: 4x3 Linear over 16 ranks: one element per rank, the
    last rank holds the pad."""
    g = _read_golden(os.path.join(golden_dir, "fig3_linear_4x3_w16.txt"))
    shapes = [tuple(g["weight_shape"]), tuple(g["bias_shape"])]
    W = g["world_size"][0]
    off, N, S, P, pad = oracle.layout(shapes, W)
    assert N == g["numel"][0] and S == g["shard_numel"][0]
    assert P == g["padded_numel"][0] and pad == g["pad"][0]
    assert off == [0, 12, 15]
    w = np.arange(1, 13, dtype=np.float32).reshape(3, 4)
    b = np.arange(13, 16, dtype=np.float32)
    shards, _ = oracle.flatten_shard([w, b], W)
    assert len(shards) == 16 and all(s.shape == (1,) for s in shards)
    # every rank but the last holds one real element, in flatten order
    assert [float(s[0]) for s in shards[:15]] == [float(i) for i in range(1, 16)]
    pr = g["pad_rank"][0]
    assert shards[pr].view(np.uint32)[0] == 0      # the pad is +0.0f


@pytest.mark.parametrize("W", [1, 2, 3, 5, 8, 12, 16, 64])
def test_padding_closed_form_and_bound(W):
    """Sec. 3.2.1: padding makes the size divisible by W and is at most W-1."""
    rng = np.random.default_rng(W)
    for _ in range(50):
        p = int(rng.integers(1, 6))
        shapes = [tuple(int(x) for x in rng.integers(0, 7, size=rng.integers(0, 4))) for _ in range(p)]
        off, N, S, P, pad = oracle.layout(shapes, W)
        n_i = [int(np.prod(s, dtype=np.int64)) if len(s) else 1 for s in shapes]
        assert off == [sum(n_i[:i]) for i in range(p + 1)]
        assert N == sum(n_i)
        assert P % W == 0 and P // W == S
        assert 0 <= pad <= W - 1 and pad == P - N
        assert P == -(-N // W) * W                  # ceil(N/W) * W


def test_layout_special_cases():
    # W = 1: no pad, the shard is the flat buffer
    off, N, S, P, pad = oracle.layout([(3, 5), (7,)], 1)
    assert (N, S, P, pad) == (22, 22, 22, 0)
    # N < W: ranks >= N hold only zeros
    a = np.array([1.5, -2.5, 3.5], dtype=np.float32)
    shards, (off, N, S, P, pad) = oracle.flatten_shard([a], 8)
    assert (N, S, P, pad) == (3, 1, 8, 5)
    assert [float(s[0]) for s in shards] == [1.5, -2.5, 3.5, 0, 0, 0, 0, 0]
    # N multiple of W: no pad
    assert oracle.layout([(4, 6)], 8)[4] == 0
    # a scalar has numel 1, a zero dim has numel 0
    off, N, *_ = oracle.layout([(), (0, 4), (2,)], 2)
    assert off == [0, 1, 1, 3] and N == 3
    with pytest.raises(ValueError):
        oracle.layout([(2,)], 0)
    with pytest.raises(ValueError):
        oracle.layout([(-1,)], 2)


def test_config_sizes_table():
    """Sizes of the five benchmark configurations, computed by hand from the
    shapes: N = 12 d^2 + 13 d for a GPT block with ffn = 4d."""
    def gpt(d):
        return 12 * d * d + 13 * d
    cases = [
        (workloads.config(0).units[0], 8, gpt(768), 0),
        (workloads.config(1).units[0], 8, 50257 * 768 + 1024 * 768 + 2 * 768, 0),
        (workloads.config(2).units[0], 12, gpt(2048), 4),
        (workloads.config(3).units[0], 64, 4 * 4096 * 4096 + 3 * 4096 * 11008 + 2 * 4096, 0),
        (workloads.config(4).units[0], 16, gpt(12288), 0),
    ]
    for unit, W, N_expect, pad_expect in cases:
        off, N, S, P, pad = oracle.layout(unit.shapes, W)
        assert N == N_expect and pad == pad_expect and P == N + pad and S * W == P
    assert gpt(768) == 7_087_872 and gpt(2048) == 50_358_272 and gpt(12288) == 1_812_099_072
    # cfg 2: odd shard size, the last rank holds 4 pad elements
    assert oracle.layout(workloads.config(2).units[0].shapes, 12)[2] == 4_196_523


def _ragged_params(seed=0):
    rng = np.random.default_rng(seed)
    unit = workloads.ragged_unit()
    return unit, [rng.standard_normal(s).astype(np.float32) for s in unit.shapes]


@pytest.mark.parametrize("W", [1, 2, 3, 7, 8, 12, 64])
def test_flatten_matches_concatenate_and_views_invert(W):
    """flatten+pad is numpy.concatenate plus zero fill; concat(shards) == flat;
    views of the fp32 unshard give back every parameter bit for bit."""
    unit, params = _ragged_params(W)
    shards, (off, N, S, P, pad) = oracle.flatten_shard(params, W)
    ref = np.concatenate([a.reshape(-1) for a in params] + [np.zeros(pad, np.float32)])
    flat = np.concatenate(shards)
    assert flat.size == P
    assert np.array_equal(flat.view(np.uint32), ref.view(np.uint32))
    assert not flat[N:].view(np.uint32).any()
    un = oracle.unshard_f32(shards)
    assert np.array_equal(un.view(np.uint32), ref.view(np.uint32))
    for v, a in zip(oracle.views(un, off, unit.shapes), params):
        assert v.shape == a.shape
        assert np.array_equal(v.view(np.uint32), a.view(np.uint32))
        assert v.size == 0 or np.shares_memory(v, un)          # zero copy


def test_flatten_is_row_major_and_order_sensitive():
    a = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    b = np.array([7, 8], dtype=np.float32)
    flat = oracle.flatten_pad([a, b], 9)
    assert flat.tolist() == [1, 2, 3, 4, 5, 6, 7, 8, 0]
    flat = oracle.flatten_pad([b, a], 8)
    assert flat.tolist() == [7, 8, 1, 2, 3, 4, 5, 6]
    # a transposed (non-contiguous) input is flattened in its logical row-major order
    flat = oracle.flatten_pad([a.T], 6)
    assert flat.tolist() == [1, 4, 2, 5, 3, 6]


@pytest.mark.parametrize("W", [1, 3, 8])
def test_unshard_bf16_is_cast_of_parameters(W):
    """cast-then-gather == gather-then-cast; views of the bf16 buffer equal the
    cast of each original parameter."""
    unit, params = _ragged_params(10 + W)
    shards, (off, N, S, P, pad) = oracle.flatten_shard(params, W)
    lp = oracle.unshard_bf16(shards)
    assert lp.dtype == np.uint16 and lp.size == P
    assert np.array_equal(lp, oracle.cast_bf16(np.concatenate(shards)))
    assert not lp[N:].any()
    for v, a in zip(oracle.views(lp, off, unit.shapes), params):
        assert np.array_equal(v, oracle.cast_bf16(a))


@pytest.mark.parametrize("W", [1, 3, 8])
def test_gather_of_cast_shards_equals_unshard(W):
    """Each rank casts its own shard and the gather moves bf16 (Sec. 4.4): the
    same bytes as casting while gathering; and the gather is a concatenation."""
    unit, params = _ragged_params(20 + W)
    shards, (off, N, S, P, pad) = oracle.flatten_shard(params, W)
    lp = [oracle.cast_bf16(s) for s in shards]
    got = oracle.gather_lp(lp)
    assert np.array_equal(got, np.concatenate(lp))
    assert np.array_equal(got, oracle.unshard_bf16(shards))


@pytest.mark.parametrize("cfg", range(workloads.NUM_CONFIGS))
def test_memory_model_of_the_sharded_layout(cfg):
    """Sec. 3.2.1: peak parameter memory is O(sum_i psi_i / F + max_i psi_i);
    Sec. 4.4 with mixed precision: K_full / F * sum_i psi_i + K_low * max_i psi_i.
    The layout must realise these with no more slack than the pad: per unit the
    persistent full-precision shard is K_full * S_i with
    psi_i / F <= S_i < psi_i / F + 1, and the transient low-precision unsharded
    buffer is K_low * P_i with psi_i <= P_i <= psi_i + F - 1."""
    wl = workloads.config(cfg)
    F = wl.world_size
    K_full, K_low = 4, 2
    psis, Ss, Ps = [], [], []
    for u in wl.units:
        off, N, S, P, pad = oracle.layout(u.shapes, F)
        assert N == sum(workloads.numel(s) for s in u.shapes)
        assert N <= S * F < N + F and P == S * F and pad == P - N
        psis.append(N); Ss.append(S); Ps.append(P)
    persistent = K_full * sum(Ss)
    transient = K_low * max(Ps)
    model = K_full * sum(psis) / F + K_low * max(psis)
    slack = K_full * len(psis) + K_low * (F - 1)             # < one element per unit, plus one unit's pad
    assert model <= persistent + transient < model + slack
    # without sharding the same parameters would take K_full * sum psi: the saving approaches a factor F
    assert persistent <= K_full * sum(psis) / F + K_full * len(psis)
