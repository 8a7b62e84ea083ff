"""Pins for the oracle's hybrid-sharding reduction (Sec. 3.2.2, eq. (1)) and
gradient accumulation (Sec. 3.3.4).  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import exact_f32 as ex


def _same_bits(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))


def _exact_two_level(col, G, F, pre, post):
    outer = None
    for i in range(G):
        inner = ex.div(col[i * F], pre)
        for l in range(1, F):
            inner = ex.add(inner, ex.div(col[i * F + l], pre))
        outer = inner if outer is None else ex.add(outer, inner)
    return ex.div(outer, post)


@pytest.mark.parametrize("G,F,pre,post", [(2, 8, 4.0, 4.0), (4, 2, 2.0, 4.0), (3, 4, 4.0, 3.0), (2, 3, 1.0, 6.0),
                                          (1, 5, 1.0, 5.0), (8, 1, 2.0, 4.0)])
def test_two_level_order_matches_exact_model(G, F, pre, post):
    rng = np.random.default_rng(G * 10 + F)
    S = 6
    sl = [(rng.standard_normal(S) * 10.0 ** rng.integers(-3, 4, size=S)).astype(np.float32) for _ in range(G * F)]
    sl[0][0] = -0.0
    out = oracle.reduce_slices_hybrid(sl, G, F, pre, post)
    expect = np.array([_exact_two_level([float(s[k]) for s in sl], G, F, pre, post) for k in range(S)], np.float32)
    assert _same_bits(out, expect)


def test_eq1_decomposition_is_exact_on_integers():
    """Eq. (1): the sum over all ranks equals the sum over groups of the group
    sums.  With small integer gradients every step is exact, so the hybrid
    result equals the flat reduce-scatter and the integer mean."""
    rng = np.random.default_rng(5)
    G, F, S = 2, 8, 50
    ints = rng.integers(-500, 500, size=(G * F, S))
    sl = [row.astype(np.float32) for row in ints]
    hyb = oracle.reduce_slices_hybrid(sl, G, F, 4.0, 4.0)
    flat = oracle.reduce_slices(sl, 4.0, 4.0)
    assert _same_bits(hyb, flat)
    assert [Fraction(float(x)) for x in hyb] == [Fraction(int(s), G * F) for s in ints.sum(axis=0)]


def test_single_group_is_the_flat_reduce_scatter():
    rng = np.random.default_rng(6)
    sl = [rng.standard_normal(33).astype(np.float32) for _ in range(12)]
    assert _same_bits(oracle.reduce_slices_hybrid(sl, 1, 12, 4.0, 3.0), oracle.reduce_slices(sl, 4.0, 3.0))


def test_two_level_order_differs_from_flat_order_in_binary32():
    """(1e8, 1 | -1e8, 1): group sums are 1e8 and -1e8, so the two-level result
    is 0, while the flat rank order gives 1.  Eq. (1) is exact only in real
    arithmetic; the witness shows the oracle really sums per group first."""
    sl = [np.array([v], np.float32) for v in (1e8, 1.0, -1e8, 1.0)]
    assert oracle.reduce_slices_hybrid(sl, 2, 2, 1.0, 1.0)[0] == 0.0
    assert oracle.reduce_slices(sl, 1.0, 1.0)[0] == 1.0
    # and with the groups the other way round (F = 1): plain rank order again
    assert oracle.reduce_slices_hybrid(sl, 4, 1, 1.0, 1.0)[0] == 1.0


def test_hybrid_bf16_upcast_exact():
    rng = np.random.default_rng(8)
    h = [rng.integers(0, 0x7F00, size=17).astype(np.uint16) for _ in range(8)]
    f = [(x.astype(np.uint32) << 16).view(np.float32) for x in h]
    assert _same_bits(oracle.reduce_slices_hybrid(h, 2, 4, 2.0, 4.0), oracle.reduce_slices_hybrid(f, 2, 4, 2.0, 4.0))


def test_accumulate_is_float32_addition():
    rng = np.random.default_rng(9)
    a = (rng.standard_normal(1000) * 10.0 ** rng.integers(-4, 4, size=1000)).astype(np.float32)
    b = (rng.standard_normal(1000) * 10.0 ** rng.integers(-4, 4, size=1000)).astype(np.float32)
    got = oracle.accumulate(a, b)
    assert _same_bits(got, a + b)                                   # numpy's binary32 add
    exact = np.array([ex.add(float(x), float(y)) for x, y in zip(a[:200], b[:200])], np.float32)
    assert _same_bits(got[:200], exact)
    assert _same_bits(oracle.accumulate(a, np.zeros_like(a)), a)
    h = rng.integers(0, 0x7F00, size=1000).astype(np.uint16)
    assert _same_bits(oracle.accumulate(a, h), a + (h.astype(np.uint32) << 16).view(np.float32))


def test_accumulation_with_and_without_communication_agree_on_integers():
    """Sec. 3.3.4: reduce-scatter every micro-batch and add the shards, or add
    the unsharded gradients locally and reduce-scatter once.  Integer-valued
    gradients make every step exact, so both give the same shard."""
    rng = np.random.default_rng(10)
    W, S, micro = 4, 25, 3
    P = W * S
    g = rng.integers(-100, 100, size=(micro, W, P)).astype(np.float32)
    r = 2
    with_comm = np.zeros(S, np.float32)
    for mb in range(micro):
        with_comm = oracle.accumulate(with_comm, oracle.reduce_scatter([g[mb, w] for w in range(W)], r, 2.0, 2.0))
    local = [np.zeros(P, np.float32) for _ in range(W)]
    for mb in range(micro):
        local = [oracle.accumulate(local[w], g[mb, w]) for w in range(W)]
    without_comm = oracle.reduce_scatter(local, r, 2.0, 2.0)
    assert _same_bits(with_comm, without_comm)
    expect = g.sum(axis=(0, 1))[r * S:(r + 1) * S] / W
    assert np.array_equal(with_comm.astype(np.float64), expect.astype(np.float64))
