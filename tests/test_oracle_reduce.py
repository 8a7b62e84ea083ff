"""Pins for the oracle's reduce-scatter (Sec. 3, Sec. 3.2.2 eq. (1)): rank-
ordered binary32 sum with pre/post divide, one rank's chunk.  CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import exact_f32 as ex


def _exact_rank_ordered(col, pre, post):
    """One output element from W inputs by exact-rational evaluation with one
    rounding per IEEE operation."""
    acc = ex.div(col[0], pre)
    for x in col[1:]:
        acc = ex.add(acc, ex.div(x, pre))
    return ex.div(acc, post)


def _same_bits(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))


@pytest.mark.parametrize("W,pre,post", [(1, 1.0, 1.0), (2, 1.0, 2.0), (3, 3.0, 1.0), (4, 2.0, 2.0),
                                        (5, 1.0, 5.0), (12, 4.0, 3.0)])
def test_brute_force_sum_then_slice_tiny(W, pre, post):
    """reduce-scatter == slice of the full reduction == exact-arithmetic model."""
    rng = np.random.default_rng(100 + W)
    S = 5
    P = S * W
    bufs = [(rng.standard_normal(P) * 10.0 ** rng.integers(-3, 4, size=P)).astype(np.float32) for _ in range(W)]
    bufs[0][:3] = [-0.0, 0.0, 1e-40]           # signed zeros and a denormal
    for b in bufs[1:]:
        b[0] = -0.0
    full = oracle.reduce_full_f32(bufs, pre, post)
    expect = np.array([_exact_rank_ordered([float(b[j]) for b in bufs], pre, post) for j in range(P)],
                      dtype=np.float32)
    assert _same_bits(full, expect)
    outs = [oracle.reduce_scatter(bufs, r, pre, post) for r in range(W)]
    for r in range(W):
        assert _same_bits(outs[r], full[r * S:(r + 1) * S])
    assert _same_bits(np.concatenate(outs), full)
    # slice form: only the rank's slices are handed over
    for r in range(W):
        sl = [b[r * S:(r + 1) * S].copy() for b in bufs]
        assert _same_bits(oracle.reduce_slices(sl, pre, post), outs[r])


def test_minus_zero_survives():
    """The accumulator starts from rank 0's term, so all -0 inputs give -0."""
    bufs = [np.array([-0.0, -0.0], np.float32) for _ in range(2)]
    bufs[1][1] = 0.0
    out = oracle.reduce_scatter(bufs, 0, 2.0, 1.0)
    assert out[0] == 0 and math.copysign(1.0, float(out[0])) == -1.0
    out1 = oracle.reduce_scatter(bufs, 1, 2.0, 1.0)
    assert math.copysign(1.0, float(out1[0])) == 1.0     # (-0) + (+0) = +0


def test_order_witness_sequential_rank_order():
    """((1e8 + 1) - 1e8) + 1 = 1 in binary32 rank order; a pairwise tree or the
    reverse order would give 0."""
    vals = [1e8, 1.0, -1e8, 1.0]
    bufs = [np.full(4, v, np.float32) for v in vals]
    out = oracle.reduce_scatter(bufs, 2, 1.0, 1.0)
    assert out.tolist() == [1.0]
    # the other association orders really differ, so the witness is meaningful
    f = np.float32
    assert (f(1e8) + f(1.0)) + (f(-1e8) + f(1.0)) == 0.0
    assert ((f(1.0) + f(-1e8)) + f(1.0)) + f(1e8) == 0.0


def test_integer_gradients_give_exact_mean():
    """Small integers and W a power of two: every step is exact, so the result
    is the integer sum over W exactly."""
    rng = np.random.default_rng(3)
    W, S = 8, 33
    ints = rng.integers(-1000, 1000, size=(W, W * S))
    bufs = [row.astype(np.float32) for row in ints]
    for r in (0, 3, 7):
        out = oracle.reduce_scatter(bufs, r, 4.0, 2.0)
        expect = [Fraction(int(s), W) for s in ints[:, r * S:(r + 1) * S].sum(axis=0)]
        assert [Fraction(float(x)) for x in out] == expect


def test_identical_short_mantissa_ranks_power_of_two_is_identity():
    """Identical gradients with 8-bit mantissas on W = 16 ranks: every partial
    sum k * g / 4 (k <= 16) fits in 24 bits, so the mean is g exactly."""
    rng = np.random.default_rng(4)
    W, S = 16, 40
    g = rng.standard_normal(W * S).astype(np.float32)
    g = (g.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    out = oracle.reduce_scatter([g.copy() for _ in range(W)], 5, 4.0, 4.0)
    assert _same_bits(out, g[5 * S:6 * S])


def test_pre_and_post_are_true_divisions():
    """post = 3 is a real rounding step: x / 3, not x * (1/3)."""
    xs = np.arange(1, 2000, dtype=np.float32)
    out = oracle.reduce_scatter([xs], 0, 1.0, 3.0)
    expect = np.array([ex.div(float(x), 3.0) for x in xs], np.float32)
    assert _same_bits(out, expect)
    recip = xs * np.float32(1.0 / 3.0)
    assert not _same_bits(out, recip)            # the two really differ somewhere
    out = oracle.reduce_slices([xs, np.zeros_like(xs)], 3.0, 1.0)
    assert _same_bits(out, expect)


def test_pre_divide_happens_before_the_sum():
    """Dividing each term before adding is what keeps large gradients finite:
    3e38 on two ranks with pre = 2 gives 3e38; summing first would overflow."""
    big = np.array([3e38, -3e38], np.float32)
    out = oracle.reduce_slices([big, big], 2.0, 1.0)
    assert _same_bits(out, big)
    tiny = np.array([1e-45], np.float32)                 # smallest denormal: halves to zero (tie to even)
    out = oracle.reduce_slices([tiny, tiny], 2.0, 1.0)
    assert out[0] == 0.0


def test_bf16_inputs_upcast_exactly():
    """bf16 gradient buffers: upcast is bits << 16, then the fp32 path."""
    rng = np.random.default_rng(5)
    W, S = 4, 21
    h = [rng.integers(0, 0x7F80, size=W * S).astype(np.uint16) | (rng.integers(0, 2, size=W * S).astype(np.uint16) << 15)
         for _ in range(W)]
    f = [(x.astype(np.uint32) << 16).view(np.float32) for x in h]
    for r in range(W):
        assert _same_bits(oracle.reduce_scatter(h, r, 2.0, 2.0), oracle.reduce_scatter(f, r, 2.0, 2.0))
    col = [float(x[7]) for x in f]
    assert float(oracle.reduce_scatter(h, 0, 2.0, 2.0)[7]) == _exact_rank_ordered(col, 2.0, 2.0)


def test_world_size_one():
    g = np.array([1.5, -2.25, 0.0, -0.0], np.float32)
    assert _same_bits(oracle.reduce_scatter([g], 0, 1.0, 1.0), g)
