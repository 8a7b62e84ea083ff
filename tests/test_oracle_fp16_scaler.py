"""Pins for the oracle's fp16 cast and sharded gradient scaler (Sec. 4.4).  CPU only."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from exact_f32 import bits_to_fraction


def _f16_value(h: int) -> Fraction:
    """Value of a non-negative finite binary16 pattern; Inf's pattern stands for 2^16."""
    exp, man = (h >> 10) & 0x1F, h & 0x3FF
    if exp == 0:
        return Fraction(man, 1 << 24)
    return Fraction(man + 1024) * Fraction(2) ** (exp - 25)


def _nearest_f16_exact(u: int) -> int:
    sign = (u >> 16) & 0x8000
    x = bits_to_fraction(u & 0x7FFFFFFF)
    # bracket x between consecutive half patterns (pattern order = value order for non-negatives)
    lo, hi = 0, 0x7C00
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if _f16_value(mid) <= x:
            lo = mid
        else:
            hi = mid
    if x >= _f16_value(0x7C00):
        return sign | 0x7C00
    dl, dh = x - _f16_value(lo), _f16_value(hi) - x
    r = lo if dl < dh else hi if dh < dl else (lo if lo % 2 == 0 else hi)
    return sign | r


HAND = [(0x3F800000, 0x3C00), (0x477FE000, 0x7BFF), (0x477FF000, 0x7C00), (0x477FEFFF, 0x7BFF), (0x47800000, 0x7C00),
        (0x33800000, 0x0001), (0x33000000, 0x0000), (0x33000001, 0x0001), (0x38800000, 0x0400), (0x387FE000, 0x0400),
        (0x387FC000, 0x03FF), (0x80000000, 0x8000), (0x00000001, 0x0000), (0x7F800000, 0x7C00), (0xFF800000, 0xFC00),
        (0x3F801000, 0x3C00), (0x3F803000, 0x3C02), (0x3F801001, 0x3C01), (0xC7FFFFFF, 0xFC00)]


def test_f16_hand_vectors():
    for u, expect in HAND:
        assert oracle.f16_rne_scalar(u) == expect, hex(u)


def test_f16_nan_rule():
    for u in (0x7FC00000, 0xFFC00000, 0x7F800001, 0x7FA00000, 0x7F802000):
        h = oracle.f16_rne_scalar(u)
        assert (h & 0x7C00) == 0x7C00 and (h & 0x03FF) != 0 and (h & 0x0200)
        assert (h >> 15) == (u >> 31)


def test_f16_nearest_neighbour_exact():
    rng = np.random.default_rng(3)
    pats = [int(x) for x in rng.integers(0x33000000 - 0x01000000, 0x47900000, size=3000)]
    pats += [(e << 23) | m for e in range(100, 145) for m in (0, 1, 0x0FFF, 0x1000, 0x1001, 0x2FFF, 0x3000, 0x7FFFFF)]
    pats += [p | 0x80000000 for p in pats[::5]]
    got = oracle.cast_f16(np.array(pats, dtype=np.uint32).view(np.float32))
    for u, g in zip(pats, got):
        assert int(g) == _nearest_f16_exact(u), hex(u)


def _check_against_numpy(u):
    mine = oracle.cast_f16(u.view(np.float32))
    with np.errstate(over="ignore", under="ignore"):
        ref = u.view(np.float32).astype(np.float16).view(np.uint16)
    nan = ((u & 0x7F800000) == 0x7F800000) & ((u & 0x007FFFFF) != 0)
    bad = np.flatnonzero(mine[~nan] != ref[~nan])
    assert bad.size == 0, hex(int(u[~nan][bad[0]]))


def test_f16_against_numpy_conversion():
    """numpy's float32 -> float16 (a library RNE cast): every value of the top
    19 bits with the rounding-relevant low patterns, and a random sample of all
    patterns."""
    top = np.arange(0, 1 << 19, dtype=np.uint32) << 13
    for low in (0, 1, 0x0FFF, 0x1000, 0x1001, 0x1FFF):
        _check_against_numpy(top | np.uint32(low))
    rng = np.random.default_rng(11)
    _check_against_numpy(rng.integers(0, 1 << 32, size=1 << 22, dtype=np.uint64).astype(np.uint32))


def test_f16_all_patterns_against_torch():
    """Every one of the 2^32 binary32 patterns against torch's CPU conversion
    (a second library RNE cast); NaNs follow the oracle's own rule: sign kept,
    quiet bit set, top payload bits kept."""
    chunk = 1 << 26
    for first in range(0, 1 << 32, chunk):
        mine = oracle.cast_f16_bits(first, chunk)
        u = np.arange(first, first + chunk, dtype=np.uint32)
        ref = torch.from_numpy(u.view(np.int32)).view(torch.float32).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
        if (first >> 23) & 0xFF != 0xFF and ((first + chunk - 1) >> 23) & 0xFF != 0xFF:
            assert np.array_equal(mine, ref), hex(first)          # no NaN pattern in this chunk
            continue
        nan = ((u & 0x7F800000) == 0x7F800000) & ((u & 0x007FFFFF) != 0)
        assert np.array_equal(mine[~nan], ref[~nan]), hex(first)
        if nan.any():
            m, un = mine[nan], u[nan]
            assert (((m & 0x7C00) == 0x7C00) & ((m & 0x0200) != 0)).all()
            assert np.array_equal(m >> 15, (un >> 31).astype(np.uint16))
            assert np.array_equal(m & 0x01FF, ((un >> 13) & 0x01FF).astype(np.uint16))


@pytest.mark.parametrize("W", [1, 3, 8])
def test_unshard_f16_is_cast_of_the_concatenated_shards(W):
    """Sec. 4.4 gather in fp16: slot w of the flat buffer holds rank w's shard,
    cast element by element.  Ragged shard length, distinct content per rank
    (so that a reversed or rank-ignoring gather cannot pass), compared with the
    pinned cast of numpy's concatenation and with numpy's own conversion."""
    rng = np.random.default_rng(40 + W)
    S = 37
    shards = [((rng.standard_normal(S) * 10.0 ** rng.integers(-6, 5, size=S)).astype(np.float32) + np.float32(w))
              for w in range(W)]
    got = oracle.unshard_f16(shards)
    assert got.shape == (W * S,)
    assert np.array_equal(got, oracle.cast_f16(np.concatenate(shards)))
    with np.errstate(over="ignore", under="ignore"):
        assert np.array_equal(got, np.concatenate(shards).astype(np.float16).view(np.uint16))
    for w in range(W):
        assert np.array_equal(got[w * S:(w + 1) * S], oracle.cast_f16(shards[w]))


def test_f16_upcast_all_patterns_against_numpy():
    h = np.arange(0, 1 << 16, dtype=np.uint16)
    mine = oracle.upcast_f16(h).view(np.uint32)
    ref = h.view(np.float16).astype(np.float32).view(np.uint32)
    nan = ((h & 0x7C00) == 0x7C00) & ((h & 0x03FF) != 0)
    assert np.array_equal(mine[~nan], ref[~nan])
    assert np.isnan(mine[nan].view(np.float32)).all()


def test_f16_reduce_is_upcast_then_fp32_reduce():
    rng = np.random.default_rng(4)
    h = [rng.integers(0, 0x7BFF, size=40).astype(np.uint16) | (rng.integers(0, 2, size=40).astype(np.uint16) << 15)
         for _ in range(6)]
    f = [oracle.upcast_f16(x) for x in h]
    a = oracle.reduce_slices_f16(h, 2.0, 3.0)
    b = oracle.reduce_slices(f, 2.0, 3.0)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_unscale_check_against_torch():
    rng = np.random.default_rng(5)
    for case in range(6):
        g = (rng.standard_normal(257) * 1e3).astype(np.float32)
        if case == 1:
            g[100] = np.inf
        if case == 2:
            g[5] = np.nan
        if case == 3:
            g[7] = -np.inf
        if case == 4:
            g[9] = 3e38                       # finite, and stays finite when scaled down
        inv = np.float32(1.0 / 65536.0) if case != 5 else np.float32(3.0)
        if case == 5:
            g[11] = 2e38                      # overflows when multiplied by 3
        mine, found = oracle.unscale_check(g, float(inv))
        tg = [torch.tensor(g.copy())]
        tf = torch.zeros(1)
        with np.errstate(over="ignore", invalid="ignore"):
            torch._amp_foreach_non_finite_check_and_unscale_(tg, tf, torch.tensor([inv]))
        assert found == float(tf.item()), case
        ok = np.isfinite(mine)
        assert np.array_equal(mine[ok].view(np.uint32), tg[0].numpy()[ok].view(np.uint32))
        assert found == (0.0 if case in (0, 4, 5) else 1.0)    # the check reads the value before the multiply


def test_sharded_flag_equals_flag_of_the_whole_gradient():
    """Only one rank's shard holds the Inf; every rank must still skip."""
    W, S = 8, 16
    full = np.ones(W * S, np.float32)
    full[5 * S + 3] = np.inf
    flags = [oracle.unscale_check(full[r * S:(r + 1) * S], 0.5)[1] for r in range(W)]
    assert flags == [0.0] * 5 + [1.0] + [0.0] * 2           # a local decision would split the ranks
    combined = oracle.found_inf_combine(flags)
    assert combined == oracle.unscale_check(full, 0.5)[1] == 1.0
    assert oracle.found_inf_combine([0.0] * W) == 0.0


def test_scaler_update_against_torch():
    rng = np.random.default_rng(6)
    scale, tracker = 65536.0, 0
    ts, tt = torch.tensor([65536.0]), torch.tensor([0], dtype=torch.int32)
    for i in range(200):
        found = float(rng.random() < 0.15)
        scale, tracker = oracle.scaler_update(scale, tracker, found, 2.0, 0.5, 5)
        torch._amp_update_scale_(ts, tt, torch.tensor([found]), 2.0, 0.5, 5)
        assert scale == float(ts.item()) and tracker == int(tt.item()), i
    # closed form: k good steps in a row with interval n multiply the scale by 2^(k // n)
    s, t = 1.0, 0
    for _ in range(12):
        s, t = oracle.scaler_update(s, t, 0.0, 2.0, 0.5, 4)
    assert (s, t) == (8.0, 0)
    assert oracle.scaler_update(8.0, 3, 1.0, 2.0, 0.5, 4) == (4.0, 0)
