"""Pins for the oracle's fp32 -> bf16 round-to-nearest-even cast (Sec. 4.4's
full-to-low precision cast, this build's reading of the rounding).  CPU only."""
from fractions import Fraction

import numpy as np
import torch

import oracle
from exact_f32 import bits_to_fraction

HAND = [
    (0x3F800000, 0x3F80),   # 1.0
    (0x3F808000, 0x3F80),   # tie, even below -> stays
    (0x3F818000, 0x3F82),   # tie, odd below -> up
    (0x3F808001, 0x3F81),   # just above the tie -> up
    (0x3F807FFF, 0x3F80),   # just below the tie -> down
    (0x7F7F8000, 0x7F80),   # rounds up past the largest bf16 -> +Inf
    (0x7F7F7FFF, 0x7F7F),   # largest value that stays finite
    (0xFF7F8000, 0xFF80),   # -> -Inf
    (0x00008000, 0x0000),   # denormal tie, even below -> 0
    (0x00018000, 0x0002),   # denormal tie, odd below -> up
    (0x00008001, 0x0001),   # denormal just above the tie: not flushed
    (0x80000000, 0x8000),   # -0 keeps its sign
    (0x00000000, 0x0000),
    (0x7F800000, 0x7F80),   # Inf stays Inf
    (0xFF800000, 0xFF80),
]


def test_hand_vectors():
    for u, expect in HAND:
        assert oracle.bf16_rne_scalar(u) == expect, hex(u)


def test_nan_stays_quiet_nan_with_sign():
    for u in (0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF800001, 0x7FFFFFFF, 0x7F80FFFF, 0x7FA00000):
        h = oracle.bf16_rne_scalar(u)
        assert (h & 0x7F80) == 0x7F80 and (h & 0x007F) != 0, hex(u)     # still NaN
        assert h & 0x0040                                                # quiet
        assert (h >> 15) == (u >> 31)                                    # sign kept
        assert (h & 0x003F) == ((u >> 16) & 0x003F)                      # top payload bits kept


def _nearest_bf16_exact(u: int) -> int:
    """Nearest bf16 neighbour of a finite binary32 pattern, found by comparing
    exact distances; ties go to the neighbour with an even last bit."""
    sign = u & 0x80000000
    a = u & 0x7FFFFFFF
    lo = a & 0xFFFF0000
    hi = lo + 0x10000                  # next bf16 up in magnitude (0x7F800000 stands for 2^128)
    x, xl, xh = bits_to_fraction(a), bits_to_fraction(lo), bits_to_fraction(hi)
    dl, dh = x - xl, xh - x
    if dl < dh:
        r = lo
    elif dh < dl:
        r = hi
    else:
        r = lo if ((lo >> 16) & 1) == 0 else hi
    return (sign | r) >> 16


def test_nearest_neighbour_in_exact_arithmetic():
    rng = np.random.default_rng(7)
    lows = [0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000]
    highs = list(range(0, 0x7F80, 37)) + [0x0000, 0x0001, 0x007F, 0x0080, 0x7F7E, 0x7F7F]
    pats = [(h << 16) | l for h in highs for l in lows]
    pats += [int(x) for x in rng.integers(0, 0x7F800000, size=4000)]
    pats += [p | 0x80000000 for p in pats[::3]]
    got = oracle.cast_bf16(np.array(pats, dtype=np.uint32).view(np.float32))
    for u, g in zip(pats, got):
        assert int(g) == _nearest_bf16_exact(u), hex(u)


def test_every_bit_pattern_against_torch():
    """All 2^32 binary32 patterns: non-NaN results equal torch's CPU
    float32 -> bfloat16 conversion (a library RNE cast); NaN stays NaN."""
    chunk = 1 << 26
    for first in range(0, 1 << 32, chunk):
        mine = oracle.cast_bf16_bits(first, chunk)
        u = np.arange(first, first + chunk, dtype=np.uint32)
        t = torch.from_numpy(u.view(np.int32)).view(torch.float32)
        ref = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        if (first >> 23) & 0xFF != 0xFF and ((first + chunk - 1) >> 23) & 0xFF != 0xFF:
            assert np.array_equal(mine, ref), hex(first)          # no NaN pattern in this chunk
            continue
        nan = ((u & 0x7F800000) == 0x7F800000) & ((u & 0x007FFFFF) != 0)
        assert np.array_equal(mine[~nan], ref[~nan]), hex(first)
        if nan.any():
            m = mine[nan]
            assert (((m & 0x7F80) == 0x7F80) & ((m & 0x007F) != 0)).all()


def test_cast_is_monotone_and_idempotent():
    u = np.arange(0, 0x7F800000, 4099, dtype=np.uint32)
    h = oracle.cast_bf16(u.view(np.float32)).astype(np.uint32)
    assert (np.diff(h.astype(np.int64)) >= 0).all()
    again = oracle.cast_bf16((h << 16).astype(np.uint32).view(np.float32))
    assert np.array_equal(again.astype(np.uint32), h)
