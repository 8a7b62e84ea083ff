"""Pins for the oracle's sharded Adam step (Sec. 5.4 names Adam; the update
rule is this build's reading: Kingma & Ba with bias correction).  CPU only."""
from fractions import Fraction
import math

import numpy as np
import pytest
import torch

import oracle

LR, B1, B2, EPS = 1e-4, 0.9, 0.999, 1e-8


def f32(x):
    return float(np.float32(x))


def test_closed_form_first_step_from_zero_state():
    """t = 1, m = v = 0: m = (1-b1) g, v = (1-b2) g^2 and the bias corrections
    cancel, so p_new = p - lr * g / (|g| + eps)."""
    g = np.array([1e-3, -1e-3, 3.7e-5, -2.0, 1e-9, 5e-12, 123.0], np.float32)
    p = np.array([0.02, -0.01, 0.5, 1.0, -3.0, 0.25, 0.0], np.float32)
    z = np.zeros_like(p)
    pn, mn, vn = oracle.adam_f32(p, g, z, z, 1, LR, B1, B2, EPS)
    lr, b1, b2, eps = (Fraction(f32(x)) for x in (LR, B1, B2, EPS))
    for k in range(len(g)):
        gk, pk = Fraction(float(g[k])), Fraction(float(p[k]))
        m_exact = (1 - b1) * gk
        v_exact = (1 - b2) * gk * gk
        step = lr * gk / (abs(gk) + eps)
        assert abs(Fraction(float(mn[k])) - m_exact) <= Fraction(1, 10 ** 6) * abs(m_exact)
        assert abs(Fraction(float(vn[k])) - v_exact) <= Fraction(1, 10 ** 6) * abs(v_exact)
        p_exact = pk - step
        tol = Fraction(1, 10 ** 6) * max(abs(p_exact), abs(pk))
        assert abs(Fraction(float(pn[k])) - p_exact) <= tol, k
        assert abs(Fraction(float(pn[k])) - pk) <= lr + tol                 # |step| <= lr


def test_zero_gradient_changes_nothing_at_first_step():
    p = np.array([0.3, -0.0, 0.0, 1e-30], np.float32)
    z = np.zeros_like(p)
    pn, mn, vn = oracle.adam_f32(p, z, z, z, 1, LR, B1, B2, EPS)
    assert np.array_equal(pn.view(np.uint32)[[0, 3]], p.view(np.uint32)[[0, 3]])
    assert (pn[1:3] == 0).all() and not mn.any() and not vn.any()


def test_pad_stays_zero():
    """Pad positions hold p = g = m = v = 0 and must stay zero through a step."""
    z = np.zeros(5, np.float32)
    for t in (1, 2, 100):
        pn, mn, vn = oracle.adam_f32(z, z, z, z, t, LR, B1, B2, EPS)
        assert not pn.any() and not mn.any() and not vn.any()


@pytest.mark.parametrize("t", [1, 2, 5, 1000])
def test_single_step_matches_torch_adam_float64(t):
    """torch.optim.Adam (float64, no weight decay, no amsgrad) from the same
    state; the oracle's binary64 evaluation must agree to rounding noise and
    the binary32 evaluation to the parity tolerance."""
    rng = np.random.default_rng(t)
    n = 257
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32) if t > 1 else np.zeros(n, np.float32)
    v = (rng.random(n) * 1e-6).astype(np.float32) if t > 1 else np.zeros(n, np.float32)
    tp = torch.tensor(p, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=f32(LR), betas=(f32(B1), f32(B2)), eps=f32(EPS))
    tp.grad = torch.tensor(g, dtype=torch.float64)
    if t > 1:
        opt.state[tp]["step"] = torch.tensor(float(t - 1))
        opt.state[tp]["exp_avg"] = torch.tensor(m, dtype=torch.float64)
        opt.state[tp]["exp_avg_sq"] = torch.tensor(v, dtype=torch.float64)
    opt.step()
    ref_p = tp.detach().numpy()
    ref_m = opt.state[tp]["exp_avg"].numpy()
    ref_v = opt.state[tp]["exp_avg_sq"].numpy()
    p64, m64, v64 = oracle.adam_f64(p, g, m, v, t, LR, B1, B2, EPS)
    assert np.allclose(p64, ref_p, rtol=1e-12, atol=0)
    assert np.allclose(m64, ref_m, rtol=1e-12, atol=1e-300)
    assert np.allclose(v64, ref_v, rtol=1e-12, atol=1e-300)
    p32, m32, v32 = oracle.adam_f32(p, g, m, v, t, LR, B1, B2, EPS)
    # m can cancel (b1*m and (1-b1)*g of opposite sign): bound by the larger term
    m_scale = np.maximum(np.abs(ref_m), np.maximum(np.abs(m) * f32(B1), np.abs(g) * (1 - f32(B1))))
    assert (np.abs(m32 - ref_m) <= 1e-6 * m_scale).all()
    assert (np.abs(v32 - ref_v) <= 1e-6 * np.abs(ref_v)).all()
    assert (np.abs(p32 - ref_p) <= 1e-6 * np.maximum(np.abs(ref_p), np.abs(p))).all()


def test_ten_steps_track_torch_adam():
    rng = np.random.default_rng(11)
    n = 64
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    tp = torch.tensor(p, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=f32(LR), betas=(f32(B1), f32(B2)), eps=f32(EPS))
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    for t in range(1, 11):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = oracle.adam_f32(p, g, m, v, t, LR, B1, B2, EPS)
    assert (np.abs(p - tp.detach().numpy()) <= 1e-5 * np.abs(p).max()).all()
    assert np.allclose(v, opt.state[tp]["exp_avg_sq"].numpy(), rtol=1e-5, atol=0)


def test_constant_gradient_limit():
    """With a constant gradient the step tends to -lr * g / (|g| + eps)."""
    g = np.array([2e-3, -5e-4], np.float32)
    p = np.array([1.0, 1.0], np.float32)
    m = np.zeros(2, np.float32)
    v = np.zeros(2, np.float32)
    for t in range(1, 6):
        p_new, m, v = oracle.adam_f32(p, g, m, v, t, LR, B1, B2, EPS)
        step = p_new.astype(np.float64) - p.astype(np.float64)
        expect = -f32(LR) * g.astype(np.float64) / (np.abs(g.astype(np.float64)) + f32(EPS))
        assert np.allclose(step, expect, rtol=2e-3)         # ulp(1.0) / lr ~ 1e-3
        p = p_new


def test_checkpoint_resume():
    """State is caller-owned: two steps == one step, copy the state, one step."""
    rng = np.random.default_rng(12)
    n = 100
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g1 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g2 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    z = np.zeros(n, np.float32)
    p1, m1, v1 = oracle.adam_f32(p0, g1, z, z, 1, LR, B1, B2, EPS)
    p2, m2, v2 = oracle.adam_f32(p1, g2, m1, v1, 2, LR, B1, B2, EPS)
    saved = [a.copy() for a in (p1, m1, v1)]
    q2, n2, w2 = oracle.adam_f32(*[saved[0]], g2, saved[1], saved[2], 2, LR, B1, B2, EPS)
    for a, b in ((p2, q2), (m2, n2), (v2, w2)):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


# ---- the tolerance the parity tests use, checked between the oracle's two evaluations ----------
# (t, bit patterns of p, g, m, v): inputs, found by a CPU sweep over p ~ N(0, 0.02), g, m ~ N(0, 1e-3),
# v ~ U(0, 1e-6), for which the binary32 and the binary64 evaluation of the same update differ by more
# than 1e-6 * max(|p_new|, |p_old|): |p| is tiny and the two terms of the new m nearly cancel.
_WITNESSES = [
    (2, 0xB298DB91, 0x3AC1C4E4, 0xB92D34EF, 0x353A0473),
    (2, 0xB35498CF, 0x3AB0688E, 0xB91B23CB, 0x3422755C),
    (9, 0xB3E2742E, 0xBA8383A8, 0x38E6178F, 0x334241A0),
    (300, 0x3382BC3B, 0x3A81C64B, 0xB8DEE612, 0x350BADD7),
    (300, 0x34D5DD87, 0xBB1DF0C9, 0x399661A1, 0x35014421),
]


def test_tolerance_needs_the_update_scale_between_binary32_and_binary64():
    from adam_parity import adam_close, adam_scales
    hp = (1e-4, 0.9, 0.999, 1e-8)
    for t, *bits in _WITNESSES:
        p, g, m, v = (np.array([b], dtype=np.uint32).view(np.float32) for b in bits)
        assert abs(float(p[0])) < 2e-6 and float(m[0]) * float(g[0]) < 0          # tiny p, cancelling m
        rp, rm, rv = oracle.adam_f32(p, g, m, v, t, *hp)
        dp, dm, dv = oracle.adam_f64(p, g, m, v, t, *hp)
        ok, bad = adam_close(rp, rm, rv, dp, dm, dv, p, m, g)
        assert not ok and bad[0] == 1 and bad[1:] == (0, 0), (t, bad)             # p alone is beyond the naive bound
        rel = abs(float(rp[0]) - float(dp[0])) / max(abs(float(dp[0])), abs(float(p[0])))
        assert 1e-6 < rel < 5e-6
        _, U = adam_scales(p, g, m, dv, t, *hp)
        ok, bad = adam_close(rp, rm, rv, dp, dm, dv, p, m, g, update_scale=U)
        assert ok, (t, bad)


@pytest.mark.parametrize("t", [1, 2, 9, 300])
def test_binary32_oracle_within_tolerance_of_binary64(t):
    """4 M elements of the GPU sweep's distribution, plus rows with p = 0 and
    |p| <= lr, where the bound is a bound on the update itself."""
    from adam_parity import adam_close, adam_scales
    hp = (1e-4, 0.9, 0.999, 1e-8)
    rng = np.random.default_rng(100 + t)
    n = 1 << 22
    p = rng.normal(0, 0.02, n).astype(np.float32)
    p[: n // 8] = 0.0
    p[n // 8: n // 4] = rng.uniform(-1e-4, 1e-4, n // 4 - n // 8).astype(np.float32)
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    m = rng.normal(0, 1e-3, n).astype(np.float32) if t > 1 else np.zeros(n, np.float32)
    v = rng.uniform(0, 1e-6, n).astype(np.float32) if t > 1 else np.zeros(n, np.float32)
    rp, rm, rv = oracle.adam_f32(p, g, m, v, t, *hp)
    dp, dm, dv = oracle.adam_f64(p, g, m, v, t, *hp)
    _, U = adam_scales(p, g, m, dv, t, *hp)
    ok, bad = adam_close(rp, rm, rv, dp, dm, dv, p, m, g, update_scale=U)
    assert ok, bad
    # on the p = 0 rows the bound is relative to the update: |dp32 - dp64| <= 2e-6 * s * M / d
    z = slice(0, n // 8)
    assert (np.abs(rp[z].astype(np.float64) - dp[z]) <= 1e-6 * np.maximum(U[z], np.abs(dp[z]))).all()


def test_tolerance_with_update_scale_rejects_the_other_adam_readings():
    """At p = 0 the bound discriminates the reading taken (eps outside the root,
    bias corrections applied): each other reading moves the update by far more."""
    from adam_parity import adam_close, adam_scales
    lr, b1, b2, eps = 1e-4, 0.9, 0.999, 1e-8
    rng = np.random.default_rng(9)
    n = 4096
    p = np.zeros(n, np.float32)
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    m = rng.normal(0, 1e-3, n).astype(np.float32)
    v = rng.uniform(0, 1e-6, n).astype(np.float32)
    t = 3
    dp, dm, dv = oracle.adam_f64(p, g, m, v, t, lr, b1, b2, eps)
    _, U = adam_scales(p, g, m, dv, t, lr, b1, b2, eps)
    bc1, bc2 = 1 - float(np.float32(b1)) ** t, 1 - float(np.float32(b2)) ** t
    inside = -(lr / bc1) * dm / (np.sqrt(dv / bc2 + eps))                 # eps inside the root
    no_bc2 = -(lr / bc1) * dm / (np.sqrt(dv) + eps)                       # second bias correction dropped
    eps_scaled = -(lr / bc1) * dm / ((np.sqrt(dv) + eps) / np.sqrt(bc2))  # eps added before the correction
    for other in (inside, no_bc2, eps_scaled):
        ok, bad = adam_close(other, dm, dv, dp, dm, dv, p, m, g, update_scale=U)
        assert not ok and bad[0] > n // 2
