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
