"""The Adam parity check shared by the CPU and GPU tests.

The bar the task states is "Adam within 1e-6 relative".  Read for one element
with old state (p, m, v), gradient g and step t (Sec. 5.4 only names Adam, so
the reading is this build's):

  m, v:  |a - b| <= rel * max(|a|, |b|, M)        M = max(|b1 m|, |(1 - b1) g|)
  p:     |a - b| <= rel * max(|a|, |b|, |p|, U)   U = 2 s M / d,  s = lr / (1 - b1^t),
                                                  d = sqrt(v') / sqrt(1 - b2^t) + eps

M enters because the two terms of the new m may cancel, and U (twice the
largest update the terms of m can produce) because the update inherits that
cancellation and because p - update can cancel as well.  Where the derivation
comes from: a binary32 evaluation makes three roundings for m' (absolute error
<= 3u M, u = 2^-24), at most five relative ones for d and three more for the
quotient, the product and the difference, so its distance from the exact
result is below (3u + 2 * 8u) s M / d + u |p'| < 1.2e-6 * max(|p'|, s M / d)
in the worst case and a third of that typically.  With U = 0 (the bound this
build used at first) two correctly rounded evaluations can differ by more than
1e-6 of max(|p'|, |p|) when |p| is tiny and m cancels; test_oracle_adam.py
keeps such inputs as a witness.

The kernels are written to mirror the binary32 oracle operation for operation
(no contraction, IEEE divide and square root), so against that oracle the GPU
tests assert bit identity; the tolerance above is what they assert against the
binary64 evaluation.
"""
from __future__ import annotations

import numpy as np

import oracle


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def adam_scales(p_old, g, m_old, v_new, t, lr, beta1, beta2, eps):
    """(M, U) of the module docstring, in binary64."""
    M = np.maximum(np.abs(_f64(m_old)) * float(np.float32(beta1)), np.abs(_f64(g)) * (1.0 - float(np.float32(beta1))))
    s = float(np.float32(lr)) / (1.0 - float(np.float32(beta1)) ** t)
    d = np.sqrt(_f64(v_new)) / np.sqrt(1.0 - float(np.float32(beta2)) ** t) + float(np.float32(eps))
    with np.errstate(divide="ignore", invalid="ignore"):
        U = np.where(M > 0, 2.0 * s * M / d, 0.0)
    return M, U


def adam_close(got_p, got_m, got_v, ref_p, ref_m, ref_v, p_old, m_old=None, g=None, beta1=0.9, rel=1e-6,
               update_scale=None):
    """Tolerance of the Adam parity (see the module docstring); update_scale is
    U, or None for the bound without it.  Returns (ok, (bad_p, bad_m, bad_v))."""
    ref_p, ref_m, ref_v = (_f64(x) for x in (ref_p, ref_m, ref_v))
    gp, gm, gv = (_f64(x) for x in (got_p, got_m, got_v))
    m_scale = np.maximum(np.abs(ref_m), np.abs(gm))
    if m_old is not None and g is not None:
        m_scale = np.maximum(m_scale, np.maximum(np.abs(_f64(m_old)) * beta1, np.abs(_f64(g)) * (1 - beta1)))
    ok_m = np.abs(gm - ref_m) <= rel * m_scale
    ok_v = np.abs(gv - ref_v) <= rel * np.maximum(np.abs(ref_v), np.abs(gv))
    p_scale = np.maximum(np.maximum(np.abs(ref_p), np.abs(gp)), np.abs(_f64(p_old)))
    if update_scale is not None:
        p_scale = np.maximum(p_scale, update_scale)
    ok_p = np.abs(gp - ref_p) <= rel * p_scale
    return bool(ok_m.all() and ok_v.all() and ok_p.all()), (int((~ok_p).sum()), int((~ok_m).sum()), int((~ok_v).sum()))


def _bits(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a.view(np.uint32)


def assert_adam_bits(got_p, got_m, got_v, ref_p, ref_m, ref_v, what=""):
    """The HIP path's p, m, v against the binary32 oracle's: bit for bit."""
    for name, a, b in (("p", got_p, ref_p), ("m", got_m, ref_m), ("v", got_v, ref_v)):
        bad = np.flatnonzero(_bits(a) != _bits(b))
        assert bad.size == 0, (f"{what}: {name} is not bit-identical to the binary32 oracle: {bad.size} of {b.size} "
                               f"differ, first at {int(bad[0])}: {hex(int(_bits(a)[bad[0]]))} vs "
                               f"{hex(int(_bits(b)[bad[0]]))}")


def assert_adam_parity(got_p, got_m, got_v, p_old, g, m_old, v_old, t, hyper, what=""):
    """got_* (binary32 arrays from the HIP path) against the oracle from the
    same inputs: bit-identical to the binary32 evaluation, and within 1e-6
    (module docstring) of the binary64 one.  Returns the binary32 reference."""
    lr, beta1, beta2, eps = hyper
    rp, rm, rv = oracle.adam_f32(p_old, g, m_old, v_old, t, lr, beta1, beta2, eps)
    assert_adam_bits(got_p, got_m, got_v, rp, rm, rv, what)
    dp, dm, dv = oracle.adam_f64(p_old, g, m_old, v_old, t, lr, beta1, beta2, eps)
    _, U = adam_scales(p_old, g, m_old, dv, t, lr, beta1, beta2, eps)
    ok, bad = adam_close(got_p, got_m, got_v, dp, dm, dv, p_old, m_old, g, beta1=beta1, update_scale=U)
    assert ok, f"{what}: beyond 1e-6 of the binary64 oracle (p, m, v): {bad}"
    return rp, rm, rv
