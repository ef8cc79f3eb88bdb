"""CPU check of the packed-fp16 activation used by the matrix-core expert kernel.

The kernel evaluates GELU(z) = z Phi(z) for z = p * a + b (Eq. 1 scale of the GEMM1 accumulator a,
plus the expert bias) with fp16 multiply-adds and a polynomial for Phi.  This test re-runs exactly
that sequence of roundings in numpy (one rounding per fused multiply-add, round-toward-zero for the
fp32 -> fp16 conversions) with the coefficients of csrc/gelu_poly.h, and compares with the erf
definition of Section 3.1's expert activation.  It pins the coefficient table and the claim that
the activation error is of the size of a bf16 rounding: at most 2^-8 (3.4e-3 observed), rms below 8e-4, of the
larger of |z| and |p a|.
"""
import math
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "paper_2510_04286_amd", "csrc", "gelu_poly.h")


def _consts():
    txt = open(HEADER).read()
    m = int(re.search(r"kGeluM = (\d+)", txt).group(1))
    kappa = float(re.search(r"kGeluKappa = ([0-9.eE+-]+)f", txt).group(1))
    w0 = float(re.search(r"kGeluW0 = ([0-9.eE+-]+)f", txt).group(1))
    q = [float(v.rstrip("f")) for v in re.search(r"kGeluQ\[[^\]]*\] = \{([^}]*)\}", txt).group(1).split(",")]
    assert len(q) == m + 1
    return m, kappa, w0, q


def _rne(x):
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


def _rtz(x):
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(over="ignore"):
        h = x.astype(np.float16)
    over = np.abs(h.astype(np.float64)) > np.abs(x)
    h = np.where(over, np.nextafter(h, np.float16(0)), h)
    h = np.where(np.isinf(h), np.sign(x) * 65504.0, h)
    return h.astype(np.float64)


def _kernel_gelu(acc, p, b):
    """kappa-scaled fp16 pipeline of activation_tile(); returns GELU(z) (the kernel's 1/kappa sits in W2)."""
    m, kappa, w0, q = _consts()
    qh = [float(np.float16(c)) for c in q]
    A = _rtz(np.float32(acc))
    p2 = _rtz(np.float32(p) * np.float32(kappa))
    bias = _rne(np.float32(b) * np.float32(kappa))
    s = _rne(A * p2 + bias)
    v = _rne(s * s - float(np.float16(w0)))
    Q = _rne(v * qh[m] + qh[m - 1])
    for c in range(m - 2, -1, -1):
        Q = _rne(Q * v + qh[c])
    with np.errstate(invalid="ignore"):
        F = np.clip(_rne(s * Q + 0.5), 0.0, 1.0)
    return _rne(s * F) / kappa


def _gelu(z):
    return np.array([0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in np.ravel(z)]).reshape(np.shape(z))


def test_table_shape_makes_the_clamp_saturate():
    m, kappa, w0, q = _consts()
    assert m % 2 == 0 and q[m] > 0, "even degree with positive leading coefficient: s*Q(v) leaves [-1/2, 1/2] for large |z|"
    z = np.linspace(3.3, 240.0, 20000)
    s = kappa * z
    val = s * np.polyval(q[::-1], s * s - w0)
    assert np.all(val >= 0.5 - 1e-3)


def test_fp16_activation_error_is_one_bf16_rounding():
    rng = np.random.default_rng(7)
    for span in (0.5, 1.0, 2.0, 3.0, 4.0, 8.0):
        n = 200000
        z_target = rng.uniform(-span, span, n)
        p = rng.uniform(0.02, 1.0, n)
        b = rng.uniform(-0.125, 0.125, n)
        acc = (z_target - b) / p
        z = np.float64(np.float32(p)) * np.float64(np.float32(acc)) + np.float64(np.float32(b))
        got = _kernel_gelu(acc, p, b)
        err = np.abs(got - _gelu(z))
        # the accumulator is rounded to fp16 before the bias is added, so the bound is relative to the larger of
        # the result and the scaled accumulator (a sum that cancels keeps the rounding of its terms)
        scale = np.maximum(np.maximum(np.abs(z), np.abs(p * acc)), 0.05)
        assert np.max(err / scale) < 2.0 ** -8, (span, float(np.max(err / scale)))
        assert np.sqrt(np.mean((err / scale) ** 2)) < 8e-4


def test_saturation_and_zero():
    z = np.array([-300.0, -40.0, -9.0, 9.0, 40.0, 300.0])
    got = _kernel_gelu(z, np.ones_like(z), np.zeros_like(z))
    ref = np.where(z > 0, z, 0.0)
    assert np.all(np.abs(got - ref) <= 2.0 ** -10 * np.abs(z))
    assert _kernel_gelu(np.zeros(1), np.ones(1), np.zeros(1))[0] == 0.0
    # a lane without a row carries p = 0: the activation of the bias alone, finite
    assert np.isfinite(_kernel_gelu(np.array([1e30]), np.zeros(1), np.array([0.1]))[0])
