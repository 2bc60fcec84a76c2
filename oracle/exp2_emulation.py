"""Software 2^x of paper Sec. 3.1.3 in numpy -- TEST INFRASTRUCTURE ONLY.

The section gives the recipe but not the numbers: range reduction 2^x = 2^floor(x) * 2^frac(x),
a degree-n polynomial for 2^frac with p0 = 1 and the other coefficients chosen to minimise the
relative error on [0, 1) (the authors used Sollya; the coefficients are not printed), Horner
evaluation with FMAs, and the integer part added into the exponent field.

fit_coefficients(n) derives the polynomial from that statement alone: a linear program
    minimise t  subject to  |1 + sum_{i>=1} p_i x^i - 2^x| <= t 2^x   on a Chebyshev grid of [0, 1],
with its rows scaled by 1e4 so that the solver's feasibility tolerance (1e-7 in absolute terms, the
size of the degree-5 error itself) is far below the error being minimised.
exp2_emulated(x, coeffs) then takes the section's five steps in order, in fp32:
  1. clamp x to >= -127;
  2. floor(x)  (the section adds and subtracts 2^23 + 2^22 in round-down mode; np.floor is the
     same function of x);
  3. frac = x - floor(x);
  4. Horner with fused multiply-adds (each FMA = exact product and sum, one rounding to fp32);
  5. the integer part shifted into the exponent field and added to the bits of the polynomial.
The pin is the section's accuracy table (tests/golden/exp2_accuracy_table.txt): a polynomial
derived this way must land on the printed error levels.
"""
from __future__ import annotations

import numpy as np
from scipy.optimize import linprog


ROW_SCALE = 1e4     # the unknown t is the relative error in units of 1 / ROW_SCALE


def fit_coefficients(degree: int, grid: int = 4001):
    """Minimax-relative-error coefficients p_1..p_degree (p_0 = 1) as fp64."""
    x = 0.5 + 0.5 * np.cos(np.pi * (np.arange(grid) + 0.5) / grid)
    f = 2.0 ** x
    A = ROW_SCALE * np.stack([x ** i for i in range(1, degree + 1)], axis=1)
    c = np.zeros(degree + 1)
    c[-1] = 1.0
    A_ub = np.vstack([np.hstack([A, -f[:, None]]), np.hstack([-A, -f[:, None]])])
    b_ub = ROW_SCALE * np.concatenate([f - 1.0, -(f - 1.0)])
    res = linprog(c, A_ub=A_ub, b_ub=b_ub, bounds=[(None, None)] * degree + [(0, None)], method="highs")
    if not res.success:
        raise RuntimeError("minimax fit failed")
    return res.x[:degree]


def _fma32(a, b, c):
    """fp32 fused multiply-add: the product of two fp32 numbers is exact in fp64."""
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)


def exp2_emulated(x, coeffs):
    """2^x for fp32 x by the five steps of Sec. 3.1.3; coeffs = p_1..p_n (rounded to fp32 here)."""
    x = np.maximum(np.asarray(x, dtype=np.float32), np.float32(-127.0))          # step 1
    fl = np.floor(x)                                                            # step 2
    frac = (x - fl).astype(np.float32)                                          # step 3
    p = [np.float32(1.0)] + [np.float32(v) for v in coeffs]
    acc = np.full(x.shape, p[-1], dtype=np.float32)                             # step 4 (Horner)
    for coef in reversed(p[:-1]):
        acc = _fma32(acc, frac, np.full(x.shape, coef, dtype=np.float32))
    bits = acc.view(np.int32) + (fl.astype(np.int32) << 23)                     # step 5
    return bits.view(np.float32)


def to_bf16(x):
    """Round fp32 to bf16 (nearest even), returned as fp32."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32)


def error_table(coeffs, n=1 << 22, seed=0):
    """(fp32 max, fp32 mean, bf16 max, bf16 mean) relative errors on n uniform inputs in [0, 1)."""
    x = np.random.default_rng(seed).random(n, dtype=np.float32)
    ref = np.exp2(x.astype(np.float64))
    y = exp2_emulated(x, coeffs)
    e32 = np.abs(y.astype(np.float64) - ref) / ref
    e16 = np.abs(to_bf16(y).astype(np.float64) - ref) / ref
    return float(e32.max()), float(e32.mean()), float(e16.max()), float(e16.mean())
