"""Comparison helpers for the GPU parity tests: the tolerance of the benchmark spec
(bf16 outputs and gradients within max-abs 2e-2 and relative Frobenius 1e-2 of the fp64
oracle on N(0,1) inputs), written once."""
import numpy as np

MAX_ABS = 2e-2
REL_FRO = 1e-2
# LSE is fp32 and of size O(ln N + |S|): a pure fp32 quantity, held to a much tighter bound.
LSE_ABS = 2e-3


def errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in GPU result"
    diff = got - ref
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))


def assert_close(got, ref, what, max_abs=MAX_ABS, rel_fro=REL_FRO):
    ma, rf = errors(got, ref)
    assert ma <= max_abs and rf <= rel_fro, f"{what}: max-abs {ma:.3e} (<= {max_abs}), rel-Fro {rf:.3e} (<= {rel_fro})"
    return ma, rf


def assert_close_outlier(got, ref, what):
    """Heavy-tailed inputs (the x8 outlier workload): gradients can exceed 8 in magnitude, where
    one bf16 half-ulp alone is 2e-2.  Gate elementwise on 2e-2 + 2^-8 |ref| and on the same
    relative Frobenius bound."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.isfinite(got).all(), "non-finite values in GPU result"
    excess = np.abs(got - ref) - (MAX_ABS + 2.0 ** -8 * np.abs(ref))
    ma, rf = errors(got, ref)
    assert excess.max() <= 0 and rf <= REL_FRO, f"{what}: worst excess {excess.max():.3e}, max-abs {ma:.3e}, rel-Fro {rf:.3e}"
    return ma, rf
