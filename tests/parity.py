"""Comparison rules between the HIP path and the CPU oracle (used by the GPU tests, the
smoke check and the benchmark's self-check).

Integers (hash indices, probes, baked D_c) must match bit for bit.

Floating point.  The bar is a maximum relative error of 1e-5 for fp32 results and 2e-3 where
fp16 is involved in the result.  "Relative" is meant in the backward-error sense: an
interpolated value or an accumulated gradient is a sum of signed terms, and any
implementation that adds them in fp32 in some order is off by a multiple of
eps * (sum of the terms' magnitudes), which can exceed the value itself when the terms
cancel.  The oracle therefore returns that magnitude sum next to every result (ymag for
the encoding, A_f / A_c for the gradients) and the test is

    |gpu - ref| <= tol * max(|ref|, magnitude) + floor

with floor = 2^-25 for fp16 outputs (half a unit of the fp16 subnormal grid: features of
size 1e-4 live on that grid, where precision is absolute, not relative) and a denormal-sized
floor otherwise.
"""
import numpy as np

TOL_F32 = 1e-5
TOL_F16 = 2e-3
F16_SUBNORMAL_HALF_ULP = 2.0 ** -25


def check_exact(name, got, want):
    got = np.asarray(got); want = np.asarray(want)
    assert got.shape == want.shape, f"{name}: shape {got.shape} vs {want.shape}"
    bad = np.flatnonzero(got.ravel().astype(np.int64) != want.ravel().astype(np.int64))
    assert bad.size == 0, (f"{name}: {bad.size} of {got.size} integers differ; first at flat index "
                           f"{bad[0]}: got {got.ravel()[bad[0]]}, want {want.ravel()[bad[0]]}")


def rel_err(got, ref, mag, floor):
    got = np.asarray(got, dtype=np.float64)
    scale = np.maximum(np.abs(ref), mag)
    return (np.abs(got - ref) - floor).clip(min=0.0) / np.maximum(scale, 1e-300)


PLAIN = {}      # name -> plain max|gpu - ref| / max|ref| of the last comparison under that name (reported, not a bar)


def plain_rel_err(got, ref):
    """max|gpu - ref| / max|ref| over a whole tensor: the figure a reader expects next to the term-normalised one."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    top = float(np.abs(ref).max(initial=0.0))
    return float(np.abs(got - ref).max(initial=0.0)) / top if top > 0.0 else 0.0


def check_close(name, got, ref, mag, fp16_out):
    tol = TOL_F16 if fp16_out else TOL_F32
    floor = F16_SUBNORMAL_HALF_ULP if fp16_out else 1e-37
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    err = rel_err(got, ref, mag, floor)
    worst = int(np.argmax(err))
    assert err.ravel()[worst] <= tol, (
        f"{name}: max rel err {err.ravel()[worst]:.3e} > {tol:g} at flat index {worst}: "
        f"got {got.ravel()[worst]!r}, ref {ref.ravel()[worst]!r}, magnitude {np.asarray(mag).ravel()[worst]!r}")
    PLAIN[name] = plain_rel_err(got, ref)
    return float(err.max(initial=0.0))
