"""The bar every floating-point product of the HIP path has to meet against the fp64 oracle.

Two checks, both asserted:

  * the norm: ||gpu - oracle||_F / ||oracle||_F <= 1e-2 (the stated tolerance for bf16 operands with
    fp32 accumulation);
  * every element: |gpu - oracle| <= 2^-7 |oracle| + a * rms(oracle).  One rounding of an fp32 sum to
    bf16 (8 significant bits) is off by at most 2^-8 |value|; the fp32 accumulation over K terms adds
    about sqrt(K) 2^-24 of the terms' norm, far below 2^-9 rms for every K here, and it is what is left
    where the terms cancel (|oracle| ~ 0).  So a = 2^-9 for a single product.  Where an intermediate
    product is rounded to bf16 before a second product (X L, dY R^T), each of its entries carries a
    relative error of up to 2^-8 that does not cancel with the result: a = 2^-6 then (six standard
    deviations of a sum of such errors whose terms are as large as the result's own).
    The norm alone would let a wrong 16 x 64 fragment of a large ragged case pass; this does not:
    an element that is zero, stale or belongs elsewhere misses the bound unless the true value is
    itself within ~2^-6 rms of it.
"""
import numpy as np

from oracle import slope_oracle as so

TOL = 1e-2
REL = 2.0 ** -7
ABS_ONE_ROUNDING = 2.0 ** -9
ABS_TWO_STAGE = 2.0 ** -6


def check_product(got_bits, want, what, two_stage=False, tol=TOL):
    """got_bits: uint16 bf16 bit patterns from the GPU; want: fp64 oracle result of the same shape.
    Returns the relative Frobenius error; raises AssertionError naming the worst element."""
    got = so.bf16_to_f64(np.asarray(got_bits))
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    err = so.rel_fro(got, want)
    assert err <= tol, f"{what}: relative Frobenius error {err:.3e} > {tol}"
    rms = float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    bound = REL * np.abs(want) + (ABS_TWO_STAGE if two_stage else ABS_ONE_ROUNDING) * rms
    excess = np.abs(got - want) - bound
    if excess.size and excess.max() > 0:
        idx = np.unravel_index(int(np.argmax(excess)), excess.shape)
        bad = int((excess > 0).sum())
        raise AssertionError(f"{what}: {bad} of {excess.size} elements outside the element-wise bound; worst at "
                             f"{tuple(int(i) for i in idx)}: gpu {got[idx]:.6g} oracle {want[idx]:.6g} "
                             f"bound {bound[idx]:.3g}")
    return err
