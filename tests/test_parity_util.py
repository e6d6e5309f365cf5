"""The checker that the GPU parity tests use must itself reject the mistakes it is there for
(CPU only: the "GPU result" here is the oracle's own product rounded to bf16, with a mistake planted)."""
import numpy as np
import pytest

from oracle import slope_oracle as so
from paper_2405_16325_amd import inputs
from tests.parity_util import check_product


def rounded_product(b=300, d_out=320, d_in=256, seed=5):
    t = inputs.layer_inputs(b, d_out, d_in, 0, seed)
    want = so.spmm_fwd(t["X"], t["W"], so.prune_rows(t["W"]))
    return inputs.f32_to_bf16_bits(want.astype(np.float32)), want


def test_accepts_a_correctly_rounded_result():
    got, want = rounded_product()
    assert check_product(got, want, "Y") < 3e-3


def test_rejects_a_zeroed_fragment_that_the_norm_lets_pass():
    got, want = rounded_product(b=4100, d_out=4160, d_in=64, seed=6)      # the ragged case of the GPU tests
    got = got.copy()
    got[-16:, -64:] = 0                                       # one 16 x 64 corner fragment of 17 M elements
    assert so.rel_fro(so.bf16_to_f64(got), want) <= 1e-2      # the norm alone does not see it
    with pytest.raises(AssertionError, match="element-wise"):
        check_product(got, want, "Y")


def test_rejects_a_swapped_pair_of_elements_and_a_wrong_sign():
    got, want = rounded_product()
    swapped = got.copy()
    swapped[10, 20], swapped[10, 21] = got[10, 21], got[10, 20]
    with pytest.raises(AssertionError):
        check_product(swapped, want, "Y")
    flipped = got.copy()
    flipped[5, 7] ^= 0x8000
    with pytest.raises(AssertionError):
        check_product(flipped, want, "Y")


def test_rejects_non_finite_values_and_shape_mismatch():
    got, want = rounded_product()
    bad = got.copy()
    bad[0, 0] = 0x7FC0
    with pytest.raises(AssertionError, match="non-finite"):
        check_product(bad, want, "Y")
    with pytest.raises(AssertionError):
        check_product(got[:, :-1], want, "Y")
