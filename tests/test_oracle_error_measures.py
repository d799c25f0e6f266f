"""Pins of the two error measures the parity checks use (tolerances of the benchmark spec: relative Frobenius error and largest
elementwise error over the largest reference magnitude).  The expected values are worked out by hand from bf16 bit
patterns whose values are small integers, so every norm below is an exact rational or a square root of one."""
import math

import numpy as np

from oracle import ops

# bf16 bit patterns of small values: 0x3f80 = 1, 0x4000 = 2, 0x4040 = 3, 0x4080 = 4, 0xc000 = -2, 0x0000 = 0
ONE, TWO, THREE, FOUR, MINUS_TWO, ZERO = 0x3F80, 0x4000, 0x4040, 0x4080, 0xC000, 0x0000


def bits(*v):
    return np.array(v, dtype=np.uint16)


def test_identical_inputs_have_zero_error():
    r = bits(ONE, MINUS_TWO, THREE, FOUR)
    assert ops.rel_frobenius(r, r) == 0.0
    assert ops.max_abs_over_max_ref(r, r) == 0.0


def test_hand_example():
    # ref = (3, 4, 0, -2): |ref|_F = sqrt(29), max |ref| = 4.  got = (1, 4, 2, -2): differences (-2, 0, 2, 0).
    ref, got = bits(THREE, FOUR, ZERO, MINUS_TWO), bits(ONE, FOUR, TWO, MINUS_TWO)
    assert ops.rel_frobenius(got, ref) == math.sqrt(8.0) / math.sqrt(29.0)
    assert ops.max_abs_over_max_ref(got, ref) == 2.0 / 4.0


def test_not_symmetric_the_reference_normalises():
    # swapping the roles changes the denominator: |got|_F = sqrt(25) = 5, max |got| = 4
    ref, got = bits(THREE, FOUR, ZERO, MINUS_TWO), bits(ONE, FOUR, TWO, MINUS_TWO)
    assert ops.rel_frobenius(ref, got) == math.sqrt(8.0) / 5.0
    assert ops.max_abs_over_max_ref(ref, got) == 2.0 / 4.0
    ref2, got2 = bits(ONE, ONE), bits(THREE, ONE)
    assert ops.max_abs_over_max_ref(got2, ref2) == 2.0      # over max |ref| = 1 ...
    assert ops.max_abs_over_max_ref(ref2, got2) == 2.0 / 3  # ... and over max |ref| = 3


def test_sign_and_shape():
    # a sign flip of one element of value 2 is an error of 4; matrices are flattened by the Frobenius norm
    ref = np.array([[TWO, TWO], [TWO, TWO]], dtype=np.uint16)
    got = np.array([[TWO, MINUS_TWO], [TWO, TWO]], dtype=np.uint16)
    assert ops.rel_frobenius(got, ref) == 4.0 / 4.0
    assert ops.max_abs_over_max_ref(got, ref) == 4.0 / 2.0


def test_one_bf16_ulp_is_inside_the_tolerances_and_one_percent_is_not():
    # 1 + 2^-7 is the bf16 neighbour of 1: a relative error of 2^-7 = 7.8e-3 in ONE element of 64 stays below the
    # 5e-3 Frobenius bound (2^-7 / 8) and below 1e-2 of the maximum; the same error in every element does not
    ref = np.full(64, ONE, dtype=np.uint16)
    got = ref.copy()
    got[5] = ONE + 1
    assert ops.rel_frobenius(got, ref) == 2.0 ** -7 / 8.0
    assert ops.max_abs_over_max_ref(got, ref) == 2.0 ** -7
    assert ops.rel_frobenius(np.full(64, ONE + 1, dtype=np.uint16), ref) == 2.0 ** -7 > 5e-3
