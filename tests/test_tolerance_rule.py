"""The comparison rule the GPU parity tests apply (harness.check_scaled), checked on the CPU with
made-up outputs: what it must accept and what it must refuse."""
import numpy as np
import pytest

import workloads as W


@pytest.fixture(scope="module")
def H():
    import harness
    return harness


def _case(dtype, ref_vals, errs):
    ref = np.asarray(ref_vals, dtype=np.float64)
    got = W.to_bits((ref + np.asarray(errs)).astype(np.float32), dtype)
    return got, ref


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_plain_bar_below_magnitude_four(H, dtype):
    tol = H.TOL[dtype]
    ref = np.zeros(1000)
    ref[:10] = [0.0, 0.5, -0.5, 1.0, -1.75, 2.0, 3.0, -3.5, 3.9, 0.25]
    got = W.to_bits(ref.astype(np.float32), dtype)                # exactly representable values: zero error
    H.check_scaled(got, ref, dtype, "exact")
    bad = got.copy()
    bad[1] = W.to_bits(np.array([0.5 + 2.0 * tol], np.float32), dtype)[0]
    with pytest.raises(AssertionError):
        H.check_scaled(bad, ref, dtype, "one element off by twice the bar")
    ok = got.copy()
    ok[1] = W.to_bits(np.array([0.5 + 0.5 * tol], np.float32), dtype)[0]
    H.check_scaled(ok, ref, dtype, "half the bar")


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_large_outputs_get_the_format_rounding_and_nothing_more(H, dtype):
    tol, mant = H.TOL[dtype], H.MANTISSA_BITS[dtype]
    budget = tol - 2.0 ** (-mant)                                 # the bar minus half an ulp in [2, 4)
    ref = np.zeros(100000)
    ref[0] = 5.0 + 2.0 ** (1 - mant)                              # in [4, 8): ulp 2^(2 - mant), this is a midpoint
    half = 2.0 ** (1 - mant)
    got = W.to_bits(ref.astype(np.float32), dtype)
    got[0] = W.to_bits(np.array([5.0], np.float32), dtype)[0]     # the neighbouring value: half an ulp away
    assert abs(W.from_bits(got[:1], dtype)[0] - ref[0]) == pytest.approx(half)
    H.check_scaled(got, ref, dtype, "rounded the other way at a midpoint")
    got[0] = W.to_bits(np.array([5.0 - 2.0 * half], np.float32), dtype)[0]        # one more ulp off
    assert abs(W.from_bits(got[:1], dtype)[0] - ref[0]) > half + budget
    with pytest.raises(AssertionError):
        H.check_scaled(got, ref, dtype, "an ulp and a half off")


def test_large_outputs_must_be_rare_and_outputs_finite(H):
    dtype = W.BF16
    ref = np.zeros(100000)
    ref[:65] = 4.5
    got = W.to_bits(ref.astype(np.float32), dtype)
    with pytest.raises(AssertionError):
        H.check_scaled(got, ref, dtype, "65 large outputs of 100000 at 1e-4", max_exempt=1e-4)
    H.check_scaled(got, ref, dtype, "65 large outputs of 100000 at 1e-3", max_exempt=1e-3)
    ref[65:] = 0.0
    ref[:64] = 4.5
    ref[64] = 0.0
    H.check_scaled(W.to_bits(ref.astype(np.float32), dtype), ref, dtype, "64 are always allowed", max_exempt=1e-6)
    nan = W.to_bits(ref.astype(np.float32), dtype)
    nan[7] = 0x7FC0
    with pytest.raises(AssertionError):
        H.check_scaled(nan, ref, dtype, "a NaN in the output")
    H.check_scaled(np.zeros((0, 4), np.uint16), np.zeros((0, 4)), dtype, "empty")
