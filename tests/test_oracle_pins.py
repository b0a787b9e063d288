"""The CPU oracle against its pins (closed forms, library attention, brute force, identities)."""
import pytest

import pins


@pytest.mark.parametrize("check", pins.ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(oracle, check):
    check(None)


def test_golden_regression_c1(oracle):
    """The stored oracle output for the smallest workload (written by tests/golden/make_golden.py,
    which calls only the generator and the oracle) still comes out of both unchanged."""
    import os
    import numpy as np
    import workloads as W
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c1_decode_oracle.txt")
    lines = [l for l in open(path) if not l.startswith("#")]
    want = np.array([[float(x) for x in l.split()] for l in lines])
    case = W.make_case(W.CONFIGS["C1"])
    kc, vc = pins.filled(case)
    got = pins.run_decode(case, kc, vc)
    np.testing.assert_allclose(got[0, :, :8], want, rtol=0, atol=1e-15)
