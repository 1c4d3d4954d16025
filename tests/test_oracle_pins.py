"""The fp64 CPU oracle against closed forms, invariants, library routines and brute force."""
import pytest

import pins


@pytest.mark.parametrize("check", pins.ALL_CHECKS, ids=lambda f: f.__name__)
def test_oracle_pin(check):
    check()


def test_oracle_reproduces_stored_tiny_result():
    """The stored fp64 result on the 'tiny' workload (written by tests/golden/make_golden.py from the
    oracle alone) still comes out: guards the oracle and the input generator against drift."""
    import os

    import numpy as np

    import oracle
    import workloads
    w = workloads.CONFIGS["tiny"]
    ks, vs = w.make_kv()
    out, lse = oracle.attn(w.make_q(), ks, vs, w.kv_lens(), w.scale)
    n = 0
    with open(os.path.join(os.path.dirname(__file__), "golden", "tiny_oracle.txt")) as f:
        for line in f:
            p = line.split()
            if p[0] == "lse":
                assert abs(lse[int(p[1]), int(p[2]), int(p[3])] - float(p[4])) < 1e-13
                n += 1
            elif p[0] == "out":
                assert abs(out[int(p[1]), int(p[2]), int(p[3]), int(p[4])] - float(p[5])) < 1e-13
                n += 1
    assert n == 32 + 32 * 8
