"""The oracle against its own stored outputs (tests/golden/): guards against an unintended change
of its arithmetic.  The fixtures are written by tests/golden/make_golden.py from the oracle alone."""
import importlib.util
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
make_golden = importlib.util.module_from_spec(spec)
spec.loader.exec_module(make_golden)


def read_fixture(path):
    out = {}
    with open(path) as f:
        lines = [l for l in f.read().splitlines() if not l.startswith("#")]
    for head, body in zip(lines[0::2], lines[1::2]):
        name, *shape = head.split()
        out[name] = np.array([float.fromhex(t) for t in body.split()]).reshape([int(s) for s in shape])
    return out


@pytest.mark.parametrize("case", make_golden.CASES, ids=[c[0] for c in make_golden.CASES])
def test_oracle_reproduces_its_stored_outputs(case):
    want = read_fixture(make_golden.path(case))
    got = make_golden.compute(case)
    assert set(got) == set(want)
    for name in want:
        assert got[name].shape == want[name].shape
        # same compiler flags (-O2, no fast-math), one thread: differences could only come from libm's exp
        np.testing.assert_allclose(got[name], want[name], rtol=1e-13, atol=1e-15, err_msg=name)
