"""The oracle still returns what tests/golden/oracle_digest.txt recorded.

The file is written by tests/golden/make_oracle_digest.py from oracle/ alone (the paper prints no
numeric example to store).  It pins nothing about correctness - the other test_oracle_* files do
that - it only makes a change of the oracle's arithmetic visible: integers and hashes must match
exactly, floating-point sums to 1e-8 relative (summation order inside the BLAS may differ)."""
import os
import re
import runpy

HERE = os.path.dirname(os.path.abspath(__file__))
NUM = re.compile(r"^[-+]?\d+\.\d+e[-+]\d+$")


def test_oracle_digest_is_unchanged():
    mod = runpy.run_path(os.path.join(HERE, "golden", "make_oracle_digest.py"), run_name="digest")
    now = mod["digest_lines"]()
    with open(os.path.join(HERE, "golden", "oracle_digest.txt")) as f:
        stored = f.read().splitlines()
    assert len(now) == len(stored)
    for a, b in zip(now, stored):
        ta, tb = a.split(), b.split()
        assert len(ta) == len(tb), (a, b)
        for x, y in zip(ta, tb):
            if NUM.match(y):
                assert abs(float(x) - float(y)) <= 1e-8 * max(1.0, abs(float(y))), (a, b)
            else:
                assert x == y, (a, b)
