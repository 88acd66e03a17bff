"""The oracle must keep reproducing its committed worked example (tests/golden/oracle_trace.txt,
written by tests/golden/make_golden.py from the oracle alone).  This is a drift detector, not a
pin: the pins are in the other test_oracle_*.py files.  A deliberate change of the oracle's
arithmetic re-writes the fixture in the same commit and says why."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_committed_trace():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = open(os.path.join(HERE, "golden", "oracle_trace.txt")).read().splitlines()
    assert mod.trace_lines() == want


def test_trace_anchor_values_are_the_closed_forms():
    """Anchor lines of the fixture against the closed forms of the dynamic-tree reading
    (Sec. IV-B): bin centres of [0.1, 1] divided by 10^E."""
    import numpy as np
    lines = [l.split() for l in open(os.path.join(HERE, "golden", "oracle_trace.txt")) if l[0] in "su"]
    got = {(a, int(b)): float.fromhex(c) for a, b, c in lines}
    f32 = lambda x: float(np.float32(x))
    assert got[("signed", 127)] == 0.0 and got[("signed", 255)] == 1.0 and got[("unsigned", 0)] == 0.0
    assert got[("signed", 254)] == f32(1 - 0.9 / 128) and got[("signed", 0)] == -f32(1 - 0.9 / 128)
    assert got[("signed", 128)] == f32(0.55e-6) and got[("signed", 129)] == f32(0.325e-5)
    assert got[("signed", 191)] == f32(0.1 + 0.9 / 128) and got[("signed", 192)] == f32(0.1 + 0.9 * 3 / 128)
    assert got[("unsigned", 1)] == f32(0.325e-6) and got[("unsigned", 254)] == f32(1 - 0.9 / 256)
