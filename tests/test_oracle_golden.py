"""The oracle must keep reproducing its committed worked example (tests/golden/oracle_trace.txt,
written by tests/golden/make_golden.py from the oracle alone).  This is a drift detector, not a
pin: the pins are in the other test_oracle_*.py files.  A deliberate change of the oracle's
arithmetic re-writes the fixture in the same commit and says why."""
import importlib.util
import os

import numpy as np

import oracle

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


def _paper_values():
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")):
        if line.strip() and not line.startswith("#"):
            k, v, _ = [s.strip() for s in line.split("|", 2)]
            vals[k] = float(v)
    return vals


def test_oracle_format_matches_the_numbers_the_paper_prints():
    pv = _paper_values()
    qs, qu = oracle.build_codebook(True), oracle.build_codebook(False)
    # smallest magnitudes sit in the decade 10^-7 .. 10^-6 (one decimal exponent per leading zero bit)
    lo = 10.0 ** pv["smallest_decimal_exponent"]
    assert lo <= qs[qs > 0].min() < 10 * lo and lo <= qu[qu > 0].min() < 10 * lo
    # the top decade of the signed map has denominator+1 equally spaced values: 63 steps
    top = qs[(qs >= 0.1) & (qs < 1.0)]
    assert top.size == pv["finest_fraction_denominator"] + 1
    assert np.allclose(np.diff(top.astype(np.float64)), 0.9 / (pv["finest_fraction_denominator"] + 1), rtol=1e-5)
    # memory: one byte per state entry plus one float per block
    B = int(pv["block_size"])
    n = 10 * B
    for states, fp32_bytes in ((1, pv["bytes_per_weight_fp32_states_sgd"]), (2, pv["bytes_per_weight_fp32_states_adam"])):
        q8_bytes = states * (n + 4 * oracle.nblocks(n, B))
        saving = 100.0 * (1 - q8_bytes / (fp32_bytes * n))
        assert abs(saving - (pv["state_memory_saving_percent"] - 100.0 / B)) < 1e-9
        assert round(saving) == pv["state_memory_saving_percent"]
