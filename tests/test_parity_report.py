"""The mismatch report of the whole-tensor GPU parity tests, exercised on the CPU: distances to
code midpoints are measured correctly, and an entry is located from the state before the step."""
import numpy as np

import oracle
from tests import harness as H

f32 = np.float32


def test_midpoint_distance_in_ulps():
    qs, _ = H.codebooks()
    mids = ((qs[:-1].astype(np.float64) + qs[1:].astype(np.float64)) / 2)
    m = mids[200]
    below = f32(m) if float(f32(m)) < m else np.nextafter(f32(m), f32(-1))
    above = np.nextafter(below, f32(2))
    d = H.midpoint_distance_ulps(qs, np.array([below, above, qs[200], qs[201]], f32))
    assert d[0] <= 1.0 and d[1] <= 1.0 and d[0] + d[1] == 1.0        # the midpoint lies between the two neighbours
    gap_ulps = (float(qs[201]) - float(qs[200])) / 2 / float(np.spacing(qs[200]))
    assert abs(d[2] - gap_ulps) <= 1.0 and d[3] > 1000        # half a local gap (the gaps on both sides agree to an ulp)


def test_entry_is_located_from_the_previous_state():
    """Every entry's code after a step is the nearest code of the normalized value that the
    report re-forms from the state before the step; its midpoint distance is large unless the
    entry was built to sit on a midpoint."""
    qs, qu = H.codebooks()
    n, B = 700, 256
    rng = np.random.default_rng(9)
    w = rng.uniform(-0.1, 0.1, n).astype(f32)
    st = H.zero_state(n, B)
    for t in range(1, 4):
        g = (rng.standard_normal(n) * 1e-3).astype(f32)
        prev = {k: v.copy() for k, v in st.items()}
        H.oracle_adam8(w, g, st, B, t=t)
        for idx in (0, 255, 256, 699):
            for key, q in (("m_q", qs), ("r_q", qu)):
                b = idx // B
                s = slice(b * B, min(n, (b + 1) * B))
                x, y = oracle.adam8bit_block_normalized(np.zeros(s.stop - s.start, f32), g[s], prev["m_q"][s], prev["r_q"][s],
                                                        prev["N_m"][b], prev["N_r"][b], qs, qu, **H.ADAM, t=t)
                v = (x if key == "m_q" else y)[idx - s.start]
                assert oracle.nearest_code(q, v) == st[key][idx]
                u = H.entry_midpoint_distance(prev, g, n, B, idx, key, H.ADAM, t)
                assert u == H.midpoint_distance_ulps(q, np.array([v], f32))[0]


def test_budget_line():
    class C:
        entries, code_mismatches, worst_ulps, worst_param = 2_000_000_000, 0, 0.0, 0.0
    before = len(H.REPORT_LINES)
    H.report_parity("example", [C()])
    assert "0 of 2000000000 code entries differ" in H.REPORT_LINES[-1]
    del H.REPORT_LINES[before:]
    C.code_mismatches = 3000                      # 1.5e-6 of the entries: over the budget
    try:
        H.report_parity("example", [C()])
    except AssertionError:
        pass
    else:
        raise AssertionError("budget not enforced")
    del H.REPORT_LINES[before:]
