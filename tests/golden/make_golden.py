#!/usr/bin/env python3
"""Writes tests/golden/oracle_trace.txt: a small worked example of the 8-bit steps computed
by the CPU oracle alone (nothing here touches the HIP library).  The file is a drift
detector for the oracle's arithmetic: codebook anchors (closed forms of the bin-centre
reading of the dynamic-tree type, Sec. IV-B), then three 8-bit Adam steps (Eq. adam +
Eq. quant1-quant3) and three 8-bit SGD steps (Eq. sgd) on a fixed 40-element tensor, B = 16
so that several blocks and a short last block appear.  Values are printed as exact
hexadecimal floats and code lists.

    python tests/golden/make_golden.py          (re-writes the fixture)
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402


def fixed_inputs():
    i = np.arange(40, dtype=np.float64)
    w = (0.1 * np.sin(1.0 + 0.7 * i)).astype(np.float32)
    grads = [(1e-3 * np.cos(0.3 * i * (t + 1)) * (1.0 + 50.0 * (i == 7 * t + 3))).astype(np.float32) for t in range(3)]
    return w, grads


def trace_lines():
    qs, qu = oracle.build_codebook(True), oracle.build_codebook(False)
    out = ["# codebook anchors: index value (hex float)"]
    for name, q, idx in (("signed", qs, (0, 1, 126, 127, 128, 129, 191, 192, 254, 255)),
                         ("unsigned", qu, (0, 1, 2, 3, 127, 128, 254, 255))):
        for j in idx:
            out.append("%s %d %s" % (name, j, float(q[j]).hex()))
    B, n = 16, 40
    nb = oracle.nblocks(n, B)
    for opt in ("adam", "sgd"):
        w, grads = fixed_inputs()
        mq = np.full(n, 127, np.uint8); rq = np.zeros(n, np.uint8)
        Nm = np.zeros(nb, np.float32); Nr = np.zeros(nb, np.float32)
        for t, g in enumerate(grads, 1):
            if opt == "adam":
                oracle.adam8bit_step(w, g, mq, rq, Nm, Nr, qs, qu, B, 1e-3, 0.9, 0.999, 1e-8, 0.0, t, 0)
            else:
                oracle.sgd8bit_step(w, g, mq, Nm, qs, B, 0.1, 0.9, 1e-4)
            out.append("# %s step %d" % (opt, t))
            out.append("m_q " + " ".join(str(int(c)) for c in mq))
            out.append("N_m " + " ".join(float(x).hex() for x in Nm))
            if opt == "adam":
                out.append("r_q " + " ".join(str(int(c)) for c in rq))
                out.append("N_r " + " ".join(float(x).hex() for x in Nr))
            out.append("w " + " ".join(float(x).hex() for x in w))
    return out


if __name__ == "__main__":
    with open(os.path.join(HERE, "oracle_trace.txt"), "w") as f:
        f.write("\n".join(trace_lines()) + "\n")
    print("wrote", os.path.join(HERE, "oracle_trace.txt"))
