"""Shared plumbing of the GPU parity tests: run the same seeded inputs through the CPU
oracle (numpy arrays) and through the C-ABI library (torch device tensors) and compare.
Holds no arithmetic of the method."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

import oracle

ADAM = dict(alpha=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
SGD = dict(alpha=0.1, beta=0.9)
PARAM_RTOL = 1e-6          # bar stated for parameters: relative error after every step

_QS = _QU = None


def codebooks():
    global _QS, _QU
    if _QS is None:
        _QS, _QU = oracle.build_codebook(True), oracle.build_codebook(False)
    return _QS, _QU


def host_threads() -> int:
    try:
        return max(1, min(16, len(os.sched_getaffinity(0))))
    except AttributeError:
        return 1


_pool = None


def pool():
    global _pool
    if _pool is None:
        _pool = ThreadPoolExecutor(host_threads())
    return _pool


def zero_state(n, B, adam=True):
    nb = oracle.nblocks(n, B)
    st = dict(m_q=np.full(n, 127, np.uint8), N_m=np.zeros(nb, np.float32))
    if adam:
        st.update(r_q=np.zeros(n, np.uint8), N_r=np.zeros(nb, np.float32))
    return st


def oracle_adam8(w, g, st, B, wd=0.0, t=1, flags=0, hp=ADAM, split=True, bf16=False, f16=False):
    """In place; splits the tensor at block boundaries over host threads (blocks are independent).
    bf16 / f16: w and g are uint16 arrays of bfloat16 / binary16 patterns."""
    step = oracle.adam8bit_step_bf16 if bf16 else (oracle.adam8bit_step_f16 if f16 else oracle.adam8bit_step)
    qs, qu = codebooks()
    n = w.size
    nb = oracle.nblocks(n, B)
    nthr = host_threads() if (split and n >= (1 << 18)) else 1
    per = -(-nb // nthr)

    def run(k):
        b0, b1 = k * per, min(nb, (k + 1) * per)
        if b0 >= b1:
            return
        s = slice(b0 * B, min(n, b1 * B))
        step(w[s], g[s], st["m_q"][s], st["r_q"][s], st["N_m"][b0:b1], st["N_r"][b0:b1],
             qs, qu, B, hp["alpha"], hp["beta1"], hp["beta2"], hp["eps"], wd, t, flags)
    if nthr == 1:
        run(0)                                   # also when called from a worker of pool()
    else:
        list(pool().map(run, range(nthr)))


def oracle_sgd8(w, g, st, B, wd=0.0, hp=SGD, bf16=False, f16=False):
    qs, _ = codebooks()
    step = oracle.sgd8bit_step_bf16 if bf16 else (oracle.sgd8bit_step_f16 if f16 else oracle.sgd8bit_step)
    step(w, g, st["m_q"], st["N_m"], qs, B, hp["alpha"], hp["beta"], wd)


def rel_err(w_gpu: np.ndarray, w_ref: np.ndarray) -> float:
    if w_ref.size == 0:
        return 0.0
    d = np.abs(w_gpu.astype(np.float64) - w_ref.astype(np.float64))
    return float((d / np.maximum(np.abs(w_ref.astype(np.float64)), 1e-30)).max())


def assert_state_equal(tag, dev: dict, ref: dict, w_dev, w_ref):
    """codes and absmax bit-exact, parameters within PARAM_RTOL."""
    for k in ref:
        a = dev[k].cpu().numpy()
        b = ref[k]
        if a.dtype == np.float32:
            a, b = a.view(np.uint32), b.view(np.uint32)
        if not np.array_equal(a, b):
            bad = np.flatnonzero(a != b)
            raise AssertionError("%s: %s differs at %d of %d entries, first index %d: gpu %r oracle %r"
                                 % (tag, k, bad.size, a.size, bad[0], a[bad[0]], b[bad[0]]))
    e = rel_err(w_dev.cpu().numpy(), w_ref)
    assert e <= PARAM_RTOL, "%s: parameter relative error %.3g" % (tag, e)
    return e


# ------------------------------------------------------------------ whole-tensor parity with a mismatch report
REPORT_LINES = []          # printed by tests/conftest.py in the terminal summary, also for passing tests
MISMATCH_BUDGET = 1e-6     # allowed fraction of code mismatches, each within 1 ulp of a code midpoint


def report(line: str):
    REPORT_LINES.append(line)
    print(line, flush=True)


def midpoint_distance_ulps(q: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Distance of each normalized value x to the nearest midpoint of neighbouring codes, in
    units of the binary32 spacing at x (midpoints are exact in binary64)."""
    mids = (q[:-1].astype(np.float64) + q[1:].astype(np.float64)) / 2
    x64 = x.astype(np.float64)
    d = np.abs(x64[:, None] - mids[None, :]).min(axis=1)
    ulp = np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)
    return d / ulp


def entry_midpoint_distance(prev, g, n, B, idx, key, hp, t) -> float:
    """ulps between the normalized new state of entry `idx` ("m_q" or "r_q") and the nearest code
    midpoint; the oracle re-forms the entry's block from the state before the step (`prev`) and
    the step's gradient.  Without weight decay the states do not depend on the weights."""
    qs, qu = codebooks()
    b = int(idx) // B
    s = slice(b * B, min(n, (b + 1) * B))
    x, y = oracle.adam8bit_block_normalized(np.zeros(s.stop - s.start, np.float32), g[s],
                                            prev["m_q"][s], prev["r_q"][s], prev["N_m"][b], prev["N_r"][b], qs, qu,
                                            hp["alpha"], hp["beta1"], hp["beta2"], hp["eps"], 0.0, t, 0)
    v = (x if key == "m_q" else y)[int(idx) - s.start: int(idx) - s.start + 1]
    return float(midpoint_distance_ulps(qs if key == "m_q" else qu, v)[0])


class WholeTensorParity:
    """Oracle trajectory of EVERY block of one device tensor under 8-bit Adam (free-running from the
    zero state), compared with the device result entry by entry after every step.

    Per step: the gradient comes to the host, the oracle advances all blocks (block ranges split
    over the host threads; blocks are independent), and codes, block maxima and weights are
    compared on the device chunk by chunk.  Code mismatches are counted; each one is located
    against the code midpoints (the oracle re-forms the normalized value of that entry from the
    previous state) and must lie within 1 ulp of a midpoint, their total within MISMATCH_BUDGET
    of the entries; the device state is then overwritten with the oracle's there (teacher forcing),
    so that one tie does not hide what follows.  Block maxima must agree bit for bit, weights
    within PARAM_RTOL."""

    def __init__(self, name, w_dev, B, hp=ADAM, chunk=1 << 26):
        import torch
        self.torch = torch
        self.name, self.B, self.hp, self.chunk = name, B, hp, chunk
        self.n = n = w_dev.numel()
        self.w = w_dev.cpu().numpy()
        self.st = zero_state(n, B)
        self.g_host = torch.empty(n, dtype=torch.float32, pin_memory=True)
        self.entries = 0
        self.code_mismatches = 0
        self.worst_ulps = 0.0
        self.worst_param = 0.0

    def oracle_step(self, g_dev, t, split=True):
        """Advance the host trajectory by one step with the device gradient; keeps what the
        report needs of the previous state."""
        self.g_host.copy_(g_dev)
        self.torch.cuda.synchronize()
        self.g = self.g_host.numpy()
        self.prev = {k: v.copy() for k, v in self.st.items()}
        self.t = t
        oracle_adam8(self.w, self.g, self.st, self.B, t=t, hp=self.hp, split=split)

    def _locate(self, idx, key):
        return entry_midpoint_distance(self.prev, self.g, self.n, self.B, idx, key, self.hp, self.t)

    def compare(self, w_dev, d, tag):
        """d: dict of device tensors m_q, r_q, N_m, N_r.  Returns the number of code mismatches of this step."""
        torch = self.torch
        n, step_bad = self.n, 0
        for key in ("N_m", "N_r"):
            ref = torch.from_numpy(self.st[key]).cuda()
            bad = int((d[key].view(torch.int32) != ref.view(torch.int32)).sum())
            assert bad == 0, "%s: %s differs in %d of %d blocks" % (tag, key, bad, ref.numel())
        for lo in range(0, n, self.chunk):
            hi = min(n, lo + self.chunk)
            for key in ("m_q", "r_q"):
                ref = torch.from_numpy(self.st[key][lo:hi]).cuda()
                ne = d[key][lo:hi] != ref
                bad = int(ne.sum())
                if bad:
                    where = (torch.nonzero(ne).flatten() + lo).cpu().numpy()
                    for i in where[:64]:
                        u = self._locate(i, key)
                        self.worst_ulps = max(self.worst_ulps, u)
                        assert u <= 1.0, "%s: %s[%d] differs (gpu %d, oracle %d) %.3g ulps away from the nearest midpoint" % (
                            tag, key, i, int(d[key][int(i)]), int(self.st[key][int(i)]), u)
                    d[key][lo:hi].copy_(ref)                     # teacher forcing
                    step_bad += bad
            ref = torch.from_numpy(self.w[lo:hi]).cuda()
            got = w_dev[lo:hi]
            if not torch.equal(got, ref):
                r64 = ref.double()
                err = float(((got.double() - r64).abs() / r64.abs().clamp_min(1e-30)).max())
                self.worst_param = max(self.worst_param, err)
                assert err <= PARAM_RTOL, "%s: parameter relative error %.3g" % (tag, err)
        self.entries += 2 * n
        self.code_mismatches += step_bad
        return step_bad

    def summary(self):
        return self.entries, self.code_mismatches, self.worst_ulps, self.worst_param


def report_parity(title, checks):
    """One line for the terminal summary: mismatching codes, their fraction, distance to the
    midpoints, parameter error, over all steps and tensors of `checks`; enforces the budget."""
    entries = sum(c.entries for c in checks)
    bad = sum(c.code_mismatches for c in checks)
    ulps = max([c.worst_ulps for c in checks] + [0.0])
    perr = max([c.worst_param for c in checks] + [0.0])
    frac = bad / max(1, entries)
    report("%s: %d of %d code entries differ from the oracle (fraction %.3g, allowed %.0e; farthest from a midpoint: "
           "%.3g ulps); block maxima bit-exact; max parameter relative error %.3g (allowed %.0e)"
           % (title, bad, entries, frac, MISMATCH_BUDGET, ulps, perr, PARAM_RTOL))
    assert frac <= MISMATCH_BUDGET
