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
