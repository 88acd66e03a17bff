#!/usr/bin/env python3
"""Benchmark of the fused 8-bit Adam step on one MI355X.

One "step" is one q8_adam8bit_step over the whole workload: dequantize m and r, Adam update,
block absmax, re-quantization (Sec. IV of the paper), on inputs that are already resident in
HBM.  Default workload: one flat fp32 tensor of 10^9 parameters, B = 2048 (the configuration
the bandwidth target is stated on).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1b|1m] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

ADAM = dict(alpha=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
WORKLOADS = {
    "1b": dict(n=1_000_000_000, B=2048, name="config4: flat fp32 tensor, 1e9 params, 8-bit Adam, B=2048, grads N(0,1e-3)"),
    "1m": dict(n=1 << 20, B=2048, name="config1: flat fp32 tensor, 2^20 params, 8-bit Adam, B=2048, grads N(0,1e-3)"),
}


def algorithmic_bytes(n: int, B: int) -> int:
    """Bytes the method must move per step: read w, g (4+4), codes of m, r (1+1); write w (4)
    and both codes (1+1); plus read+write of two absmax values per block."""
    nb = -(-n // B)
    return 16 * n + 16 * nb


def measured_traffic(path: str):
    """HBM bytes per launch from the committed counter summary, if present (a line
    'traffic_bytes_per_launch: <int>')."""
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9]+)", open(path).read())
        return int(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(w_dev, g_dev, B: int, sample: int, steps: int):
    """The CPU oracle, as it stands, on the first `sample` parameters of the same workload,
    split at block boundaries over the host threads available to this process."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
    qs, qu = oracle.build_codebook(True), oracle.build_codebook(False)
    n = min(sample, w_dev.numel()) // B * B
    w = w_dev[:n].cpu().numpy().copy()
    g = g_dev[:n].cpu().numpy().copy()
    nb = n // B
    mq = np.full(n, 127, np.uint8); rq = np.zeros(n, np.uint8)
    Nm = np.zeros(nb, np.float32); Nr = np.zeros(nb, np.float32)
    per = -(-nb // cores)

    def run(k):
        b0, b1 = k * per, min(nb, (k + 1) * per)
        if b0 < b1:
            s = slice(b0 * B, b1 * B)
            oracle.adam8bit_step(w[s], g[s], mq[s], rq[s], Nm[b0:b1], Nr[b0:b1], qs, qu, B,
                                 ADAM["alpha"], ADAM["beta1"], ADAM["beta2"], ADAM["eps"], 0.0, 1, 0)
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(run, range(cores)))          # untimed first step: leaves a non-trivial state
        t0 = time.perf_counter()
        for _ in range(steps):
            list(ex.map(run, range(cores)))
        dt = time.perf_counter() - t0
    return dict(value=n * steps / dt, unit="params/s", cores=cores, kind="oracle",
                sample="first %d params of the workload, %d Adam steps after one untimed step, "
                       "block ranges split over %d threads" % (n, steps, cores))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="1b", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after timing, run one plain elementwise copy of the fp32 weights (4n bytes read, "
                         "4n written) so that counter runs can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2412_01195_amd import q8opt
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    q8opt.lib()
    wl = WORKLOADS[args.workload]
    n, B = wl["n"], wl["B"]
    nb = -(-n // B)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tab_s = q8opt.upload_qtable(q8opt.build_qtable(q8opt.build_codebook(True)))
    tab_u = q8opt.upload_qtable(q8opt.build_qtable(q8opt.build_codebook(False)))
    gen = torch.Generator(device=dev); gen.manual_seed(4)
    w = torch.empty(n, device=dev).uniform_(-0.1, 0.1, generator=gen)
    g = torch.empty(n, device=dev).normal_(0.0, 1e-3, generator=gen)
    m_q = torch.full((n,), 127, dtype=torch.uint8, device=dev)
    r_q = torch.zeros(n, dtype=torch.uint8, device=dev)
    N_m = torch.zeros(nb, device=dev); N_r = torch.zeros(nb, device=dev)

    t = 0

    def step():
        nonlocal t
        t += 1
        q8opt.adam8bit_step(w, g, m_q, r_q, N_m, N_r, tab_s, tab_u, B, **ADAM, t=t)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:                      # events sit on the stream the kernel is launched on
        a.record(); step(); b.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in ev]
    avg_kern_s = sum(kern_ms) / len(kern_ms) / 1e3

    if args.calibrate_copy:
        scratch = torch.empty_like(g)
        torch.mul(g, 1.0, out=scratch)
        torch.cuda.synchronize()
        del scratch

    alg = algorithmic_bytes(n, B)
    achieved = alg / avg_kern_s / 1e9
    out = {
        "metric": "fused 8-bit Adam step: params/sec (achieved HBM GB/s in roofline)",
        "value": n * args.steps / elapsed,
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 update, u8 states", "data": "synthetic",
        "config": {"workload": wl["name"], "params": n, "block_size": B, "optimizer": "adam8bit",
                   "hyper": ADAM, "bytes_per_param": 16},
        "hbm_gbps": achieved, "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(os.path.join(ROOT, "profiles", "adam8_kernel_1b_hbm_counters.md"))
                     if args.workload == "1b" else None,
                     "kernel": "adam8_kernel<2048>", "kernel_ms_avg": avg_kern_s * 1e3,
                     "kernel_ms_min": min(kern_ms), "kernel_ms_each": [round(x, 4) for x in kern_ms],
                     "algorithmic_bytes_per_launch": alg},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, g, B, args.cpu_sample, steps=2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
