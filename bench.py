#!/usr/bin/env python3
"""Benchmark of the fused 8-bit Adam step on one MI355X.

One "step" is one q8_adam8bit_step over the whole workload: dequantize m and r, Adam update,
block absmax, re-quantization (Sec. IV of the paper), on inputs that are already resident in
HBM.  Default workload: one flat fp32 tensor of 10^9 parameters, B = 2048 (the configuration
the bandwidth target is stated on).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1b|...] [--no-cpu]

Other workloads (not the headline line): 1m (configuration 1), c2, c3, c5 (multi-tensor
configurations 2, 3, 5), df (DF-ResNet-shaped list, AdamW), sgd1b, quant1b, dequant1b (the
other kernels at 1e9 elements), 1b256 / 100m and --block-size (size and block-size effects).
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
    "1b256": dict(n=1_000_000_000, B=256, name="flat fp32 tensor, 1e9 params, 8-bit Adam, B=256, grads N(0,1e-3)"),
    "100m": dict(n=100_000_000, B=2048, name="flat fp32 tensor, 1e8 params, 8-bit Adam, B=2048, grads N(0,1e-3)"),
    "bf16_1b": dict(n=1_000_000_000, B=2048, name="flat bfloat16 weights and gradients (extension), 1e9 params, 8-bit Adam, B=2048, grads N(0,1e-3)"),
    "f16_1b": dict(n=1_000_000_000, B=2048, name="flat binary16 weights and gradients (extension), 1e9 params, 8-bit Adam, B=2048, grads N(0,1e-3)"),
    "sgd1b": dict(n=1_000_000_000, B=2048, name="flat fp32 tensor, 1e9 params, 8-bit SGD momentum, B=2048, grads N(0,1e-3)"),
    "probe1b": dict(n=1_000_000_000, B=2048, name="traffic of the config-4 step without its arithmetic (measurement aid): read w, g, both "
                    "code arrays, write w and both code arrays back unchanged; 1e9 params"),
}


# committed counter summaries (HBM bytes per launch) by workload
TRAFFIC_PROFILE = {"1b": "adam8_kernel_1b_hbm_counters.md", "bf16_1b": "adam8_kernel_bf16_1b_hbm_counters.md"}


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


def load_traffic_probe():
    """The benchmark's own measurement aid (workload probe1b): libq8opt_probe.so, built next to the
    product library from the same objects plus csrc/q8opt_probe.hip.  Returns a function
    probe(w, g, m_q, r_q, qtable_signed, qtable_unsigned) that moves the bytes of one Adam step at
    B = 2048 without its arithmetic (all values written back unchanged)."""
    import ctypes as C
    import torch
    from paper_2412_01195_amd import q8opt
    path = os.path.join(os.path.dirname(q8opt.LIB_PATH), "libq8opt_probe.so")
    if not os.path.exists(path):
        raise ImportError("libq8opt_probe.so is not built (%s); run __graft_entry__.build()" % path)
    L = C.CDLL(path)
    L.q8_probe_adam8bit_traffic.argtypes = [C.c_void_p] * 6 + [C.c_int64, C.c_void_p]
    L.q8_probe_adam8bit_traffic.restype = C.c_int

    def probe(w, g, m_q, r_q, tab_s, tab_u):
        st = L.q8_probe_adam8bit_traffic(w.data_ptr(), g.data_ptr(), m_q.data_ptr(), r_q.data_ptr(), tab_s.data_ptr(),
                                         tab_u.data_ptr(), w.numel(), torch.cuda.current_stream().cuda_stream)
        if st != 0:
            raise RuntimeError("q8_probe_adam8bit_traffic failed with status %d" % st)
    return probe


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
    # the sequential definition itself: one thread, the first 2^23 of those parameters
    n1 = min(n, 1 << 23) // B * B
    s1, b1 = slice(0, n1), n1 // B
    t1 = time.perf_counter()
    for _ in range(2):
        oracle.adam8bit_step(w[s1], g[s1], mq[s1], rq[s1], Nm[:b1], Nr[:b1], qs, qu, B,
                             ADAM["alpha"], ADAM["beta1"], ADAM["beta2"], ADAM["eps"], 0.0, 1, 0)
    dt1 = time.perf_counter() - t1
    return dict(value=n * steps / dt, unit="params/s", cores=cores, kind="oracle",
                sample="first %d params of the workload, %d Adam steps after one untimed step, "
                       "block ranges split over %d threads" % (n, steps, cores),
                one_core=dict(value=n1 * 2 / dt1, unit="params/s",
                              sample="first %d params, 2 further Adam steps on one thread" % n1))


def build_workload(name, torch, q8opt, dev):
    """Returns (description, params per step, algorithmic bytes per step, kernel name, step function,
    (w, g, B) for the cpu_baseline leg or None)."""
    from paper_2412_01195_amd import synth
    tab_s = q8opt.upload_qtable(q8opt.build_qtable(q8opt.build_codebook(True)))
    tab_u = q8opt.upload_qtable(q8opt.build_qtable(q8opt.build_codebook(False)))
    gen = torch.Generator(device=dev); gen.manual_seed(4)
    keep = [tab_s, tab_u]

    def state8(n, B, adam=True):
        nb = -(-n // B)
        st = dict(m_q=torch.full((n,), 127, dtype=torch.uint8, device=dev), N_m=torch.zeros(nb, device=dev))
        if adam:
            st.update(r_q=torch.zeros(n, dtype=torch.uint8, device=dev), N_r=torch.zeros(nb, device=dev))
        return st

    if name in ("bf16_1b", "f16_1b"):
        wl = WORKLOADS[name]
        n, B = wl["n"], wl["B"]
        dt, fn, tag = ((torch.bfloat16, q8opt.adam8bit_step_bf16, "Bf16") if name == "bf16_1b"
                       else (torch.float16, q8opt.adam8bit_step_f16, "F16"))
        w = torch.empty(n, device=dev).uniform_(-0.1, 0.1, generator=gen).to(dt)
        g = torch.empty(n, device=dev).normal_(0.0, 1e-3, generator=gen).to(dt)
        st = state8(n, B, True)
        t = [0]

        def step():
            t[0] += 1
            fn(w, g, st["m_q"], st["r_q"], st["N_m"], st["N_r"], tab_s, tab_u, B, **ADAM, t=t[0])
        # read w, g (2+2) and both codes (1+1), write w (2) and both codes (1+1), absmax as in the fp32 case
        return wl["name"], n, 10 * n + 16 * (-(-n // B)), "adam8_kernel<%d, %s>" % (B, tag), step, None, keep
    if name in ("1b", "1m", "sgd1b", "1b256", "100m"):
        wl = WORKLOADS[name]
        n, B = wl["n"], wl["B"]
        w = torch.empty(n, device=dev).uniform_(-0.1, 0.1, generator=gen)
        g = torch.empty(n, device=dev).normal_(0.0, 1e-3, generator=gen)
        adam = name != "sgd1b"
        st = state8(n, B, adam)
        t = [0]
        if adam:
            def step():
                t[0] += 1
                q8opt.adam8bit_step(w, g, st["m_q"], st["r_q"], st["N_m"], st["N_r"], tab_s, tab_u, B, **ADAM, t=t[0])
            return wl["name"], n, algorithmic_bytes(n, B), "adam8_kernel<%d, float>" % B, step, (w, g, B), keep
        def step():
            q8opt.sgd8bit_step(w, g, st["m_q"], st["N_m"], tab_s, B, 0.1, 0.9, 1e-4)
        return wl["name"], n, 14 * n + 8 * (-(-n // B)), "sgd8_kernel<%d, float>" % B, step, None, keep
    if name == "probe1b":
        n = WORKLOADS[name]["n"]
        w = torch.empty(n, device=dev).uniform_(-0.1, 0.1, generator=gen)
        g = torch.empty(n, device=dev).normal_(0.0, 1e-3, generator=gen)
        st = state8(n, 2048, True)
        probe = load_traffic_probe()
        return (WORKLOADS[name]["name"], n, 16 * n, "traffic_probe_kernel",
                lambda: probe(w, g, st["m_q"], st["r_q"], tab_s, tab_u), None, keep)
    if name in ("quant1b", "dequant1b"):
        n, B = 1_000_000_000, 2048
        nb = -(-n // B)
        T = torch.empty(n, device=dev).normal_(0.0, 1e-3, generator=gen)
        TQ = torch.empty(n, dtype=torch.uint8, device=dev); N = torch.empty(nb, device=dev)
        q8opt.quantize_blockwise(tab_s, T, B, TQ, N)
        if name == "quant1b":
            return ("stand-alone block-wise quantization (Eq. quant1-2), 1e9 fp32 values, B=2048", n, 5 * n + 4 * nb,
                    "quantize_kernel<2048>", lambda: q8opt.quantize_blockwise(tab_s, T, B, TQ, N), None, keep)
        return ("stand-alone dequantization (Eq. quant3), 1e9 codes, B=2048", n, 5 * n + 4 * nb,
                "dequantize_kernel", lambda: q8opt.dequantize_blockwise(tab_s, TQ, N, B, T), None, keep)
    # multi-tensor lists
    if name == "c5":
        B, adam, min8 = 256, True, 0
        sizes = [1_562_500] * 64
        stds = [synth.heavy_tail_scale(5, i) for i in range(64)]
        desc = "config5: 64 tensors x 1 562 500 params, 8-bit Adam, B=256, Student-t(3) grads scaled 1e-6..1e-1 per tensor"
    elif name == "c2":
        B, adam, min8 = 2048, False, 0
        specs = synth.resnet34_specs(); sizes = [s.numel for s in specs]
        stds = [synth.fan_in_std(s, 1e-2) for s in specs]
        desc = "config2: ResNet34-shaped list, 111 tensors, 8 168 800 params, 8-bit SGD momentum, B=2048"
    elif name == "df":
        B, adam, min8 = 2048, True, 4096
        specs = synth.df_resnet_specs(); sizes = [s.numel for s in specs]
        stds = [synth.fan_in_std(s, 1e-2) for s in specs]
        adamw = dict(weight_decay=0.05, flags=q8opt.FLAG_DECOUPLED_WD | q8opt.FLAG_BIAS_CORRECTION)
        desc = ("DF-ResNet-shaped list (deepest reversible form), 638 tensors, 14 060 656 params, 8-bit AdamW "
                "(decoupled wd 0.05, bias correction; fp32 states under 4096 elements), B=2048")
    else:
        B, adam, min8 = 2048, True, 4096
        specs = synth.resnet293_specs(); sizes = [s.numel for s in specs]
        stds = [1e-3] * len(sizes)
        desc = "config3: ResNet293-shaped list, 891 tensors, 30 160 480 params, 8-bit Adam (fp32 states under 4096 elements), B=2048"
    tensors, alg = [], 0
    for n, sd in zip(sizes, stds):
        w = torch.empty(n, device=dev).uniform_(-0.1, 0.1, generator=gen)
        if name == "c5":
            z = torch.randn(n, device=dev, generator=gen)
            chi = torch.randn(3, n, device=dev, generator=gen).pow_(2).sum(0).div_(3.0).sqrt_()
            g = z.div_(chi).mul_(sd)
        else:
            g = torch.empty(n, device=dev).normal_(0.0, sd, generator=gen)
        t = dict(w=w, g=g)
        nb = -(-n // B)
        if n >= min8:
            t.update(state8(n, B, adam))
            alg += (16 * n + 16 * nb) if adam else (14 * n + 8 * nb)
        else:
            t["m_f32"] = torch.zeros(n, device=dev)
            if adam:
                t["r_f32"] = torch.zeros(n, device=dev)
            alg += (32 if adam else 20) * n
        tensors.append(t)
    plan = q8opt.Plan(tensors, B)
    keep += [tensors, plan]
    tt = [0]
    if adam:
        extra = adamw if name == "df" else {}

        def step():
            tt[0] += 1
            plan.multi_adam8bit_step(tab_s, tab_u, **ADAM, t=tt[0], **extra)
        kern = "adam8_kernel<%d, float>" % B
    else:
        def step():
            plan.multi_sgd8bit_step(tab_s, 0.1, 0.9, 1e-4)
        kern = "sgd8_kernel<%d, float>" % B
    return desc, sum(sizes), alg, kern, step, None, keep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed warm-up steps; default: at least 10 and at least 0.25 s worth (the chip's power "
                         "management needs 30-50 ms of continuous load to settle: launches inside that transient "
                         "run up to 30 %% slower than the steady state that follows)")
    ap.add_argument("--workload", default="1b",
                    choices=["1b", "1m", "1b256", "100m", "bf16_1b", "f16_1b", "sgd1b", "probe1b", "quant1b", "dequant1b", "c2", "c3", "c5", "df"],
                    help="1b (default) = configuration 4, the one the headline metric is quoted on")
    ap.add_argument("--block-size", type=int, default=0,
                    help="override the block size B of a flat workload (block-size sweep; not the headline line)")
    ap.add_argument("--params", type=int, default=0,
                    help="override the number of parameters of a flat workload (size sweep; not the headline line)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after timing, run one plain elementwise copy of a 1e9-float tensor (4e9 bytes read, "
                         "4e9 written) so that counter runs can scale FETCH_SIZE / WRITE_SIZE")
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
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.block_size:
        if args.workload not in WORKLOADS:
            print("bench.py: --block-size applies to the flat workloads only", file=sys.stderr)
            sys.exit(2)
        WORKLOADS[args.workload] = dict(WORKLOADS[args.workload], B=args.block_size,
                                        name=WORKLOADS[args.workload]["name"] + " [B overridden to %d]" % args.block_size)
    if args.params:
        if args.workload not in WORKLOADS:
            print("bench.py: --params applies to the flat workloads only", file=sys.stderr)
            sys.exit(2)
        WORKLOADS[args.workload] = dict(WORKLOADS[args.workload], n=args.params,
                                        name=WORKLOADS[args.workload]["name"] + " [size overridden to %d]" % args.params)
    desc, nparams, alg, kernel, step, cpu_args, keep = build_workload(args.workload, torch, q8opt, dev)

    if args.warmup is None:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        args.warmup, t_w = 10, time.perf_counter()
        while time.perf_counter() - t_w < 0.25 and args.warmup < 20000:
            for _ in range(10):
                step()
            torch.cuda.synchronize()
            args.warmup += 10
    else:
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
        src = torch.zeros(1_000_000_000, device=dev)
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    achieved = alg / avg_kern_s / 1e9
    headline = args.workload in ("1b", "1m") and not args.block_size and not args.params
    out = {
        "metric": "fused 8-bit Adam step: params/sec (achieved HBM GB/s in roofline)" if headline
                  else "%s: params/sec (achieved HBM GB/s in roofline)" % kernel,
        "value": nparams * args.steps / elapsed,
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",      # arithmetic type; storage: u8 states, f32 (or bf16) w and g
        "config": {"workload": desc, "params": nparams, "hyper": ADAM if "adam" in kernel else None,
                   "storage": "u8 states, %s w and g" % {"bf16_1b": "bf16", "f16_1b": "f16"}.get(args.workload, "f32")},
        "hbm_gbps": achieved, "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(os.path.join(ROOT, "profiles", TRAFFIC_PROFILE.get(args.workload, "")))
                     if args.workload in TRAFFIC_PROFILE and not args.block_size and not args.params else None,
                     "traffic_source": ("profiles/%s: two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this workload, "
                                        "committed together with the kernel; not measured in this run"
                                        % TRAFFIC_PROFILE[args.workload]) if args.workload in TRAFFIC_PROFILE else None,
                     "kernel": kernel, "kernel_ms_avg": avg_kern_s * 1e3,
                     "kernel_ms_min": min(kern_ms), "kernel_ms_each": [round(x, 4) for x in kern_ms],
                     "algorithmic_bytes_per_launch": alg},
    }
    if not args.no_cpu and cpu_args is not None:
        out["cpu_baseline"] = cpu_baseline(*cpu_args, args.cpu_sample, steps=4)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
