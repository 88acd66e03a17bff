"""GPU parity of the binary16-storage steps (weights and gradients held as IEEE binary16; an
extension outside the paper) against the CPU oracle: stored weights, codes and absmax all
bit-exact -- the arithmetic is the binary32 step, and the one rounding of the new weight
is decided in binary32 on both sides."""
import os

import numpy as np
import pytest

import oracle
from paper_2412_01195_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def q8():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2412_01195_amd import q8opt
    q8opt.lib()
    return q8opt


@pytest.fixture(scope="module")
def tabs(q8):
    ts = q8.upload_qtable(q8.build_qtable(q8.build_codebook(True)))
    tu = q8.upload_qtable(q8.build_qtable(q8.build_codebook(False)))
    return ts, tu


def dev16(bits):
    return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.float16)


def host16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def dev_state(st):
    return {k: torch.from_numpy(v.copy()).cuda() for k, v in st.items()}


def assert_all_equal(tag, w_dev, w_ref, st_dev, st_ref):
    got = host16(w_dev)
    assert np.array_equal(got, w_ref), "%s: %d stored weights differ" % (tag, int((got != w_ref).sum()))
    for k in st_ref:
        a, b = st_dev[k].cpu().numpy(), st_ref[k]
        if a.dtype == np.float32:
            a, b = a.view(np.uint32), b.view(np.uint32)
        assert np.array_equal(a, b), "%s: %s differs in %d entries" % (tag, k, int((a != b).sum()))


def inputs(n, seed):
    return synth.f16_bits(synth.uniform_weights(seed, 0, n))


def grad(n, seed, step, std=1e-2):
    return synth.f16_bits(synth.normal_grad(seed, 0, step, n, std))


@pytest.mark.parametrize("n,B", [(1, 64), (67, 64), (4097, 64), (1000, 128), (256 * 9 + 131, 256), (5001, 512),
                                 (1024 * 3 + 1, 1024), (2048 * 5 + 513, 2048), (2047, 2048), (4096 * 3 + 99, 4096),
                                 (300001, 256), (1 << 20, 2048)])
@pytest.mark.parametrize("mode", ["plain", "wd", "adamw_bc"])
def test_adam_f16_parity(q8, tabs, n, B, mode):
    wd, flags = {"plain": (0.0, 0), "wd": (1e-2, 0),
                 "adamw_bc": (1e-2, oracle.FLAG_BIAS_CORRECTION | oracle.FLAG_DECOUPLED_WD)}[mode]
    w = inputs(n, 100 + n % 97)
    st = H.zero_state(n, B)
    w_d, st_d = dev16(w), dev_state(st)
    for t in range(1, 5):
        g = grad(n, 200 + n % 89, t)
        H.oracle_adam8(w, g, st, B, wd=wd, t=t, flags=flags, f16=True)
        q8.adam8bit_step_f16(w_d, dev16(g), st_d["m_q"], st_d["r_q"], st_d["N_m"], st_d["N_r"], tabs[0], tabs[1], B,
                              weight_decay=wd, t=t, flags=flags, **{k: H.ADAM[k] for k in H.ADAM})
        assert_all_equal("adam f16 n=%d B=%d %s step %d" % (n, B, mode, t), w_d, w, st_d, st)


@pytest.mark.parametrize("n,B", [(1, 64), (4099, 64), (256 * 9 + 131, 256), (2048 * 5 + 513, 2048), (300001, 4096)])
@pytest.mark.parametrize("wd", [0.0, 1e-4])
def test_sgd_f16_parity(q8, tabs, n, B, wd):
    w = inputs(n, 300 + n % 97)
    st = H.zero_state(n, B, adam=False)
    w_d, st_d = dev16(w), dev_state(st)
    for t in range(1, 5):
        g = grad(n, 400 + n % 89, t)
        H.oracle_sgd8(w, g, st, B, wd=wd, f16=True)
        q8.sgd8bit_step_f16(w_d, dev16(g), st_d["m_q"], st_d["N_m"], tabs[0], B, weight_decay=wd, **H.SGD)
        assert_all_equal("sgd f16 n=%d B=%d step %d" % (n, B, t), w_d, w, st_d, st)


def test_small_updates_are_absorbed_by_rounding(q8, tabs):
    """Weights in [1, 2) with alpha = 5e-5: every update (at most alpha * 3.2) is below half a
    binary16 ulp, also for a weight of exactly 1.0 whose lower neighbour is only 2^-11 away, so
    the stored weights stay put while the states advance."""
    n, B = 1 << 16, 2048
    w = synth.f16_bits(1.0 + synth.uniform_weights(17, 0, n, 0.0, 0.99))
    g = grad(n, 18, 1)
    st = H.zero_state(n, B)
    w_d, st_d = dev16(w), dev_state(st)
    hp = dict(H.ADAM, alpha=5e-5)
    q8.adam8bit_step_f16(w_d, dev16(g), st_d["m_q"], st_d["r_q"], st_d["N_m"], st_d["N_r"], tabs[0], tabs[1], B, **hp)
    assert np.array_equal(host16(w_d), w)
    assert int((st_d["m_q"] != 127).sum()) > 0


def test_f16_list_with_fp32_state_tensors(q8, tabs):
    """Multi-tensor plan over binary16 tensors: large ones with 8-bit states, small ones with
    32-bit states (same formulas, weight rounded once)."""
    B = 256
    sizes = [3 * 3 * 64 * 64, 64, 64, 1000, 5000, 4097, 128 * 128 + 3, 10]
    qs, qu = H.codebooks()
    tens, refs = [], []
    for i, n in enumerate(sizes):
        w = inputs(n, 500 + i)
        small = n < 4096
        ref = dict(w=w, n=n, small=small)
        d = dict(w=dev16(w))
        if small:
            ref.update(m=np.zeros(n, np.float32), r=np.zeros(n, np.float32))
            d.update(m_f32=torch.zeros(n, device="cuda"), r_f32=torch.zeros(n, device="cuda"))
        else:
            ref.update(st=H.zero_state(n, B))
            d.update(dev_state(ref["st"]))
        d["g"] = torch.zeros(n, dtype=torch.float16, device="cuda")
        tens.append(d); refs.append(ref)
    plan = q8.Plan(tens, B, wg_dtype="float16")
    try:
        for t in range(1, 4):
            for i, (d, ref) in enumerate(zip(tens, refs)):
                g = grad(ref["n"], 600 + i, t)
                d["g"].copy_(dev16(g))
                if ref["small"]:
                    w32 = ref["w"].view(np.float16).astype(np.float32)
                    g32 = g.view(np.float16).astype(np.float32)
                    oracle.adam32_step(w32, g32, ref["m"], ref["r"], wd=1e-2, t=t, **H.ADAM)
                    ref["w"][:] = np.array([oracle.f32_to_f16(v) for v in w32], np.uint16)
                else:
                    H.oracle_adam8(ref["w"], g, ref["st"], B, wd=1e-2, t=t, f16=True)
            plan.multi_adam8bit_step(tabs[0], tabs[1], weight_decay=1e-2, t=t, **H.ADAM)
            for i, (d, ref) in enumerate(zip(tens, refs)):
                tag = "tensor %d step %d" % (i, t)
                if ref["small"]:
                    assert np.array_equal(host16(d["w"]), ref["w"]), tag
                    assert np.array_equal(d["m_f32"].cpu().numpy().view(np.uint32), ref["m"].view(np.uint32)), tag
                    assert np.array_equal(d["r_f32"].cpu().numpy().view(np.uint32), ref["r"].view(np.uint32)), tag
                else:
                    assert_all_equal(tag, d["w"], ref["w"], {k: d[k] for k in ref["st"]}, ref["st"])
    finally:
        plan.destroy()


def test_f16_sgd_list(q8, tabs):
    B = 2048
    specs = synth.resnet34_specs()[:24]
    tens, refs = [], []
    for i, sp in enumerate(specs):
        n = sp.numel
        w = inputs(n, 700 + i)
        st = H.zero_state(n, B, adam=False)
        d = dict(w=dev16(w), g=torch.zeros(n, dtype=torch.float16, device="cuda"), **dev_state(st))
        tens.append(d); refs.append(dict(w=w, st=st, n=n))
    plan = q8.Plan(tens, B, wg_dtype="float16")
    try:
        for t in range(1, 4):
            for i, (d, ref) in enumerate(zip(tens, refs)):
                g = grad(ref["n"], 800 + i, t)
                d["g"].copy_(dev16(g))
                H.oracle_sgd8(ref["w"], g, ref["st"], B, wd=1e-4, f16=True)
            plan.multi_sgd8bit_step(tabs[0], weight_decay=1e-4, **H.SGD)
            for i, (d, ref) in enumerate(zip(tens, refs)):
                assert_all_equal("tensor %d step %d" % (i, t), d["w"], ref["w"], {k: d[k] for k in ref["st"]}, ref["st"])
    finally:
        plan.destroy()


def test_f16_alignment_and_arguments(q8, tabs):
    n, B = 4096, 256
    buf = torch.zeros(n + 8, dtype=torch.float16, device="cuda")
    g = torch.zeros(n, dtype=torch.float16, device="cuda")
    st = dev_state(H.zero_state(n, B))
    args = (st["m_q"], st["r_q"], st["N_m"], st["N_r"], tabs[0], tabs[1], B)
    with pytest.raises(q8.Q8Error) as e:
        q8.adam8bit_step_f16(buf[1:n + 1].data_ptr(), g, *args, n=n, **H.ADAM)       # 2-byte aligned only
    assert e.value.status == q8.EALIGN
    q8.adam8bit_step_f16(buf[4:n + 4].data_ptr(), g, *args, n=n, **H.ADAM)            # 8-byte aligned: accepted
    with pytest.raises(ValueError):
        q8.adam8bit_step_f16(torch.zeros(n, device="cuda"), g, *args, **H.ADAM)       # binding refuses float32 here
    q8.adam8bit_step_f16(buf, g, *args, n=0, **H.ADAM)
    torch.cuda.synchronize()


def test_f16_large_sampled_blocks(q8, tabs):
    """2^27 + 12345 elements at B = 2048 in the benchmark's launch configuration; the oracle
    recomputes a sample of whole blocks (first, last/ragged, and random ones) each step."""
    n, B = (1 << 27) + 12345, 2048
    nb = oracle.nblocks(n, B)
    rng = np.random.default_rng(5)
    blocks = np.unique(np.concatenate([[0, 1, nb - 2, nb - 1], rng.integers(0, nb, 400)]))
    gen = torch.Generator(device="cuda"); gen.manual_seed(9)
    w_d = (torch.rand(n, device="cuda", generator=gen) - 0.5).mul_(0.1).to(torch.float16)
    st_d = dev_state(H.zero_state(n, B))
    sl = [slice(int(b) * B, min(n, (int(b) + 1) * B)) for b in blocks]
    for t in range(1, 4):
        g_d = torch.randn(n, device="cuda", generator=gen).mul_(1e-2).to(torch.float16)
        before = [(host16(w_d[s]), {k: st_d[k][s].cpu().numpy() for k in ("m_q", "r_q")},
                   {k: st_d[k][int(b):int(b) + 1].cpu().numpy() for k in ("N_m", "N_r")}, host16(g_d[s]))
                  for b, s in zip(blocks, sl)]
        q8.adam8bit_step_f16(w_d, g_d, st_d["m_q"], st_d["r_q"], st_d["N_m"], st_d["N_r"], tabs[0], tabs[1], B,
                              weight_decay=1e-2, t=t, **H.ADAM)
        for (w, codes, Ns, g), b, s in zip(before, blocks, sl):
            st = dict(m_q=codes["m_q"].copy(), r_q=codes["r_q"].copy(), N_m=Ns["N_m"].copy(), N_r=Ns["N_r"].copy())
            w = w.copy()
            H.oracle_adam8(w, g, st, B, wd=1e-2, t=t, f16=True, split=False)
            assert np.array_equal(host16(w_d[s]), w), ("w", int(b), t)
            for k in ("m_q", "r_q"):
                assert np.array_equal(st_d[k][s].cpu().numpy(), st[k]), (k, int(b), t)
            for k in ("N_m", "N_r"):
                assert np.array_equal(st_d[k][int(b):int(b) + 1].cpu().numpy().view(np.uint32), st[k].view(np.uint32)), (k, int(b), t)


def test_f16_subnormal_and_large_weights(q8, tabs):
    """Weights across binary16's whole range (subnormals below 6.1e-5 up to the largest finite
    values): the single rounding of the new weight, including into and out of the subnormal range,
    matches the oracle bit for bit."""
    n, B = 256 * 37 + 5, 256
    rng = np.random.default_rng(44)
    mag = 10.0 ** rng.uniform(-8.0, 4.8, n)
    w = synth.f16_bits((mag * rng.choice([-1.0, 1.0], n)).astype(np.float32))
    st = H.zero_state(n, B)
    w_d, st_d = dev16(w), dev_state(st)
    hp = dict(H.ADAM, alpha=1e-5)
    for t in range(1, 5):
        g = synth.f16_bits((rng.standard_normal(n) * 10.0 ** rng.uniform(-7, 1, n)).astype(np.float32))
        H.oracle_adam8(w, g, st, B, wd=1e-2, t=t, hp=hp, f16=True)
        q8.adam8bit_step_f16(w_d, dev16(g), st_d["m_q"], st_d["r_q"], st_d["N_m"], st_d["N_r"], tabs[0], tabs[1], B,
                             weight_decay=1e-2, t=t, **hp)
        assert_all_equal("f16 range step %d" % t, w_d, w, st_d, st)


def test_f16_one_billion_parameters_every_entry(q8, tabs):
    """10^9 parameters at B = 2048 in the benchmark's launch configuration (the workload
    `f16_1b` of bench.py), three steps with decoupled decay and bias correction: the oracle
    advances every block on the host threads; stored weights, codes and block maxima are
    compared entry by entry on the device after every step and must be identical."""
    n, B, chunk = 1_000_000_000, 2048, 1 << 27
    gen = torch.Generator(device="cuda"); gen.manual_seed(21)
    w_d = torch.empty(n, dtype=torch.float16, device="cuda")
    g_d = torch.empty(n, dtype=torch.float16, device="cuda")
    for lo in range(0, n, chunk):                                    # generate in pieces: bounded binary32 temporaries
        hi = min(n, lo + chunk)
        w_d[lo:hi] = (torch.rand(hi - lo, device="cuda", generator=gen) - 0.5).mul_(0.2).to(torch.float16)
    st_d = dev_state(H.zero_state(n, B))
    w_h = host16(w_d)
    st_h = H.zero_state(n, B)
    flags = q8.FLAG_BIAS_CORRECTION | q8.FLAG_DECOUPLED_WD
    for t in range(1, 4):
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            g_d[lo:hi] = torch.randn(hi - lo, device="cuda", generator=gen).mul_(1e-3).to(torch.float16)
        q8.adam8bit_step_f16(w_d, g_d, st_d["m_q"], st_d["r_q"], st_d["N_m"], st_d["N_r"], tabs[0], tabs[1], B,
                              weight_decay=1e-2, t=t, flags=flags, **H.ADAM)
        H.oracle_adam8(w_h, host16(g_d), st_h, B, wd=1e-2, t=t, flags=flags, f16=True)
        for k in ("N_m", "N_r"):
            ref = torch.from_numpy(st_h[k]).cuda()
            bad = int((st_d[k].view(torch.int32) != ref.view(torch.int32)).sum())
            assert bad == 0, "step %d: %s differs in %d blocks" % (t, k, bad)
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            for k in ("m_q", "r_q"):
                bad = int((st_d[k][lo:hi] != torch.from_numpy(st_h[k][lo:hi]).cuda()).sum())
                assert bad == 0, "step %d: %s differs in %d entries of [%d, %d)" % (t, k, bad, lo, hi)
            ref = torch.from_numpy(w_h[lo:hi].view(np.int16)).cuda()
            bad = int((w_d[lo:hi].view(torch.int16) != ref).sum())
            assert bad == 0, "step %d: %d stored weights differ in [%d, %d)" % (t, bad, lo, hi)
    H.report("f16 storage, 1e9 parameters, B=2048, 3 steps (AdamW with bias correction): every stored weight, "
             "code and block maximum identical to the oracle's")


ROUND_BINADES = os.environ.get("Q8_ROUND_BINADES", "-26,-25,-24,-15,-14,0,15,16")      # "all" = every binade of [2^-80, 2^40]


def test_f16_rounding_of_the_new_weight_over_whole_binades(q8, tabs):
    """The one rounding of the new weight to the storage type, on dense sets of binary32 values:
    beta1 = beta2 = 1 and g = 0 keep the states, codes of 1.0 with N_r = 1 make the denominator
    1, so with alpha = 1 and w = 0 the stored weight is the rounding of -(Q[code] * N_m).  One
    launch takes every binary32 N_m of a binade (2^23 blocks of 64) times 64 codes; stored
    weights, codes and block maxima against the oracle, bit for bit.  Q8_ROUND_BINADES=all runs
    the 120 binades of [2^-80, 2^40]."""
    B = 64
    binades = range(-80, 40) if ROUND_BINADES == "all" else [int(x) for x in ROUND_BINADES.split(",")]
    nb = 1 << 23
    n = nb * B
    hp = dict(alpha=1.0, beta1=1.0, beta2=1.0, eps=0.0)
    codes = np.concatenate([np.arange(0, 127, 4), np.arange(129, 256, 4)]).astype(np.uint8)
    m_q0 = np.tile(codes, nb)
    zeros16 = np.zeros(n, np.uint16)
    g_d = torch.zeros(n, dtype=torch.float16, device="cuda")
    for e in binades:
        N_m0 = (np.uint32((e + 127) << 23) + np.arange(nb, dtype=np.uint32)).view(np.float32)
        st = dict(m_q=m_q0.copy(), r_q=np.full(n, 255, np.uint8), N_m=N_m0.copy(), N_r=np.ones(nb, np.float32))
        w_ref = zeros16.copy()
        w = torch.zeros(n, dtype=torch.float16, device="cuda"); d = dev_state(st)
        q8.adam8bit_step_f16(w, g_d, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **hp)
        H.oracle_adam8(w_ref, zeros16, st, B, hp=hp, f16=True)
        bad = int((w.view(torch.int16) != torch.from_numpy(w_ref.view(np.int16)).cuda()).sum())
        assert bad == 0, "binade 2^%d: %d of %d stored weights differ" % (e, bad, n)
        print("binade 2^%d done" % e, flush=True)                 # progress for the long run (pytest -s)
        for k in ("m_q", "r_q", "N_m", "N_r"):
            assert torch.equal(d[k].view(torch.uint8), torch.from_numpy(st[k]).cuda().view(torch.uint8)), (e, k)
        del w, d
    H.report("f16: rounding of the new weight on %d whole binades of first states (%d values each): identical to "
             "the oracle's" % (len(binades), n))
