"""GPU parity of the stand-alone kernels and of the single-tensor steps against the CPU
oracle, element by element: codes and absmax bit-exact, parameters within 1e-6 relative
(the bar stated for this path).  Every call goes through the C ABI."""
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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def adversarial_tensor(q, n, B, rng):
    """Random magnitudes per block plus values whose quotient by the block maximum sits on
    codes, on code midpoints and one ulp around them."""
    T = (rng.standard_normal(n) * 10.0 ** rng.uniform(-5, 1)).astype(np.float32)
    nb = -(-n // B)
    mids = ((q[:-1].astype(np.float64) + q[1:].astype(np.float64)) / 2).astype(np.float32)
    special = np.concatenate([q, mids, np.nextafter(mids, np.float32(2)), np.nextafter(mids, np.float32(-2))])
    for b in range(nb):
        lo, hi = b * B, min(n, (b + 1) * B)
        N = np.float32(2.0 ** rng.integers(-20, 8)) if b % 2 == 0 else np.abs(T[lo:hi]).max()
        k = min(hi - lo, special.size)
        pick = rng.choice(special, size=k, replace=False)
        idx = rng.choice(hi - lo, size=k, replace=False)
        blk = T[lo:hi]
        blk[idx] = (pick * N).astype(np.float32)
        blk[np.abs(blk) > N] = 0
        if hi - lo > 1:
            blk[rng.integers(0, hi - lo)] = N if b % 3 else -N       # negative arg-max in every third block
    return T


@pytest.mark.parametrize("signed", [True, False], ids=["signed", "unsigned"])
@pytest.mark.parametrize("n,B", [(1, 64), (63, 64), (4097, 64), (1000, 128), (256 * 9 + 132, 256), (5000, 512),
                                 (1024 * 3 + 1, 1024), (2048 * 5 + 512, 2048), (2047, 2048), (2048, 2048),
                                 (4096 * 3 + 100, 4096), (300000, 2048), (300001, 256)])
def test_quantize_dequantize_parity(q8, tabs, signed, n, B):
    q = H.codebooks()[0 if signed else 1]
    tab = tabs[0 if signed else 1]
    rng = np.random.default_rng(n * 31 + B)
    T = adversarial_tensor(q, n, B, rng)
    if not signed and n > 10:
        T = np.abs(T) if n % 2 else T            # unsigned map also sees negative inputs (clamped to code 0)
    TQ_ref, N_ref = oracle.quantize_blockwise(q, T, B)
    nb = oracle.nblocks(n, B)
    TQ = torch.full((n,), 7, dtype=torch.uint8, device="cuda"); N = torch.full((nb,), -1.0, device="cuda")
    q8.quantize_blockwise(tab, dev(T), B, TQ, N)
    assert np.array_equal(N.cpu().numpy().view(np.uint32), N_ref.view(np.uint32))
    got = TQ.cpu().numpy()
    assert np.array_equal(got, TQ_ref), np.flatnonzero(got != TQ_ref)[:10]
    TD = torch.empty(n, device="cuda")
    q8.dequantize_blockwise(tab, TQ, N, B, TD)
    assert np.array_equal(TD.cpu().numpy().view(np.uint32), oracle.dequantize_blockwise(q, TQ_ref, N_ref, B).view(np.uint32))


def test_quantize_extreme_block_maxima(q8, tabs):
    """Blocks whose maximum is tiny, huge, denormal or zero take the plain-divide path."""
    q = H.codebooks()[0]
    rng = np.random.default_rng(5)
    B, nb = 256, 12
    scales = [0.0, 1e-45, 1e-40, 1e-38, 2.0 ** -61, 2.0 ** -60, 2.0 ** -59, 2.0 ** 59, 2.0 ** 60, 2.0 ** 61, 1e38, 3e38]
    T = np.concatenate([(rng.uniform(-1, 1, B) * s).astype(np.float32) for s in scales])
    TQ_ref, N_ref = oracle.quantize_blockwise(q, T, B)
    TQ = torch.empty(T.size, dtype=torch.uint8, device="cuda"); N = torch.empty(nb, device="cuda")
    q8.quantize_blockwise(tabs[0], dev(T), B, TQ, N)
    assert np.array_equal(N.cpu().numpy().view(np.uint32), N_ref.view(np.uint32))
    assert np.array_equal(TQ.cpu().numpy(), TQ_ref)


def run_adam(q8, tabs, n, B, steps, seed, std=1e-3, wd=0.0, flags=0, check_every=True):
    w_ref = synth.uniform_weights(seed, 0, n)
    st = H.zero_state(n, B)
    w = dev(w_ref); d = {k: dev(v) for k, v in st.items()}
    worst = 0.0
    for t in range(1, steps + 1):
        g = synth.normal_grad(seed, 0, t, n, std)
        q8.adam8bit_step(w, dev(g), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B,
                         **H.ADAM, weight_decay=wd, t=t, flags=flags)
        H.oracle_adam8(w_ref, g, st, B, wd=wd, t=t, flags=flags)
        if check_every or t == steps:
            worst = max(worst, H.assert_state_equal("step %d" % t, d, st, w, w_ref))
    return worst


def run_sgd(q8, tabs, n, B, steps, seed, std=1e-2, wd=1e-4):
    w_ref = synth.uniform_weights(seed, 0, n)
    st = H.zero_state(n, B, adam=False)
    w = dev(w_ref); d = {k: dev(v) for k, v in st.items()}
    for t in range(1, steps + 1):
        g = synth.normal_grad(seed, 0, t, n, std)
        q8.sgd8bit_step(w, dev(g), d["m_q"], d["N_m"], tabs[0], B, **H.SGD, weight_decay=wd)
        H.oracle_sgd8(w_ref, g, st, B, wd=wd)
        H.assert_state_equal("step %d" % t, d, st, w, w_ref)


@pytest.mark.parametrize("n,B", [(1, 2048), (5, 64), (2048, 2048), (2049, 2048), (4 * 2048 + 512, 2048),
                                 (1000, 256), (6103 * 256 + 132, 256), (777, 128), (3 * 512 + 7, 512),
                                 (5000, 1024), (3 * 4096 + 1, 4096)])
def test_adam8bit_small_and_ragged(q8, tabs, n, B):
    run_adam(q8, tabs, n, B, 6, seed=100 + B)


@pytest.mark.parametrize("n,B", [(3, 2048), (2048 * 3 + 5, 2048), (1562500, 256), (700, 64), (9000, 4096)])
def test_sgd8bit_small_and_ragged(q8, tabs, n, B):
    run_sgd(q8, tabs, n, B, 6, seed=200 + B)


def test_config1_adam_flat_1m(q8, tabs):
    """Config 1: one flat tensor of 2^20 parameters, Adam, B = 2048, 10 steps from the zero state."""
    worst = run_adam(q8, tabs, 1 << 20, 2048, 10, seed=1)
    print("config 1: max parameter relative error %.3g" % worst)


def test_adam_extension_flags(q8, tabs):
    for flags, wd in ((0, 1e-2), (1, 0.0), (2, 0.05), (3, 0.05)):
        run_adam(q8, tabs, 2048 * 3 + 77, 2048, 5, seed=300 + flags, wd=wd, flags=flags)


def test_adam_tiny_zero_and_huge_gradients(q8, tabs):
    """Rows with exact zeros, denormal-range second moments and huge values: the square
    root of the denominator switches between its short and its general form per row and
    must agree with the oracle in both."""
    n, B = 2048 * 6 + 300, 2048
    rng = np.random.default_rng(77)
    w_ref = synth.uniform_weights(78, 0, n)
    st = H.zero_state(n, B)
    w = dev(w_ref); d = {k: dev(v) for k, v in st.items()}
    scales = np.array([0.0, 1e-30, 1e-24, 1e-19, 1e-12, 1e-3, 1.0, 1e15], np.float64)
    for t in range(1, 7):
        g = (rng.standard_normal(n) * rng.choice(scales, n)).astype(np.float32)
        g[t * 2048:(t * 2048 + 256)] = 0.0                      # whole rows of zeros
        if t % 2 == 0:
            g[:4096] = (rng.standard_normal(4096) * 1e-22).astype(np.float32)   # a block of tiny values only
        q8.adam8bit_step(w, dev(g), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        H.oracle_adam8(w_ref, g, st, B, t=t)
        H.assert_state_equal("step %d" % t, d, st, w, w_ref)


def test_zero_gradient_keeps_zero_state(q8, tabs):
    n, B = 5000, 2048
    w0 = synth.uniform_weights(9, 0, n)
    w = dev(w0); g = torch.zeros(n, device="cuda")
    st = {k: dev(v) for k, v in H.zero_state(n, B).items()}
    q8.adam8bit_step(w, g, st["m_q"], st["r_q"], st["N_m"], st["N_r"], tabs[0], tabs[1], B, **H.ADAM)
    assert torch.all(st["m_q"] == 127) and torch.all(st["r_q"] == 0)
    assert torch.all(st["N_m"] == 0) and torch.all(st["N_r"] == 0)
    assert np.array_equal(w.cpu().numpy(), w0)


def test_n_zero_and_errors_on_device(q8, tabs):
    e = torch.empty(0, device="cuda"); eb = torch.empty(0, dtype=torch.uint8, device="cuda")
    q8.adam8bit_step(e, e, eb, eb, e, e, tabs[0], tabs[1], 2048, **H.ADAM)
    q8.sgd8bit_step(e, e, eb, e, tabs[0], 2048, **H.SGD)
    w = torch.zeros(64, device="cuda")
    with pytest.raises(q8.Q8Error) as err:
        q8.sgd8bit_step(w, w, torch.zeros(64, dtype=torch.uint8, device="cuda"), torch.zeros(1, device="cuda"),
                        tabs[0], 100, **H.SGD)
    assert err.value.status == q8.EBLOCK
    with pytest.raises(q8.Q8Error) as err:
        q8.sgd8bit_step(w[1:], w[1:], torch.zeros(63, dtype=torch.uint8, device="cuda"),
                        torch.zeros(1, device="cuda"), tabs[0], 64, **H.SGD)
    assert err.value.status == q8.EALIGN


def test_runs_on_the_callers_stream(q8, tabs):
    n, B = 1 << 18, 2048
    w_ref = synth.uniform_weights(11, 0, n); g = synth.normal_grad(11, 0, 1, n, 1e-3)
    st = H.zero_state(n, B)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        w = dev(w_ref); gd = dev(g); d = {k: dev(v) for k, v in st.items()}
        q8.adam8bit_step(w, gd, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM)
    s.synchronize()
    H.oracle_adam8(w_ref, g, st, B)
    H.assert_state_equal("side stream", d, st, w, w_ref)


def test_concurrent_launches_on_two_streams(q8, tabs):
    """Launches that overlap on different streams use different scheduler slots: two
    independent tensors stepped concurrently for several steps still match the oracle, and
    a later launch finds every slot left clean."""
    n, B = (1 << 21) + 777, 2048
    hosts, devs = [], []
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for k in range(2):
        w_ref = synth.uniform_weights(500 + k, 0, n)
        st = H.zero_state(n, B)
        with torch.cuda.stream(streams[k]):
            devs.append((dev(w_ref), {kk: dev(v) for kk, v in st.items()}))
        hosts.append((w_ref, st))
    for t in range(1, 6):
        gs = [synth.normal_grad(500 + k, 0, t, n, 1e-3) for k in range(2)]
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                w, d = devs[k]
                q8.adam8bit_step(w, dev(gs[k]), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B,
                                 **H.ADAM, t=t)
        for k in range(2):
            H.oracle_adam8(hosts[k][0], gs[k], hosts[k][1], B, t=t)
    torch.cuda.synchronize()
    for k in range(2):
        H.assert_state_equal("stream %d" % k, devs[k][1], hosts[k][1], devs[k][0], hosts[k][0])
    # more launches than there are scheduler slots, back to back on one stream
    w, d = devs[0]
    w_ref, st = hosts[0]
    g = synth.normal_grad(502, 0, 1, n, 1e-3); gd = dev(g)
    for t in range(6, 6 + 70):
        q8.adam8bit_step(w, gd, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        H.oracle_adam8(w_ref, g, st, B, t=t)
    H.assert_state_equal("after 70 more launches", d, st, w, w_ref)


def test_repeated_runs_are_bitwise_deterministic(q8, tabs):
    n, B = 3_000_001, 256
    w0 = synth.uniform_weights(600, 0, n); g = synth.normal_grad(600, 0, 1, n, 1e-3)
    outs = []
    for _ in range(2):
        w = dev(w0); gd = dev(g)
        d = {k: dev(v) for k, v in H.zero_state(n, B).items()}
        for t in range(1, 4):
            q8.adam8bit_step(w, gd, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        outs.append([w.cpu().numpy()] + [d[k].cpu().numpy() for k in sorted(d)])
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


def test_step_inside_a_captured_graph(q8, tabs):
    """The step enqueues one kernel and nothing else (the scheduler counter resets itself,
    no memset), so it can be captured into a HIP graph.  Each replay, with eager work and
    synchronizations in between, is checked against the oracle."""
    n, B = 300_000, 2048
    w_ref = synth.uniform_weights(700, 0, n)
    st = H.zero_state(n, B)
    w = dev(w_ref); d = {k: dev(v) for k, v in st.items()}
    g_dev = torch.zeros(n, device="cuda")
    g0 = synth.normal_grad(700, 0, 0, n, 1e-3)
    g_dev.copy_(dev(g0))
    # eager warm-up on a side stream (fills the library's per-kernel caches), as torch requires
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        q8.adam8bit_step(w, g_dev, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM)
    torch.cuda.current_stream().wait_stream(s)
    H.oracle_adam8(w_ref, g0, st, B)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        q8.adam8bit_step(w, g_dev, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM)
    for t in range(1, 6):
        g = synth.normal_grad(700, 0, t, n, 1e-3)
        g_dev.copy_(dev(g))                       # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        H.oracle_adam8(w_ref, g, st, B)
        H.assert_state_equal("replay %d" % t, d, st, w, w_ref)


def test_checkpoint_resume_and_fp32_state_import(q8, tabs):
    """The optimizer state is exactly {codes, absmax} in caller-owned buffers: a snapshot
    restored into fresh buffers continues bit-identically.  An fp32 state (e.g. from a 32-bit
    checkpoint) is imported with q8_quantize_blockwise and then stepped in 8 bits, matching
    the oracle doing the same; exporting with q8_dequantize_blockwise matches too."""
    n, B = 50_000, 2048
    qs, qu = H.codebooks()
    w0 = synth.uniform_weights(800, 0, n)
    grads = [synth.normal_grad(800, 0, t, n, 1e-3) for t in range(1, 6)]
    w = dev(w0); d = {k: dev(v) for k, v in H.zero_state(n, B).items()}
    for t in range(1, 4):
        q8.adam8bit_step(w, dev(grads[t - 1]), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
    snap_w = w.cpu().numpy().copy(); snap = {k: v.cpu().numpy().copy() for k, v in d.items()}
    for t in range(4, 6):
        q8.adam8bit_step(w, dev(grads[t - 1]), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
    w2 = dev(snap_w); d2 = {k: dev(v) for k, v in snap.items()}
    for t in range(4, 6):
        q8.adam8bit_step(w2, dev(grads[t - 1]), d2["m_q"], d2["r_q"], d2["N_m"], d2["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w2.cpu().numpy().view(np.uint32))
    for k in d:
        assert np.array_equal(d[k].cpu().numpy().view(np.uint8), d2[k].cpu().numpy().view(np.uint8)), k
    # import of a 32-bit state
    wr = w0.copy(); m32 = np.zeros(n, np.float32); r32 = np.zeros(n, np.float32)
    for t in range(1, 4):
        oracle.adam32_step(wr, grads[t - 1], m32, r32, **H.ADAM, t=t)
    nb = oracle.nblocks(n, B)
    mq = torch.empty(n, dtype=torch.uint8, device="cuda"); rq = torch.empty(n, dtype=torch.uint8, device="cuda")
    Nm = torch.empty(nb, device="cuda"); Nr = torch.empty(nb, device="cuda")
    q8.quantize_blockwise(tabs[0], dev(m32), B, mq, Nm)
    q8.quantize_blockwise(tabs[1], dev(r32), B, rq, Nr)
    st = dict(zip(("m_q", "N_m"), oracle.quantize_blockwise(qs, m32, B)))
    st.update(zip(("r_q", "N_r"), oracle.quantize_blockwise(qu, r32, B)))
    wd_ = dev(wr); dd = dict(m_q=mq, r_q=rq, N_m=Nm, N_r=Nr)
    H.assert_state_equal("import", dd, st, wd_, wr)
    for t in range(4, 6):
        q8.adam8bit_step(wd_, dev(grads[t - 1]), mq, rq, Nm, Nr, tabs[0], tabs[1], B, **H.ADAM, t=t)
        H.oracle_adam8(wr, grads[t - 1], st, B, t=t)
        H.assert_state_equal("after import, step %d" % t, dd, st, wd_, wr)
    out = torch.empty(n, device="cuda")
    q8.dequantize_blockwise(tabs[0], mq, Nm, B, out)
    assert np.array_equal(out.cpu().numpy().view(np.uint32),
                          oracle.dequantize_blockwise(qs, st["m_q"], st["N_m"], B).view(np.uint32))


@pytest.mark.parametrize("eps", [1e-8, 0.0, 2048.0], ids=["eps1e-8", "eps0", "eps2048"])
def test_adam_gradient_scale_sweep_bitwise(q8, tabs, eps):
    """Gradient magnitudes from the denormal range to 1e18, one decade per case, so that the rows
    cross both ends of the range in which the weight update uses its short square root and
    division (and eps = 2048 switches those off on the host): weights compared bit for bit."""
    n, B = 256 * 5 + 77, 256
    hp = dict(H.ADAM, eps=eps)
    decades = range(-15, 19) if eps == 0.0 else range(-44, 19)
    for k in decades:
        rng = np.random.default_rng(1000 + k)
        w_ref = synth.uniform_weights(500 + k, 0, n)
        st = H.zero_state(n, B)
        w = dev(w_ref); d = {key: dev(v) for key, v in st.items()}
        for t in range(1, 4):
            g = (rng.standard_normal(n) * 10.0 ** k).astype(np.float32)
            if eps == 0.0:
                g[g == 0] = np.float32(10.0 ** k)          # 0/0 is outside the method
            if t == 2:
                g[300:340] *= np.float32(1e-6)             # a few rows mix magnitudes
            q8.adam8bit_step(w, dev(g), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **hp, t=t)
            H.oracle_adam8(w_ref, g, st, B, t=t, hp=hp)
            H.assert_state_equal("decade %d step %d" % (k, t), d, st, w, w_ref)
            got = w.cpu().numpy()
            same = (got.view(np.uint32) == w_ref.view(np.uint32)) | ((got == 0) & (w_ref == 0))
            assert same.all(), "decade %d step %d: %d weights differ in their bits" % (k, t, int((~same).sum()))


@pytest.mark.parametrize("eps", [1e-8, 3e-3, 1.0, 700.0])
def test_weight_update_quotient_bits(q8, tabs, eps):
    """beta1 = beta2 = 0, alpha = 1, w = 0 turn the step into w = -(g / (sqrt(g*g) + eps)): four
    million random numerators and denominators per eps, spread over the whole magnitude range
    of the short division and square root, must give the oracle's (IEEE) bits."""
    n, B = 1 << 22, 2048
    rng = np.random.default_rng(int(eps * 1000) + 5)
    mant = rng.integers(0, 1 << 23, n, dtype=np.uint64).astype(np.uint32)
    expo = rng.integers(127 - 39, 127 + 19, n, dtype=np.uint64).astype(np.uint32)
    sign = rng.integers(0, 2, n, dtype=np.uint64).astype(np.uint32)
    g = ((sign << 31) | (expo << 23) | mant).view(np.float32)
    hp = dict(alpha=1.0, beta1=0.0, beta2=0.0, eps=eps)
    w_ref = np.zeros(n, np.float32)
    st = H.zero_state(n, B)
    w = dev(w_ref); d = {k: dev(v) for k, v in st.items()}
    q8.adam8bit_step(w, dev(g), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **hp)
    H.oracle_adam8(w_ref, g, st, B, hp=hp)
    got = w.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), w_ref.view(np.uint32)), int((got.view(np.uint32) != w_ref.view(np.uint32)).sum())
    H.assert_state_equal("states", d, st, w, w_ref)


def test_weight_update_division_by_all_ones_mantissas(q8, tabs):
    """The one divisor mantissa for which a reciprocal refined from a seed one ulp low does not
    end correctly rounded is all ones (then a power-of-two numerator rounds the wrong way if the
    seed was the power of two below the true reciprocal).  beta1 = 0, beta2 = 2^-23, eps = 0,
    alpha = 1, w = 0 and g = +-2^k turn the step into w = -(g / d) with d = sqrt((1 - 2^-23) g^2)
    = (2 - 2^-23) 2^(k-1), an all-ones mantissa, for every exponent of the guarded range: the
    quotient must come out as the IEEE one, -+(1 + 2^-23), so the hardware's reciprocal is the
    safe one for these divisors."""
    B = 2048
    ks = np.arange(-39, 20)
    g = np.repeat(np.ldexp(np.float32(1), ks).astype(np.float32), B)
    g[1::2] *= -1
    n = g.size
    hp = dict(alpha=1.0, beta1=0.0, beta2=float(np.float32(2.0 ** -23)), eps=0.0)
    w_ref = np.zeros(n, np.float32)
    st = H.zero_state(n, B)
    w = dev(w_ref); d = {k: dev(v) for k, v in st.items()}
    q8.adam8bit_step(w, dev(g), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **hp)
    H.oracle_adam8(w_ref, g, st, B, hp=hp)
    want = np.where(g > 0, -1.0, 1.0).astype(np.float32) * np.float32(1 + 2.0 ** -23)
    assert np.array_equal(w_ref.view(np.uint32), want.view(np.uint32))          # the construction is what it claims
    got = w.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), w_ref.view(np.uint32)), np.flatnonzero(got != w_ref)[:8]
    H.assert_state_equal("states", d, st, w, w_ref)


SQRT_BINADES = os.environ.get("Q8_SQRT_BINADES", "-80,-1,0,39")      # "all" = every binade of the guarded range


@pytest.mark.parametrize("eps,flags,t", [(0.0, 0, 1), (1e-8, 1, 3)], ids=["plain", "bias-corrected"])
def test_weight_update_root_over_whole_binades(q8, tabs, eps, flags, t):
    """The square root of the weight update on EVERY binary32 r of whole binades, end to end on
    the device: beta1 = beta2 = 1 and g = 0 leave the states where they are, codes of 1.0 and a
    block maximum N_r[b] = r make the dequantized second state any value wanted; with B = 64 one
    launch covers a binade (2^23 blocks), each block pairing its r with 64 different first
    states (64 codes of the signed map), eps = 0, alpha = 1, w = 0: w becomes -(m / sqrt(r)),
    64 quotients per root, all compared with the oracle's IEEE results bit for bit.  The second
    case adds eps = 1e-8 and the bias-correction factors of step 3 (root scaled before eps is added).
    Q8_SQRT_BINADES=all runs all 120 binades of [2^-80, 2^40] (10^9 roots, 6 * 10^10 quotients)."""
    B = 64
    binades = range(-80, 40) if SQRT_BINADES == "all" else [int(x) for x in SQRT_BINADES.split(",")]
    nb = 1 << 23
    n = nb * B
    hp = dict(alpha=1.0, beta1=1.0, beta2=1.0, eps=eps)
    if flags:
        hp.update(beta1=0.9, beta2=0.999)      # bias correction needs beta < 1; g = 0 then shrinks the states by beta
    codes = np.concatenate([np.arange(0, 127, 4), np.arange(129, 256, 4)]).astype(np.uint8)     # 64 codes, none of them 0.0
    assert codes.size == B
    m_q0 = np.tile(codes, nb)
    g_d = torch.zeros(n, device="cuda")
    for e in binades:
        r_vals = (np.uint32((e + 127) << 23) + np.arange(nb, dtype=np.uint32)).view(np.float32)
        # first states around sqrt(r), so that the quotients stay well inside the binary32 range
        N_m0 = np.ldexp(np.float32(1), np.full(nb, e // 2)).astype(np.float32)
        st = dict(m_q=m_q0.copy(), r_q=np.full(n, 255, np.uint8), N_m=N_m0.copy(), N_r=r_vals.copy())
        w_ref = np.zeros(n, np.float32)
        w = torch.zeros(n, device="cuda"); d = {k: dev(v) for k, v in st.items()}
        q8.adam8bit_step(w, g_d, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, t=t, flags=flags, **hp)
        H.oracle_adam8(w_ref, np.zeros(n, np.float32), st, B, t=t, flags=flags, hp=hp)
        ref = torch.from_numpy(w_ref).cuda()
        bad = int((w.view(torch.int32) != ref.view(torch.int32)).sum())
        assert bad == 0, "binade 2^%d: %d of %d quotients differ" % (e, bad, n)
        print("binade 2^%d done" % e, flush=True)                 # progress for the long run (pytest -s)
        for k in ("m_q", "r_q", "N_m", "N_r"):
            assert torch.equal(d[k].view(torch.uint8), torch.from_numpy(st[k]).cuda().view(torch.uint8)), (e, k)
        del w, d, ref
    H.report("square root and division of the weight update (eps=%g, flags=%d) on every r of %d whole binades "
             "(%d roots, 64 quotients each): identical to the oracle's" % (eps, flags, len(binades), len(binades) * nb))


HARD_DIVISORS = os.environ.get("Q8_HARD_DIVISORS", "262144")       # "all" = every divisor mantissa (2^23)


def test_weight_update_division_on_every_hard_pair_of_many_divisors(q8, tabs, tmp_path):
    """The hard operands of the weight update's division, through the kernel: for a range of
    divisor mantissas n (2^18 of them in the suite, Q8_HARD_DIVISORS=all: all 2^23) every numerator
    m whose quotient lies within 16 * 2^-48 of a rounding midpoint (the set the host check
    enumerates, tests/exact_check.cpp).  One block of 64 per pair: codes of 1.0 with N_m = m 2^a
    and N_r = RN((n 2^b)^2) make the first state the numerator and the root of the second the
    divisor exactly; beta1 = beta2 = 1, g = 0, eps = 0, alpha = 1, w = 0 give w = -(m / d).  The
    hardware's reciprocal, one Newton step and one residual correction must return the IEEE
    quotient on every one of them."""
    import ctypes as C
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no host compiler for the pair enumeration")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib = str(tmp_path / "libexact_check.so")
    subprocess.check_call(["g++", "-O2", "-std=c++20", "-ffp-contract=off", "-fno-fast-math", "-mfma", "-shared", "-fPIC",
                           "-I" + os.path.join(root, "paper_2412_01195_amd", "csrc"),
                           os.path.join(root, "tests", "exact_check.cpp"), "-o", lib])
    L = C.CDLL(lib)
    L.list_near_midpoint_pairs.argtypes = [C.c_uint32, C.c_uint32, C.c_int, C.c_void_p, C.c_void_p, C.c_int64]
    L.list_near_midpoint_pairs.restype = C.c_int64
    ndiv = (1 << 23) if HARD_DIVISORS == "all" else int(HARD_DIVISORS)
    B, per_launch = 64, 1 << 24
    hp = dict(alpha=1.0, beta1=1.0, beta2=1.0, eps=0.0)
    rng = np.random.default_rng(99)
    n0 = (1 << 23) + (int(rng.integers(0, (1 << 23) - ndiv + 1)) if ndiv < (1 << 23) else 0)
    total = 0
    step = 1 << 16                                                 # divisors per enumeration call
    pend_m, pend_n = [], []

    def run(mi, ni):
        nonlocal total
        k = mi.size
        e_d = rng.integers(-40, 20, k)                             # d = n 2^(e_d - 23) in [2^-40, 2^20]
        e_m = np.clip(e_d + rng.integers(-30, 30, k), -80, 38)
        m = np.ldexp(mi.astype(np.float64), e_m - 23)              # positive: rounding to nearest is symmetric
        d = np.ldexp(ni.astype(np.float64), e_d - 23)
        st = dict(m_q=np.full(k * B, 255, np.uint8), r_q=np.full(k * B, 255, np.uint8),
                  N_m=m.astype(np.float32), N_r=(d * d).astype(np.float32))     # sqrt(RN(d^2)) = d
        w_ref = np.zeros(k * B, np.float32)
        w = torch.zeros(k * B, device="cuda"); dd = {kk: dev(v) for kk, v in st.items()}
        g0 = torch.zeros(k * B, device="cuda")
        q8.adam8bit_step(w, g0, dd["m_q"], dd["r_q"], dd["N_m"], dd["N_r"], tabs[0], tabs[1], B, **hp)
        want = -(m.astype(np.float32) / d.astype(np.float32))                  # IEEE quotient of the two binary32 operands
        got = w.view(k, B)
        ref = torch.from_numpy(want).cuda()
        bad = int((got.view(torch.int32) != ref.view(torch.int32)[:, None]).sum())
        assert bad == 0, "%d of %d quotients differ" % (bad, k * B)
        H.oracle_adam8(w_ref, np.zeros(k * B, np.float32), st, B, hp=hp)       # and the oracle agrees with that
        assert np.array_equal(w_ref.reshape(k, B)[:, 0].view(np.uint32), want.view(np.uint32))
        total += k
        print("%d pairs done" % total, flush=True)

    for lo in range(n0, n0 + ndiv, step):
        hi = min(n0 + ndiv, lo + step)
        cap = (hi - lo) * 40
        bm = np.empty(cap, np.uint32); bn = np.empty(cap, np.uint32)
        cnt = L.list_near_midpoint_pairs(lo, hi, 16, bm.ctypes.data, bn.ctypes.data, cap)
        assert 0 < cnt < cap
        pend_m.append(bm[:cnt]); pend_n.append(bn[:cnt])
        if sum(x.size for x in pend_m) >= per_launch:
            run(np.concatenate(pend_m), np.concatenate(pend_n)); pend_m, pend_n = [], []
    if pend_m:
        run(np.concatenate(pend_m), np.concatenate(pend_n))
    H.report("weight-update division on every near-midpoint numerator of %d divisor mantissas (%d pairs): identical to "
             "the IEEE quotient" % (ndiv, total))


def _quantize_threaded(q, T, B):
    """oracle.quantize_blockwise over disjoint block ranges on the host threads."""
    n = T.size
    nb = oracle.nblocks(n, B)
    TQ = np.empty(n, np.uint8); N = np.empty(nb, np.float32)
    nthr = H.host_threads()
    per = -(-nb // nthr)

    def run(k):
        b0, b1 = k * per, min(nb, (k + 1) * per)
        if b0 < b1:
            e = slice(b0 * B, min(n, b1 * B))
            TQ[e], N[b0:b1] = oracle.quantize_blockwise(q, T[e], B)
    list(H.pool().map(run, range(nthr)))
    return TQ, N


@pytest.mark.parametrize("nbits", [0x3F800000, 0x2B7FFFFF, 0x4E2C9A35], ids=["N=1", "N=all-ones*2^-41", "N=7.2e8"])
def test_quantize_every_value_under_a_block_maximum(q8, tabs, nbits):
    """Normalisation by the block maximum and nearest-code search on EVERY binary32 value a block
    with maximum N can hold: each block starts with N itself and continues with 2047 consecutive
    bit patterns; the signed map sees all values of [-N, N] (2 * (bits(N) + 1), about 2 * 10^9),
    the unsigned map all of [0, N].  Codes and block maxima against the oracle, bit for bit."""
    B = 2048
    N = np.array([nbits], np.uint32).view(np.float32)[0]
    count = int(nbits) + 1                                        # non-negative values <= N
    per = B - 1
    nblk = -(-count // per)
    chunk_blocks = 1 << 17                                        # 2.7e8 elements per piece
    for signed, tab, q in ((True, tabs[0], H.codebooks()[0]), (False, tabs[1], H.codebooks()[1])):
        for sign in ((0, 1) if signed else (0,)):
            for b0 in range(0, nblk, chunk_blocks):
                b1 = min(nblk, b0 + chunk_blocks)
                pat = np.arange(b0 * per, b1 * per, dtype=np.int64)
                pat = np.minimum(pat, count - 1).astype(np.uint32)           # the tail repeats N
                T = np.empty((b1 - b0, B), np.uint32)
                T[:, 0] = nbits
                T[:, 1:] = pat.reshape(b1 - b0, per)
                T = T.reshape(-1)
                if sign:
                    T[np.arange(T.size) % B != 0] |= np.uint32(0x80000000)   # the maximum itself stays +N
                T = T.view(np.float32)
                TQ_ref, N_ref = _quantize_threaded(q, T, B)
                TQ = torch.empty(T.size, dtype=torch.uint8, device="cuda"); Nd = torch.empty(b1 - b0, device="cuda")
                q8.quantize_blockwise(tab, dev(T), B, TQ, Nd)
                assert torch.equal(Nd.view(torch.int32), torch.from_numpy(N_ref).cuda().view(torch.int32))
                bad = int((TQ != torch.from_numpy(TQ_ref).cuda()).sum())
                assert bad == 0, "%s map, sign %d, blocks [%d, %d): %d codes differ" % (
                    "signed" if signed else "unsigned", sign, b0, b1, bad)
    H.report("quantize: every binary32 value under the block maximum %.9g (%d patterns per sign), both maps: "
             "codes identical to the oracle's" % (float(N), count))


def test_host_threads_launch_concurrently(q8, tabs):
    """Four host threads, each with its own stream and tensor, call the library at the same time
    (ctypes releases the GIL during the call): the per-device records and occupancy caches are
    shared, the results must not be."""
    import threading
    n, B, steps, nthr = (1 << 18) + 333, 1024, 25, 4
    hosts, devs, grads = [], [], []
    for k in range(nthr):
        w_ref = synth.uniform_weights(900 + k, 0, n)
        st = H.zero_state(n, B)
        hosts.append((w_ref, st))
        devs.append((dev(w_ref), {kk: dev(v) for kk, v in st.items()}))
        grads.append([dev(synth.normal_grad(900 + k, 0, t, n, 1e-3)) for t in range(1, 4)])
    torch.cuda.synchronize()
    errors = []

    def worker(k):
        try:
            s = torch.cuda.Stream()
            w, d = devs[k]
            with torch.cuda.stream(s):
                for t in range(1, steps + 1):
                    q8.adam8bit_step(w, grads[k][t % 3], d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B,
                                     **H.ADAM, t=t)
            s.synchronize()
        except Exception as e:                      # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(nthr)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for k in range(nthr):
        w_ref, st = hosts[k]
        for t in range(1, steps + 1):
            H.oracle_adam8(w_ref, grads[k][t % 3].cpu().numpy(), st, B, t=t)
        H.assert_state_equal("thread %d" % k, devs[k][1], st, devs[k][0], w_ref)


def test_traffic_probe_leaves_everything_unchanged(q8, tabs):
    """The benchmark's measurement aid (a library of its own, not the product's) rewrites w and
    both code arrays with the values it read."""
    import bench
    probe = bench.load_traffic_probe()
    n = 2048 * 9 + 777
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal(n).astype(np.float32); g0 = rng.standard_normal(n).astype(np.float32)
    m0 = rng.integers(0, 256, n, dtype=np.uint8); r0 = rng.integers(0, 256, n, dtype=np.uint8)
    w, g, m, r = dev(w0), dev(g0), dev(m0), dev(r0)
    probe(w, g, m, r, tabs[0], tabs[1])
    probe(w, g, m, r, tabs[0], tabs[1])
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w0.view(np.uint32)) and np.array_equal(g.cpu().numpy(), g0)
    assert np.array_equal(m.cpu().numpy(), m0) and np.array_equal(r.cpu().numpy(), r0)


@pytest.mark.parametrize("B", [256, 2048])
def test_nonfinite_gradients_stay_inside_their_blocks(q8, tabs, B):
    """Results for NaN / Inf inputs are unspecified, but the call completes, nothing is read or
    written out of bounds (every table key is clamped into the LDS map), and -- blocks being
    independent -- every block without such an input still matches the oracle bit for bit."""
    n = 20 * B + 77
    w_ref = synth.uniform_weights(1300, 0, n)
    st = H.zero_state(n, B)
    w = dev(w_ref); d = {k: dev(v) for k, v in st.items()}
    bad_blocks = [1, 7, 12]
    for t in range(1, 4):
        g = synth.normal_grad(1300, 0, t, n, 1e-3)
        g[1 * B + 5] = np.nan
        g[7 * B] = np.inf
        g[12 * B + B - 1] = -np.inf
        g[12 * B + 3] = np.nan
        q8.adam8bit_step(w, dev(g), d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        torch.cuda.synchronize()
        with np.errstate(all="ignore"):
            H.oracle_adam8(w_ref, g, st, B, t=t, split=False)
        keep = np.ones(n, bool)
        for b in bad_blocks:
            keep[b * B:(b + 1) * B] = False
        bkeep = np.ones(oracle.nblocks(n, B), bool)
        bkeep[bad_blocks] = False
        for k in ("m_q", "r_q"):
            assert np.array_equal(d[k].cpu().numpy()[keep], st[k][keep]), (t, k)
        for k in ("N_m", "N_r"):
            assert np.array_equal(d[k].cpu().numpy().view(np.uint32)[bkeep], st[k].view(np.uint32)[bkeep]), (t, k)
        assert np.array_equal(w.cpu().numpy().view(np.uint32)[keep], w_ref.view(np.uint32)[keep])
        # keep the two trajectories together where the results are unspecified
        for k in d:
            d[k].copy_(dev(st[k]))
        w.copy_(dev(w_ref))
