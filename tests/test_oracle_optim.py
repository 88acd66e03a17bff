"""Pins of the oracle's update rules (Eq. sgd, Eq. adam) and of the 8-bit composition
(Sec. I and Sec. IV-B: states 8-bit -> 32-bit, weight update, re-quantization).
Closed forms and an independently written numpy recurrence stand against the C code."""
import numpy as np
import pytest

import oracle

QS = oracle.build_codebook(True)
QU = oracle.build_codebook(False)
f32 = np.float32
ADAM = dict(alpha=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)


def np_adam(w, g, m, r, alpha, beta1, beta2, eps, wd=0.0):
    """Eq. adam, one binary32 operation per numpy call (numpy never fuses)."""
    a, b1, b2, e = f32(alpha), f32(beta1), f32(beta2), f32(eps)
    if wd:
        g = g + f32(wd) * w
    m = b1 * m + (f32(1) - b1) * g
    r = b2 * r + ((f32(1) - b2) * g) * g
    w = w - a * (m / (np.sqrt(r) + e))
    return w, m, r


def np_sgd(w, g, m, alpha, beta, wd=0.0):
    if wd:
        g = g + f32(wd) * w
    m = f32(beta) * m + g
    return w - f32(alpha) * m, m


def test_adam32_equals_numpy_recurrence_bitwise():
    rng = np.random.default_rng(0)
    n = 5000
    w = rng.uniform(-0.1, 0.1, n).astype(f32); m = np.zeros(n, f32); r = np.zeros(n, f32)
    w2, m2, r2 = w.copy(), m.copy(), r.copy()
    for t in range(1, 8):
        g = (rng.standard_normal(n) * 1e-3).astype(f32)
        oracle.adam32_step(w, g, m, r, **ADAM, t=t)
        w2, m2, r2 = np_adam(w2, g, m2, r2, **ADAM)
        assert np.array_equal(w, w2) and np.array_equal(m, m2) and np.array_equal(r, r2)
        assert w2.dtype == f32 and m2.dtype == f32 and r2.dtype == f32


def test_adam32_with_coupled_decay_equals_numpy():
    rng = np.random.default_rng(1)
    n = 1000
    w = rng.uniform(-0.1, 0.1, n).astype(f32); m = np.zeros(n, f32); r = np.zeros(n, f32)
    w2, m2, r2 = w.copy(), m.copy(), r.copy()
    for t in range(1, 4):
        g = (rng.standard_normal(n) * 1e-3).astype(f32)
        oracle.adam32_step(w, g, m, r, **ADAM, wd=1e-2, t=t)
        w2, m2, r2 = np_adam(w2, g, m2, r2, **ADAM, wd=1e-2)
        assert np.array_equal(w, w2) and np.array_equal(m, m2) and np.array_equal(r, r2)


def test_adam_first_step_closed_form():
    g = np.array([1e-3, -2e-3, 0.5, 0.0, -7.0], f32)
    w0 = np.array([0.1, -0.1, 0.0, 0.3, 1.0], f32)
    w = w0.copy(); m = np.zeros(5, f32); r = np.zeros(5, f32)
    oracle.adam32_step(w, g, m, r, **ADAM)
    g64 = g.astype(np.float64)
    omb1 = float(f32(1) - f32(0.9)); omb2 = float(f32(1) - f32(0.999))   # binary32 subtraction
    m_ref, r_ref = omb1 * g64, omb2 * g64 * g64
    w_ref = w0 - 1e-3 * m_ref / (np.sqrt(r_ref) + 1e-8)
    assert np.allclose(m, m_ref, rtol=3e-7, atol=0) and np.allclose(r, r_ref, rtol=1e-5, atol=0)
    assert np.allclose(w, w_ref, rtol=0, atol=2e-7)
    # the first step moves every weight with g != 0 by about alpha*0.1/sqrt(0.001) against sign(g)
    step = (w0 - w)[g != 0] * np.sign(g[g != 0])
    assert np.allclose(step, 1e-3 * 0.1 / np.sqrt(0.001), rtol=1e-3)
    assert w[3] == w0[3] and m[3] == 0 and r[3] == 0


def test_adam_constant_gradient_closed_form():
    g = np.array([3e-3, -1e-2, 4.0], f32); n = 3
    w = np.zeros(n, f32); m = np.zeros(n, f32); r = np.zeros(n, f32)
    for t in range(1, 41):
        oracle.adam32_step(w, g, m, r, **ADAM, t=t)
        g64 = g.astype(np.float64)
        assert np.allclose(m, (1 - 0.9 ** t) * g64, rtol=2e-5)
        assert np.allclose(r, (1 - 0.999 ** t) * g64 * g64, rtol=2e-4)


def test_sgd32_equals_numpy_and_closed_form():
    rng = np.random.default_rng(2)
    n = 3000
    w = rng.uniform(-0.1, 0.1, n).astype(f32); m = np.zeros(n, f32)
    w2, m2 = w.copy(), m.copy()
    for t in range(6):
        g = (rng.standard_normal(n) * 1e-2).astype(f32)
        oracle.sgd32_step(w, g, m, 0.1, 0.9, 1e-4)
        w2, m2 = np_sgd(w2, g, m2, 0.1, 0.9, 1e-4)
        assert np.array_equal(w, w2) and np.array_equal(m, m2)
    # constant gradient, no decay: m_t = g (1 - beta^t) / (1 - beta), w_t = w_0 - alpha sum m
    g = np.array([1e-2, -3.0], f32); w = np.zeros(2, f32); m = np.zeros(2, f32)
    acc = np.zeros(2)
    for t in range(1, 30):
        oracle.sgd32_step(w, g, m, 0.1, 0.9, 0.0)
        mt = g.astype(np.float64) * (1 - 0.9 ** t) / (1 - 0.9)
        acc += mt
        assert np.allclose(m, mt, rtol=1e-5)
        assert np.allclose(w, -0.1 * acc, rtol=1e-5)
    w = np.ones(4, f32); m = np.zeros(4, f32); g = np.array([1, -2, 3, 0], f32)
    oracle.sgd32_step(w, g, m, 0.5, 0.9, 0.0)
    assert np.array_equal(m, g) and np.array_equal(w, 1 - 0.5 * g)      # m_0 = g_0


# ------------------------------------------------------------------ extension flags
# Bias correction and decoupled decay are not printed in Eq. adam (the paper only names AdamW
# with weight decay 0.05 in its training settings), so their definition is this build's own:
#   alpha_t = RN32( alpha / (1 - beta1^t) ),  c = RN32( 1 / sqrt(1 - beta2^t) )   [binary64 inside]
#   d = RN(RN(sqrt(r) * c) + eps);  w' = RN(w - RN(RN(alpha*wd) * w));  w = RN(w' - RN(alpha_t * RN(m/d)))
# The pins below hold the C code to that definition bit for bit.
def np_scalars(alpha, beta1, beta2, t):
    """alpha_t and c formed in binary64 from the binary32 hyper-parameters, rounded once."""
    a, b1, b2 = (np.float64(f32(x)) for x in (alpha, beta1, beta2))
    bc1 = np.float64(1.0) - b1 ** np.float64(t)
    bc2 = np.float64(1.0) - b2 ** np.float64(t)
    return f32(a / bc1), f32(np.float64(1.0) / np.sqrt(bc2))


def np_adam_ext(w, g, m, r, alpha, beta1, beta2, eps, wd, t, flags):
    """One step with the extension flags, one binary32 operation per numpy call."""
    a, b1, b2, e, lam = f32(alpha), f32(beta1), f32(beta2), f32(eps), f32(wd)
    bias, decoupled = bool(flags & oracle.FLAG_BIAS_CORRECTION), bool(flags & oracle.FLAG_DECOUPLED_WD)
    if wd and not decoupled:
        g = g + lam * w
    m = b1 * m + (f32(1) - b1) * g
    r = b2 * r + ((f32(1) - b2) * g) * g
    root = np.sqrt(r)
    if bias:
        a_t, c = np_scalars(alpha, beta1, beta2, t)
        step = a_t * (m / (root * c + e))
    else:
        step = a * (m / (root + e))
    if wd and decoupled:
        w = w - (a * lam) * w
    return w - step, m, r


@pytest.mark.parametrize("flags", [1, 2, 3])
@pytest.mark.parametrize("t0", [1, 997])
def test_extension_flags_equal_numpy_recurrence_bitwise(flags, t0):
    rng = np.random.default_rng(40 + flags)
    n = 6000
    w = rng.uniform(-0.1, 0.1, n).astype(f32); m = np.zeros(n, f32); r = np.zeros(n, f32)
    w2, m2, r2 = w.copy(), m.copy(), r.copy()
    for t in range(t0, t0 + 6):
        g = (rng.standard_normal(n) * 1e-3).astype(f32)
        oracle.adam32_step(w, g, m, r, **ADAM, wd=0.05, t=t, flags=flags)
        w2, m2, r2 = np_adam_ext(w2, g, m2, r2, **ADAM, wd=0.05, t=t, flags=flags)
        assert w2.dtype == f32
        assert np.array_equal(m, m2) and np.array_equal(r, r2)
        assert np.array_equal(w, w2), "flags %d step %d: %d weights differ" % (flags, t, (w != w2).sum())


def test_extension_pin_tells_the_plausible_variants_apart():
    """The inputs of the bit-for-bit pin above separate the definition from its nearest
    variants: a fused sqrt(r)*c + eps, step before decay, and binary32 scalars."""
    rng = np.random.default_rng(43)
    n = 6000
    w = rng.uniform(-0.1, 0.1, n).astype(f32)
    g = (rng.standard_normal(n) * 1e-3).astype(f32)
    m = (rng.standard_normal(n) * 1e-3).astype(f32); r = (rng.random(n) * 1e-6).astype(f32)
    t = 7
    ref, _, _ = np_adam_ext(w, g, m, r, **ADAM, wd=0.05, t=t, flags=3)
    a_t, c = np_scalars(ADAM["alpha"], ADAM["beta1"], ADAM["beta2"], t)
    _, m1, r1 = np_adam_ext(w, g, m, r, **ADAM, wd=0.0, t=t, flags=0)
    root = np.sqrt(r1)
    fused = (root.astype(np.float64) * np.float64(c) + np.float64(f32(1e-8))).astype(f32)    # exact product, one rounding
    w_fused = (w - (f32(1e-3) * f32(0.05)) * w) - a_t * (m1 / fused)
    assert (w_fused != ref).sum() > 10
    w_swapped = w - a_t * (m1 / (root * c + f32(1e-8)))
    w_swapped = w_swapped - (f32(1e-3) * f32(0.05)) * w          # decay applied after the step, to the old w
    assert (w_swapped != ref).sum() > 10
    differs = 0
    for tt in range(1, 40):
        a64, c64 = np_scalars(1e-3, 0.9, 0.999, tt)
        a32 = f32(1e-3) / (f32(1) - f32(0.9) ** f32(tt))
        c32 = f32(1) / np.sqrt(f32(1) - f32(0.999) ** f32(tt))
        differs += int(a32 != a64) + int(c32 != c64)
    assert differs > 10


def _fraction_of(x):
    from fractions import Fraction
    return Fraction(float(x))


@pytest.mark.parametrize("t", [1, 2, 3, 7, 10, 100, 997, 1000, 4321, 10 ** 6, 10 ** 9])
@pytest.mark.parametrize("betas", [(0.9, 0.999), (0.8, 0.99), (0.95, 0.9999)])
def test_bias_correction_scalars_are_correctly_rounded(t, betas):
    """alpha / (1 - beta1^t) and 1 / sqrt(1 - beta2^t) as real numbers, from the binary32
    hyper-parameters, rounded to nearest binary32: checked in exact rational arithmetic
    (the square root through the squares of the rounding interval's end points)."""
    from fractions import Fraction
    alpha = 1e-3
    b1, b2 = betas
    s = oracle.adam_scalars(alpha, b1, b2, 1e-8, wd=0.05, t=t, flags=oracle.FLAG_BIAS_CORRECTION)
    assert s["omb1"] == f32(1) - f32(b1) and s["omb2"] == f32(1) - f32(b2)
    assert s["alpha_wd"] == f32(alpha) * f32(0.05)

    def power_enclosure(beta):
        """[lo, hi] around beta^t: exact for moderate t; for huge t, 0 < beta^t <= exp(-t (1 - beta))
        (ln x <= x - 1), which the assertion keeps below 1e-40."""
        fb = _fraction_of(f32(beta))
        if t <= 5000:
            return fb ** t, fb ** t
        assert t * (1.0 - float(f32(beta))) > 93.0          # exp(-93) < 1e-40
        return Fraction(0), Fraction(1, 10 ** 40)
    lo1, hi1 = power_enclosure(b1)
    lo2, hi2 = power_enclosure(b2)

    def half_ulp_interval(x):
        x = f32(x)
        dn, up = np.nextafter(x, f32(-np.inf)), np.nextafter(x, f32(np.inf))
        return (_fraction_of(x) + _fraction_of(dn)) / 2, (_fraction_of(x) + _fraction_of(up)) / 2
    # alpha_t: the exact quotient lies in the rounding interval of the stored value
    lo, hi = half_ulp_interval(s["alpha_t"])
    q_lo = _fraction_of(f32(alpha)) / (1 - lo1)
    q_hi = _fraction_of(f32(alpha)) / (1 - hi1)
    assert lo <= q_lo and q_hi <= hi
    # isbc2: lo <= 1/sqrt(bc2) <= hi  <=>  lo^2 * bc2 <= 1 <= hi^2 * bc2
    lo, hi = half_ulp_interval(s["isbc2"])
    assert lo * lo * (1 - lo2) <= 1 and hi * hi * (1 - hi2) >= 1
    assert lo * lo * (1 - hi2) <= 1 and hi * hi * (1 - lo2) >= 1


def test_flags_zero_ignore_the_step_count():
    s0 = oracle.adam_scalars(1e-3, 0.9, 0.999, 1e-8, t=1)
    s9 = oracle.adam_scalars(1e-3, 0.9, 0.999, 1e-8, t=9)
    assert s0 == s9 and s0["alpha_t"] == f32(1e-3) and s0["isbc2"] == f32(1)


def test_bias_corrected_adamw_tracks_the_textbook_form():
    """Loose sanity check against the textbook statement in binary64: m/(1-b1^t), r/(1-b2^t),
    w <- w (1 - alpha wd) - alpha mhat / (sqrt(rhat) + eps)."""
    rng = np.random.default_rng(4)
    n = 2000
    w = rng.uniform(-0.1, 0.1, n).astype(f32); m = np.zeros(n, f32); r = np.zeros(n, f32)
    w64 = w.astype(np.float64); m64 = np.zeros(n); r64 = np.zeros(n)
    for t in range(1, 6):
        g = (rng.standard_normal(n) * 1e-3).astype(f32)
        oracle.adam32_step(w, g, m, r, **ADAM, wd=0.05, t=t,
                           flags=oracle.FLAG_BIAS_CORRECTION | oracle.FLAG_DECOUPLED_WD)
        m64 = 0.9 * m64 + (1 - f32(0.9).astype(np.float64)) * g
        r64 = f32(0.999).astype(np.float64) * r64 + (1 - f32(0.999).astype(np.float64)) * g.astype(np.float64) ** 2
        mhat = m64 / (1 - 0.9 ** t); rhat = r64 / (1 - 0.999 ** t)
        w64 = w64 * (1 - 1e-3 * 0.05) - 1e-3 * mhat / (np.sqrt(rhat) + 1e-8)
        assert np.allclose(w, w64, rtol=0, atol=5e-7 * t)


def _run8(n, B, steps, seed, adam=True):
    rng = np.random.default_rng(seed)
    w = rng.uniform(-0.1, 0.1, n).astype(f32)
    nb = oracle.nblocks(n, B)
    mq = np.full(n, 127, np.uint8); rq = np.zeros(n, np.uint8)
    Nm = np.zeros(nb, f32); Nr = np.zeros(nb, f32)
    # the same steps composed from separately pinned pieces
    w2 = w.copy(); mq2, rq2, Nm2, Nr2 = mq.copy(), rq.copy(), Nm.copy(), Nr.copy()
    for t in range(1, steps + 1):
        g = (rng.standard_normal(n) * 1e-3).astype(f32)
        if adam:
            oracle.adam8bit_step(w, g, mq, rq, Nm, Nr, QS, QU, B, **ADAM, t=t)
            m = oracle.dequantize_blockwise(QS, mq2, Nm2, B); r = oracle.dequantize_blockwise(QU, rq2, Nr2, B)
            oracle.adam32_step(w2, g, m, r, **ADAM, t=t)
            mq2, Nm2 = oracle.quantize_blockwise(QS, m, B); rq2, Nr2 = oracle.quantize_blockwise(QU, r, B)
            assert np.array_equal(rq, rq2) and np.array_equal(Nr, Nr2)
        else:
            oracle.sgd8bit_step(w, g, mq, Nm, QS, B, 0.1, 0.9, 1e-4)
            m = oracle.dequantize_blockwise(QS, mq2, Nm2, B)
            oracle.sgd32_step(w2, g, m, 0.1, 0.9, 1e-4)
            mq2, Nm2 = oracle.quantize_blockwise(QS, m, B)
        assert np.array_equal(w, w2) and np.array_equal(mq, mq2) and np.array_equal(Nm, Nm2)
    return w


@pytest.mark.parametrize("n,B", [(2048 * 2 + 512, 2048), (700, 256), (64, 64), (5, 2048)])
def test_8bit_steps_are_the_composition_of_pinned_pieces(n, B):
    _run8(n, B, 4, 21, adam=True)
    _run8(n, B, 4, 22, adam=False)


def test_8bit_first_sgd_step_stores_quantized_gradient():
    """Eq. sgd: m_0 = g_0.  From the zero state (zero codes, N = 0) the stored state
    after one step is exactly the quantization of g."""
    rng = np.random.default_rng(6)
    n, B = 1000, 256
    g = rng.standard_normal(n).astype(f32); w = np.zeros(n, f32)
    mq = np.full(n, 127, np.uint8); Nm = np.zeros(4, f32)
    oracle.sgd8bit_step(w, g, mq, Nm, QS, B, 0.1, 0.9, 0.0)
    TQ, N = oracle.quantize_blockwise(QS, g, B)
    assert np.array_equal(mq, TQ) and np.array_equal(Nm, N)
    assert np.array_equal(w, -(f32(0.1) * g))


def test_8bit_adam_tracks_32bit_adam():
    """The 8-bit trajectory stays close to the 32-bit one (the paper's claim that the
    update precision is kept): after 20 steps weights differ by a small multiple of alpha."""
    rng = np.random.default_rng(8)
    n, B = 4096, 2048
    w8 = rng.uniform(-0.1, 0.1, n).astype(f32); w32 = w8.copy()
    mq = np.full(n, 127, np.uint8); rq = np.zeros(n, np.uint8); Nm = np.zeros(2, f32); Nr = np.zeros(2, f32)
    m = np.zeros(n, f32); r = np.zeros(n, f32)
    for t in range(1, 21):
        g = (rng.standard_normal(n) * 1e-3).astype(f32)
        oracle.adam8bit_step(w8, g, mq, rq, Nm, Nr, QS, QU, B, **ADAM, t=t)
        oracle.adam32_step(w32, g, m, r, **ADAM, t=t)
    md = oracle.dequantize_blockwise(QS, mq, Nm, B)
    # per-step rounding error <= half a gap (0.9/128 of N), geometrically accumulated with beta1
    assert np.abs(md - m).max() <= Nm.max() * (0.9 / 128) / (1 - 0.9)
    assert np.abs(w8 - w32).mean() < 20 * 1e-3 * 0.5
