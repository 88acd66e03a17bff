"""Pins of the oracle's bfloat16-storage extension (not part of the paper: weights and
gradients held as bfloat16, arithmetic and 8-bit states unchanged).

The conversion is pinned to the definition of round-to-nearest-even by exact rational
arithmetic and to an independent library conversion (PyTorch's CPU cast); the step is
pinned to the fp32-storage oracle step through what the extension promises: widen exactly,
compute the same fp32 step, round the weight once."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests.harness import ADAM, SGD, codebooks, zero_state


def _f32(bits):
    return np.array([bits], np.uint32).view(np.float32)[0]


def test_widening_is_exact_for_every_pattern():
    h = np.arange(65536, dtype=np.uint32)
    want = (h << 16).astype(np.uint32).view(np.float32)
    got = np.array([oracle.bf16_to_f32(int(x)) for x in h], np.float32)
    finite = np.isfinite(want)
    assert np.array_equal(got[finite].view(np.uint32), want[finite].view(np.uint32))
    assert np.all(np.isnan(got[np.isnan(want)]))


def _nearest_even_bf16(x: float) -> int:
    """Definition written out: among finite bfloat16 values pick the one closest to x in exact
    arithmetic, ties to the even pattern; candidates are the truncation and its successor."""
    bits = int(np.array([x], np.float32).view(np.uint32)[0])
    lo = bits >> 16
    hi = lo + 1
    vx = Fraction(float(x))
    vlo = Fraction(float(_f32(lo << 16)))
    if (hi & 0x7fff) >= 0x7f80:                       # successor is infinity: compare with the would-be next value
        e = ((lo >> 7) & 0xff) - 127
        vhi = (Fraction(2) ** (e + 1)) * (1 if x >= 0 else -1)
    else:
        vhi = Fraction(float(_f32(hi << 16)))
    dlo, dhi = abs(vx - vlo), abs(vhi - vx)
    if dlo < dhi:
        return lo
    if dhi < dlo:
        return hi
    return lo if lo % 2 == 0 else hi


def test_rounding_matches_exact_definition():
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 1 << 32, 20000, dtype=np.uint64).astype(np.uint32)
    # add exact ties, near ties, denormals, the largest finite values
    hi = rng.integers(0, 1 << 16, 3000, dtype=np.uint64).astype(np.uint32)
    special = np.concatenate([(hi << 16) | 0x8000, (hi << 16) | 0x7fff, (hi << 16) | 0x8001,
                              np.array([0x7f7fffff, 0xff7fffff, 0x7f7f8000, 0x7f7f7fff, 0x00000001, 0x00008000,
                                        0x00018000, 0x80008000, 0, 0x80000000], np.uint32)])
    bits = np.concatenate([bits, special])
    x = bits.view(np.float32)
    ok = np.isfinite(x)
    for b, v in zip(bits[ok], x[ok]):
        assert oracle.f32_to_bf16(v) == _nearest_even_bf16(v), hex(int(b))


def test_rounding_matches_library_cast():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(12)
    bits = rng.integers(0, 1 << 32, 200000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x)]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(v) for v in x], np.uint16)
    assert np.array_equal(got, want)


def test_known_values():
    assert oracle.f32_to_bf16(1.0) == 0x3f80
    assert oracle.f32_to_bf16(-2.0) == 0xc000
    assert oracle.f32_to_bf16(1.0 + 2.0 ** -8) == 0x3f80          # tie, even below
    assert oracle.f32_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3f82      # tie, even above
    assert oracle.f32_to_bf16(np.float32(3.4e38)) == 0x7f80       # rounds past the largest finite value
    assert oracle.bf16_to_f32(0x3fc0) == 1.5


def _widen(h):
    return (h.astype(np.uint32) << 16).view(np.float32)


def _narrow(x):
    return np.array([oracle.f32_to_bf16(v) for v in x], np.uint16)


def _bf16_inputs(n, seed):
    rng = np.random.default_rng(seed)
    w = _narrow((rng.standard_normal(n) * 0.05).astype(np.float32))
    g = _narrow((rng.standard_normal(n) * 1e-3).astype(np.float32))
    return w, g


@pytest.mark.parametrize("B", [64, 2048])
def test_adam_step_is_fp32_step_on_widened_values(B):
    n = 3 * 2048 + 77
    qs, qu = codebooks()
    w, g = _bf16_inputs(n, 5)
    st_a, st_b = zero_state(n, B), zero_state(n, B)
    w32 = _widen(w)
    for t in range(1, 4):
        oracle.adam8bit_step_bf16(w, g, st_a["m_q"], st_a["r_q"], st_a["N_m"], st_a["N_r"], qs, qu, B,
                                  wd=0.01, t=t, **ADAM)
        oracle.adam8bit_step(w32, _widen(g), st_b["m_q"], st_b["r_q"], st_b["N_m"], st_b["N_r"], qs, qu, B,
                             wd=0.01, t=t, **ADAM)
        w32 = _widen(_narrow(w32))                     # the stored weight is rounded once per step
        assert np.array_equal(w, _narrow(w32))
        for k in st_a:
            assert np.array_equal(st_a[k].view(np.uint8), st_b[k].view(np.uint8)), (k, t)


def test_sgd_step_is_fp32_step_on_widened_values():
    n, B = 5000, 256
    qs, _ = codebooks()
    w, g = _bf16_inputs(n, 6)
    st_a, st_b = zero_state(n, B, adam=False), zero_state(n, B, adam=False)
    w32 = _widen(w)
    for _ in range(3):
        oracle.sgd8bit_step_bf16(w, g, st_a["m_q"], st_a["N_m"], qs, B, wd=1e-4, **SGD)
        oracle.sgd8bit_step(w32, _widen(g), st_b["m_q"], st_b["N_m"], qs, B, wd=1e-4, **SGD)
        w32 = _widen(_narrow(w32))
        assert np.array_equal(w, _narrow(w32))
        assert np.array_equal(st_a["m_q"], st_b["m_q"]) and np.array_equal(st_a["N_m"], st_b["N_m"])


def test_update_below_half_ulp_leaves_weight_unchanged():
    """With alpha so small that every |alpha * m / (sqrt(r)+eps)| is under half a bfloat16 ulp of
    its weight, the stored weights cannot move; the states still do."""
    n, B = 4096, 256
    qs, qu = codebooks()
    rng = np.random.default_rng(7)
    w = _narrow((1.0 + rng.random(n)).astype(np.float32))           # in [1, 2): ulp = 2^-7
    g = _narrow((rng.standard_normal(n) * 1e-2).astype(np.float32))
    st = zero_state(n, B)
    w0 = w.copy()
    hp = dict(ADAM, alpha=1e-4)             # |step| <= alpha * (1-b1)/sqrt(1-b2) ~ 3.2e-4 < 2^-8
    oracle.adam8bit_step_bf16(w, g, st["m_q"], st["r_q"], st["N_m"], st["N_r"], qs, qu, B, **hp)
    assert np.array_equal(w, w0)
    assert np.any(st["m_q"] != 127)
