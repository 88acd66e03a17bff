"""Pins of the oracle's IEEE binary16 storage extension (weights and gradients held as
binary16; arithmetic and 8-bit states unchanged; not part of the paper).

Widening is checked for all 65536 patterns against numpy's float16, narrowing against the
definition of round-to-nearest-even in exact rational arithmetic and against numpy's cast;
the steps against the fp32-storage step on widened values."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests.harness import ADAM, SGD, codebooks, zero_state


def test_widening_equals_library_for_every_pattern():
    h = np.arange(65536, dtype=np.uint16)
    want = h.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_to_f32(int(x)) for x in h], np.float32)
    fin = np.isfinite(want)
    assert np.array_equal(got[fin].view(np.uint32), want[fin].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(np.isinf(got), np.isinf(want))
    assert np.array_equal(np.signbit(got[~np.isnan(got)]), np.signbit(want[~np.isnan(want)]))


def _all_f16_values():
    h = np.arange(0x7c00, dtype=np.uint16)              # non-negative finite patterns, ascending
    return h, [Fraction(float(v)) for v in h.view(np.float16).astype(np.float64)]


def _nearest_even_f16(x: float, pats, vals) -> int:
    """Definition: the finite binary16 value closest to x in exact arithmetic, ties to the even
    pattern; beyond the midpoint between 65504 and 65536 the result is infinity."""
    a = Fraction(abs(float(x)))
    sign = 0x8000 if np.signbit(np.float32(x)) else 0
    if a >= Fraction(65520):                             # 65504 + half a unit (32 / 2); the tie goes to the even 'pattern' infinity
        return sign | 0x7c00
    lo, hi = 0, len(vals) - 1                            # largest value <= a
    while lo < hi:
        mid = (lo + hi + 1) // 2
        if vals[mid] <= a:
            lo = mid
        else:
            hi = mid - 1
    if lo == len(vals) - 1:
        return sign | int(pats[lo])
    dlo, dhi = a - vals[lo], vals[lo + 1] - a
    if dlo < dhi:
        k = lo
    elif dhi < dlo:
        k = lo + 1
    else:
        k = lo if pats[lo] % 2 == 0 else lo + 1
    return sign | int(pats[k])


def test_rounding_matches_exact_definition():
    pats, vals = _all_f16_values()
    rng = np.random.default_rng(21)
    # magnitudes concentrated on binary16's range, plus ties / near ties built from adjacent binary16 values
    x = (rng.standard_normal(6000) * 10.0 ** rng.uniform(-9, 5.2, 6000)).astype(np.float32)
    k = rng.integers(0, 0x7bff, 3000)
    a = pats[k].view(np.float16).astype(np.float64); b = pats[k + 1].view(np.float16).astype(np.float64)
    mid = ((a + b) / 2).astype(np.float32)                # exact: one more bit than binary16 fits binary32
    special = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf)), -mid,
                              np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e30, -1e30, 2.0 ** -24,
                                        2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -26, 1e-45, 6.1e-5, 6.097e-5], np.float32)])
    for v in np.concatenate([x, special]):
        assert oracle.f32_to_f16(v) == _nearest_even_f16(v, pats, vals), float(v)


def test_rounding_matches_library_cast():
    rng = np.random.default_rng(22)
    x = (rng.standard_normal(200000) * 10.0 ** rng.uniform(-10, 6, 200000)).astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16(v) for v in x], np.uint16)
    assert np.array_equal(got, want)


def test_known_values():
    assert oracle.f32_to_f16(1.0) == 0x3c00 and oracle.f32_to_f16(-2.0) == 0xc000
    assert oracle.f32_to_f16(65504.0) == 0x7bff and oracle.f32_to_f16(65520.0) == 0x7c00
    assert oracle.f32_to_f16(1.0 + 2.0 ** -11) == 0x3c00            # tie, even below
    assert oracle.f32_to_f16(1.0 + 3 * 2.0 ** -11) == 0x3c02        # tie, even above
    assert oracle.f32_to_f16(2.0 ** -24) == 0x0001 and oracle.f32_to_f16(2.0 ** -25) == 0x0000
    assert oracle.f16_to_f32(0x3e00) == 1.5 and oracle.f16_to_f32(0x0001) == 2.0 ** -24


def _widen(h):
    return h.view(np.float16).astype(np.float32)


def _narrow(x):
    return np.array([oracle.f32_to_f16(v) for v in x], np.uint16)


@pytest.mark.parametrize("B", [64, 2048])
def test_adam_step_is_fp32_step_on_widened_values(B):
    n = 3 * 2048 + 77
    qs, qu = codebooks()
    rng = np.random.default_rng(31)
    w = _narrow((rng.standard_normal(n) * 0.05).astype(np.float32))
    g = _narrow((rng.standard_normal(n) * 1e-3).astype(np.float32))
    st_a, st_b = zero_state(n, B), zero_state(n, B)
    w32 = _widen(w)
    for t in range(1, 4):
        oracle.adam8bit_step_f16(w, g, st_a["m_q"], st_a["r_q"], st_a["N_m"], st_a["N_r"], qs, qu, B, wd=0.01, t=t, **ADAM)
        oracle.adam8bit_step(w32, _widen(g), st_b["m_q"], st_b["r_q"], st_b["N_m"], st_b["N_r"], qs, qu, B,
                             wd=0.01, t=t, **ADAM)
        w32 = _widen(_narrow(w32))
        assert np.array_equal(w, _narrow(w32))
        for k in st_a:
            assert np.array_equal(st_a[k].view(np.uint8), st_b[k].view(np.uint8)), (k, t)


def test_sgd_step_is_fp32_step_on_widened_values():
    n, B = 5000, 256
    qs, _ = codebooks()
    rng = np.random.default_rng(32)
    w = _narrow((rng.standard_normal(n) * 0.05).astype(np.float32))
    g = _narrow((rng.standard_normal(n) * 1e-2).astype(np.float32))
    st_a, st_b = zero_state(n, B, adam=False), zero_state(n, B, adam=False)
    w32 = _widen(w)
    for _ in range(3):
        oracle.sgd8bit_step_f16(w, g, st_a["m_q"], st_a["N_m"], qs, B, wd=1e-4, **SGD)
        oracle.sgd8bit_step(w32, _widen(g), st_b["m_q"], st_b["N_m"], qs, B, wd=1e-4, **SGD)
        w32 = _widen(_narrow(w32))
        assert np.array_equal(w, _narrow(w32))
        assert np.array_equal(st_a["m_q"], st_b["m_q"]) and np.array_equal(st_a["N_m"], st_b["N_m"])
