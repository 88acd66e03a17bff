"""Pins of the oracle's codebook against what the paper fixes (Sec. IV-B, dynamic-tree
data type): 8 bits -> 256 values in [-1, 1]; layout sign | zeros (decimal exponent) |
indicator | linear fraction; finest fraction step 1/63 of the span index (6 fraction
bits); smallest exponent below 1e-6.  The decoder below is written independently, in
exact rational arithmetic, and walks the bit fields explicitly."""
from fractions import Fraction

import numpy as np

import oracle


def f32_nearest(fr: Fraction) -> np.float32:
    """Correctly rounded binary32 of an exact rational (via exact comparison)."""
    x = np.float32(float(fr))            # double rounding is checked away below
    lo, hi = np.nextafter(x, np.float32(-np.inf)), np.nextafter(x, np.float32(np.inf))
    best = min((x, lo, hi), key=lambda c: abs(Fraction(float(c)) - fr))
    return np.float32(best)


def decode(bits: str, signed: bool) -> Fraction:
    """bits: 8 characters, most significant first."""
    lead, rest = bits[0], bits[1:]
    if "1" not in rest:
        return Fraction(1 if lead == "1" else 0)
    E = rest.index("1")                  # zeros before the indicator
    frac_bits = rest[E + 1:]
    if not signed:
        frac_bits = lead + frac_bits     # leading bit is the top fraction bit
    F = len(frac_bits)
    k = int(frac_bits, 2) if F else 0
    mant = Fraction(1, 10) + Fraction(9, 10) * Fraction(2 * k + 1, 2 ** (F + 1))
    mag = mant / Fraction(10) ** E
    return -mag if (signed and lead == "1") else mag


def rational_map(signed: bool):
    vals = sorted(decode(format(p, "08b"), signed) for p in range(256))
    return vals


def test_count_range_monotone():
    for signed in (True, False):
        q = oracle.build_codebook(signed)
        assert q.dtype == np.float32 and q.shape == (256,)
        assert np.all(np.diff(q.astype(np.float64)) > 0)
        assert q.max() == np.float32(1.0)
        assert q.min() >= np.float32(-1.0)
        assert (q == 0).sum() == 1
    assert oracle.build_codebook(True)[127] == 0 and oracle.build_codebook(False)[0] == 0
    assert oracle.build_codebook(True).min() < 0 and oracle.build_codebook(False).min() == 0


def test_matches_rational_bitfield_decoder():
    for signed in (True, False):
        q = oracle.build_codebook(signed)
        ref = rational_map(signed)
        assert len(set(ref)) == 256
        for j in range(256):
            assert q[j] == f32_nearest(ref[j]), (signed, j, q[j], float(ref[j]))


def test_decade_populations_and_spacing():
    for signed, pops in ((True, [64, 32, 16, 8, 4, 2, 1]), (False, [128, 64, 32, 16, 8, 4, 2])):
        ref = [v for v in rational_map(signed) if 0 < v < 1]
        for E, cnt in enumerate(pops):
            lo, hi = Fraction(1, 10 ** (E + 1)), Fraction(1, 10 ** E)
            dec = [v for v in ref if lo < v < hi]
            assert len(dec) == cnt, (signed, E, len(dec))
            gaps = {b - a for a, b in zip(dec, dec[1:])}
            if cnt > 1:
                assert gaps == {Fraction(9, 10) / cnt / 10 ** E}
            # bin centres: first value sits half a step above the decade's lower end
            assert dec[0] - lo == Fraction(9, 10) / cnt / 10 ** E / 2


def test_fraction_resolution_and_smallest_exponent():
    qs = oracle.build_codebook(True)
    top = qs[(qs > 0.1) & (qs < 1.0)]
    assert top.size == 64                       # 6 fraction bits: 63 steps across the decade
    pos = qs[qs > 0]
    assert 1e-7 <= pos.min() < 1e-6
    assert pos.min() == np.float32(0.55e-6)
    assert qs[254] == np.float32(1 - 0.9 / 128)
    assert qs[0] == -qs[254]
    # the negative half mirrors the positive one except that -1 is absent
    assert np.array_equal(qs[:127], -qs[128:255][::-1])
    qu = oracle.build_codebook(False)
    assert qu[1] == np.float32(0.325e-6) and qu[2] == np.float32(0.775e-6)
    assert qu[254] == np.float32(1 - 0.9 / 256)
    assert np.max(np.diff(qu.astype(np.float64))) <= 0.9 / 128 * (1 + 1e-5)
    assert np.max(np.diff(qs.astype(np.float64))) <= 0.9 / 64 * (1 + 1e-5)


def test_state_memory_saving_closed_form():
    """Abstract / Sec. I: 8-bit states save 75 % of state memory (per-block absmax
    overhead 4 bytes per B entries)."""
    for B, expect in ((2048, 75 - 100 / 2048), (256, 75 - 100 / 256)):
        n = B * 1000
        q8 = n + 4 * oracle.nblocks(n, B)
        assert abs((1 - q8 / (4 * n)) * 100 - expect) < 1e-9
