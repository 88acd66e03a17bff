"""The kernels replace the per-element IEEE division by the block maximum (Eq. quant1) and the
square root and division of the weight update (Eq. adam) by short fma sequences.  This file
compiles those sequences for the host from the library's own header and checks that they
return the IEEE results bit for bit: on tens of millions of random operands, on operands built
to land on and next to every decision threshold of both codebooks for block maxima across
2^-60 .. 2^60, and with every admissible value of the hardware's approximate reciprocal and
square root.  No GPU and no oracle involved: the yardstick is the host's IEEE arithmetic."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from paper_2412_01195_amd import q8opt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
f32 = np.float32


@pytest.fixture(scope="module")
def chk(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("exact") / "libexact_check.so")
    subprocess.check_call(["g++", "-O2", "-std=c++20", "-ffp-contract=off", "-fno-fast-math", "-mfma", "-shared", "-fPIC",
                           "-I" + os.path.join(ROOT, "paper_2412_01195_amd", "csrc"),
                           os.path.join(ROOT, "tests", "exact_check.cpp"), "-o", out])
    L = C.CDLL(out)
    i64, p = C.c_int64, C.c_void_p
    L.check_div_fast_pairs.argtypes = [p, p, i64, p]; L.check_div_fast_pairs.restype = i64
    L.check_div_fast_random.argtypes = [C.c_uint64, i64, p, p]; L.check_div_fast_random.restype = i64
    L.check_div_seeds.argtypes = [p, p, i64, p]; L.check_div_seeds.restype = i64
    L.check_div_seeds_mode.argtypes = [p, p, i64, C.c_int, p]; L.check_div_seeds_mode.restype = i64
    L.check_sqrt_seeds.argtypes = [p, i64, p]; L.check_sqrt_seeds.restype = i64
    L.check_sqrt_seeds_mode.argtypes = [p, i64, C.c_int, p]; L.check_sqrt_seeds_mode.restype = i64
    L.check_near_midpoint_pairs.argtypes = [C.c_uint32, C.c_uint32, C.c_int, p]; L.check_near_midpoint_pairs.restype = None
    return L


def thresholds(signed):
    tab = q8opt.build_qtable(q8opt.build_codebook(signed))
    thr = tab[1088:1088 + 1024].view(np.float32)[:255].copy()
    return thr


def test_smallest_threshold_is_far_above_the_subnormal_quotients():
    for signed in (True, False):
        thr = thresholds(signed)
        assert np.abs(thr).min() > 2.0 ** -30           # div_fast may differ from IEEE only below 2^-126


def test_div_fast_random_pairs(chk):
    a, N = C.c_float(), C.c_float()
    for seed in (1, 2, 3):
        bad = chk.check_div_fast_random(seed, 12_000_000, C.byref(a), C.byref(N))
        assert bad == 0, "%d mismatches, first a=%r N=%r" % (bad, a.value, N.value)


@pytest.mark.parametrize("signed", [True, False], ids=["signed", "unsigned"])
def test_div_fast_around_every_threshold(chk, signed):
    """For every threshold t of the codebook, every x within 2 ulps of t, and block maxima N = 2^e
    (e = -60 .. 60) and N with random mantissas: a = RN(x N) and its neighbours, so that a / N
    falls on and next to the threshold."""
    thr = thresholds(signed)
    xs = []
    for k in range(-2, 3):
        v = thr.copy()
        for _ in range(abs(k)):
            v = np.nextafter(v, f32(2.0) if k > 0 else f32(-2.0))
        xs.append(v)
    x = np.concatenate(xs)                                               # 255 * 5 targets
    rng = np.random.default_rng(7 if signed else 8)
    Ns = np.concatenate([np.ldexp(f32(1), np.arange(-60, 61)).astype(f32),
                         (np.ldexp(1.0 + rng.random(180), rng.integers(-60, 60, 180))).astype(f32),
                         np.ldexp(f32(2) - f32(2.0 ** -23), np.arange(-60, 60, 7)).astype(f32)])
    A, NN = [], []
    for N in Ns:
        a0 = (x.astype(np.float64) * np.float64(N)).astype(f32)
        for a in (a0, np.nextafter(a0, f32(np.inf)), np.nextafter(a0, f32(-np.inf))):
            keep = np.abs(a) <= N
            A.append(a[keep]); NN.append(np.full(int(keep.sum()), N, f32))
    A = np.ascontiguousarray(np.concatenate(A)); NN = np.ascontiguousarray(np.concatenate(NN))
    assert A.size > 1_000_000
    first = C.c_int64(-1)
    bad = chk.check_div_fast_pairs(A.ctypes.data, NN.ctypes.data, A.size, C.byref(first))
    assert bad == 0, "%d mismatches, first a=%r N=%r" % (bad, A[first.value], NN[first.value])


def hard_quotients(count, seed, allow_above_one):
    """Pairs of 24-bit mantissas (m, n), n odd, whose quotient lies within about 2^-48 (relative)
    of the midpoint of two neighbouring binary32 values: m P - (2K + 1) n = r for a small odd r,
    solved as m = r P^-1 mod n, with P = 2^25 for m < n (quotient in [1/2, 1)) and P = 2^24 for
    m > n (quotient in (1, 2)).  These are the operands on which a merely faithful quotient
    rounds to the wrong neighbour."""
    rng = np.random.default_rng(seed)
    ms, ns = [], []
    for n in (rng.integers(1 << 22, 1 << 23, count) * 2 + 1).tolist():      # odd, in [2^23, 2^24)
        for P in ((1 << 25), (1 << 24)) if allow_above_one else ((1 << 25),):
            inv = pow(P, -1, n)
            for r in (1, -1, 3, -3, 5, -5):
                m = (r * inv) % n
                if P == (1 << 24):
                    m += n
                    if m >= (1 << 24):
                        continue
                elif m < (1 << 23):
                    continue
                ms.append(m); ns.append(n)
    return np.array(ms, np.float64), np.array(ns, np.float64)


def test_hard_quotient_generator():
    m, n = hard_quotients(2000, 5, True)
    q = m / n                                                     # binary64: 29 spare bits
    ulp = np.where(q < 1.0, 2.0 ** -24, 2.0 ** -23)
    frac = (q / ulp) % 1.0
    assert m.size > 3000 and np.abs(frac - 0.5).max() < 2.0 ** -20     # each quotient hugs a rounding midpoint


def test_div_fast_on_quotients_next_to_rounding_midpoints(chk):
    m, n = hard_quotients(150_000, 21, False)
    rng = np.random.default_rng(22)
    e = rng.integers(-60 + 1, 60 - 24, m.size)
    sign = rng.choice([-1.0, 1.0], m.size)
    a = np.ascontiguousarray(np.ldexp(m * sign, e - 23).astype(f32)); N = np.ascontiguousarray(np.ldexp(n, e - 23).astype(f32))
    assert a.size > 200_000
    first = C.c_int64(-1)
    bad = chk.check_div_fast_pairs(a.ctypes.data, N.ctypes.data, a.size, C.byref(first))
    assert bad == 0, "%d mismatches, first a=%r N=%r" % (bad, a[first.value], N[first.value])


def test_weight_update_division_on_quotients_next_to_rounding_midpoints(chk):
    m, n = hard_quotients(150_000, 23, True)
    rng = np.random.default_rng(24)
    em = rng.integers(-80, 40 - 1, m.size)
    en = np.clip(em + rng.integers(-30, 30, m.size), -40, 30)
    a = np.ascontiguousarray((np.ldexp(m, em - 23) * rng.choice([-1.0, 1.0], m.size)).astype(f32))
    b = np.ascontiguousarray(np.ldexp(n, en - 23).astype(f32))
    first = C.c_int64(-1)
    bad = chk.check_div_seeds(a.ctypes.data, b.ctypes.data, a.size, C.byref(first))
    assert bad == 0, "%d mismatches, first m=%r d=%r" % (bad, a[first.value], b[first.value])


def test_weight_update_division_with_every_seed(chk):
    """m / d for |m| in [2^-80, 2^40], d in [2^-40, 2^31] (the range the kernels guard), log-uniform,
    with the reciprocal seed one ulp low, exact, and one ulp high."""
    rng = np.random.default_rng(11)
    n = 4_000_000
    m = (np.ldexp(1.0 + rng.random(n), rng.integers(-80, 40, n)) * rng.choice([-1.0, 1.0], n)).astype(f32)
    d = np.ldexp(1.0 + rng.random(n), rng.integers(-40, 31, n)).astype(f32)
    # also the operands of a real step: m ~ 1e-4, d = sqrt(r) + eps ~ 1e-4..1e-2, and powers of two
    m[:1000] = np.ldexp(f32(1), rng.integers(-80, 40, 1000)).astype(f32)
    d[:500] = np.ldexp(f32(1), rng.integers(-40, 31, 500)).astype(f32)
    first = C.c_int64(-1)
    bad = chk.check_div_seeds(m.ctypes.data, d.ctypes.data, n, C.byref(first))
    assert bad == 0, "%d mismatches, first m=%r d=%r" % (bad, m[first.value], d[first.value])


def test_square_root_with_every_seed(chk):
    """sqrt(r) for r in [2^-80, 2^40] log-uniform, plus exact squares and their neighbours (where
    the root sits on or next to a binary32 value), with the seed one ulp low, exact, one ulp high."""
    rng = np.random.default_rng(12)
    n = 4_000_000
    r = np.ldexp(1.0 + rng.random(n), rng.integers(-80, 40, n)).astype(f32)
    s = np.ldexp(1.0 + rng.random(300_000), rng.integers(-40, 20, 300_000)).astype(f32)
    sq = (s.astype(np.float64) ** 2).astype(f32)
    mid = ((s.astype(np.float64) + np.nextafter(s, f32(np.inf)).astype(np.float64)) / 2) ** 2      # squares of midpoints
    r = np.ascontiguousarray(np.concatenate([r, sq, np.nextafter(sq, f32(np.inf)), np.nextafter(sq, f32(0)),
                                             mid.astype(f32), np.nextafter(mid.astype(f32), f32(np.inf)),
                                             np.nextafter(mid.astype(f32), f32(0))]))
    # products of two neighbouring binary32 values that are themselves binary32: the root is the
    # geometric mean of the neighbours, just below their midpoint (residual exactly zero)
    k = np.arange(-39, 20)
    exact_products = np.concatenate([np.ldexp(1.0 + 2.0 ** -23, 2 * k), np.ldexp(2.0 - 2.0 ** -23, 2 * k + 1)]).astype(f32)
    r = np.ascontiguousarray(np.concatenate([r, exact_products]))
    r = r[(r >= f32(2.0 ** -80)) & (r <= f32(2.0 ** 40))]
    first = C.c_int64(-1)
    bad = chk.check_sqrt_seeds(r.ctypes.data, r.size, C.byref(first))
    assert bad == 0, "%d mismatches, first r=%r" % (bad, r[first.value])


def test_square_root_exhaustively_over_the_guarded_range(chk):
    """Every binary32 r in [2^-80, 2^40] (1 006 632 961 values), each with every admissible seed:
    the kernels' square root equals the IEEE one on the whole range their range test admits."""
    from concurrent.futures import ThreadPoolExecutor

    def one_binade(e):
        bits = np.uint32((e + 127) << 23) + np.arange(1 << 23, dtype=np.uint32)
        r = bits.view(f32)
        first = C.c_int64(-1)
        bad = chk.check_sqrt_seeds(r.ctypes.data, r.size, C.byref(first))
        return e, int(bad), (float(r[first.value]) if bad else None)
    with ThreadPoolExecutor(max(1, min(8, os.cpu_count() or 1))) as ex:       # the C loop releases the GIL
        for e, bad, where in ex.map(one_binade, range(-80, 40)):
            assert bad == 0, "binade 2^%d: %d mismatches, first r=%r" % (e, bad, where)
    top = np.array([2.0 ** 40], f32)
    first = C.c_int64(-1)
    assert chk.check_sqrt_seeds(top.ctypes.data, 1, C.byref(first)) == 0


def test_div_fast_over_every_numerator_mantissa(chk):
    """For 400 block maxima N (mantissas 1.0, 1 + 2^-23, 2 - 2^-23, around 1.5, and random ones;
    powers of two do not matter because scaling both operands is exact): every binary32 a in
    [N/2, N], i.e. every numerator mantissa against that divisor, 8.4 million quotients per N
    (3.4 * 10^9 in all)."""
    from concurrent.futures import ThreadPoolExecutor
    rng = np.random.default_rng(77)
    mant = np.concatenate([[0, 1, (1 << 23) - 1, 1 << 22, (1 << 22) - 1, (1 << 22) + 1],
                           rng.integers(0, 1 << 23, 394)]).astype(np.uint32)
    expo = rng.integers(-60, 60, mant.size)

    def one_divisor(k):
        nbits = np.uint32((int(expo[k]) + 127) << 23) | mant[k]
        N = np.array([nbits], np.uint32).view(f32)[0]
        lo = int(nbits) - (1 << 23)                                  # N / 2
        a = np.arange(lo, int(nbits) + 1, dtype=np.uint32).view(f32)   # every binary32 in [N/2, N]
        Ns = np.full(a.size, N, f32)
        first = C.c_int64(-1)
        bad = chk.check_div_fast_pairs(a.ctypes.data, Ns.ctypes.data, a.size, C.byref(first))
        return float(N), int(bad), (float(a[first.value]) if bad else None)
    with ThreadPoolExecutor(max(1, min(8, os.cpu_count() or 1))) as ex:
        for N, bad, where in ex.map(one_divisor, range(mant.size)):
            assert bad == 0, "N=%r: %d mismatches, first a=%r" % (N, bad, where)


def test_weight_update_division_over_every_numerator_mantissa(chk):
    """The same for m / d of the weight update: 200 divisors d in [2^-40, 2^31] (special and
    random mantissas), every binary32 m of one binade (all 2^23 numerator mantissas, exponents
    across the guarded range), each with every admissible reciprocal seed."""
    from concurrent.futures import ThreadPoolExecutor
    rng = np.random.default_rng(78)
    mant = np.concatenate([[0, 1, (1 << 23) - 1, 1 << 22, (1 << 22) - 1, (1 << 22) + 1],
                           rng.integers(0, 1 << 23, 194)]).astype(np.uint32)
    e_d = rng.integers(-40, 31, mant.size)
    e_m = rng.integers(-80, 40, mant.size)

    def one_divisor(k):
        d = np.array([np.uint32((int(e_d[k]) + 127) << 23) | mant[k]], np.uint32).view(f32)[0]
        m = (np.uint32((int(e_m[k]) + 127) << 23) + np.arange(1 << 23, dtype=np.uint32)).view(f32)
        if k & 1:
            m = -m
        ds = np.full(m.size, d, f32)
        first = C.c_int64(-1)
        bad = chk.check_div_seeds(np.ascontiguousarray(m).ctypes.data, ds.ctypes.data, m.size, C.byref(first))
        return float(d), int(bad), (float(m[first.value]) if bad else None)
    with ThreadPoolExecutor(max(1, min(8, os.cpu_count() or 1))) as ex:
        for d, bad, where in ex.map(one_divisor, range(mant.size)):
            assert bad == 0, "d=%r: %d mismatches, first m=%r" % (d, bad, where)


def test_the_one_excluded_seed_is_a_real_exception(chk):
    """The seed the checks above set aside: divisor mantissa all ones, seed = the power of two
    half an ulp below 1/d.  With it (strict mode) exactly the power-of-two numerators fail, one per
    binade; every other numerator mantissa still passes.  tests/test_gpu_kernels.py
    (test_weight_update_division_by_all_ones_mantissas) shows the hardware's reciprocal is the other
    neighbour for these divisors."""
    d = np.array([0x3E7FFFFF], np.uint32).view(f32)[0]
    m = (np.uint32(127 << 23) + np.arange(1 << 23, dtype=np.uint32)).view(f32)
    ds = np.full(m.size, d, f32)
    first = C.c_int64(-1)
    assert chk.check_div_seeds_mode(m.ctypes.data, ds.ctypes.data, m.size, 1, C.byref(first)) == 1
    assert m[first.value] == f32(1.0)
    assert chk.check_div_seeds_mode(m.ctypes.data, ds.ctypes.data, m.size, 0, C.byref(first)) == 0


def test_every_quotient_near_a_rounding_midpoint(chk):
    """The complete set of hard operands of both divisions.  They are "product with the correctly
    rounded reciprocal, one residual correction"; the value their last fma rounds lies within
    2^-22 ulp of a/b, so a wrong neighbour needs a/b within that distance of a midpoint:
    for 24-bit mantissas m, n that is |m 2^k - (2K+1) n| <= 16.  The checker solves these
    congruences for EVERY divisor mantissa n and every residue up to +-64 (four times the bound;
    +-256 was run once: 3 * 10^9 pairs), runs div_fast on both signs and div_rn_from_seed with every
    admissible seed, and also confirms for every n that one Newton step turns every admissible
    seed into RN(1/n).  Powers of two scale exactly, so mantissas are all there is to check."""
    from concurrent.futures import ThreadPoolExecutor
    lo, hi, parts = 1 << 23, 1 << 24, 64
    step = (hi - lo) // parts

    def piece(k):
        out = (C.c_int64 * 4)()
        chk.check_near_midpoint_pairs(lo + k * step, lo + (k + 1) * step, 64, out)
        return list(out)
    with ThreadPoolExecutor(max(1, min(8, os.cpu_count() or 1))) as ex:
        tot = np.sum(list(ex.map(piece, range(parts))), axis=0)
    assert tot[0] > 700_000_000, tot
    assert tot[1] == 0 and tot[2] == 0 and tot[3] == 0, "pairs %d: div_fast %d, div_rn_from_seed %d, reciprocal %d" % tuple(tot)


def test_the_one_excluded_root_seed_is_a_real_exception(chk):
    """The (r, seed) pair the square-root checks set aside: in strict mode exactly that r fails in
    each binade of odd exponent, and only with the seed one ulp above the correctly rounded
    reciprocal root.  tests/test_gpu_kernels.py (test_weight_update_root_over_whole_binades)
    runs every r through the kernel: the hardware's seed is another one."""
    for e, expect in ((1, 1), (0, 0), (-37, 1), (-38, 0)):
        r = (np.uint32((e + 127) << 23) + np.arange(1 << 23, dtype=np.uint32)).view(f32)
        first = C.c_int64(-1)
        bad = chk.check_sqrt_seeds_mode(r.ctypes.data, r.size, 1, C.byref(first))
        assert bad == expect, (e, bad)
        if expect:
            assert int(r[first.value].view(np.uint32)) & 0x7fffff == 0x6e9372
