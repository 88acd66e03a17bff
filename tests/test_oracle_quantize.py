"""Pins of the oracle's block-wise quantization (Sec. IV-B: tensor chunking, Eq. quant1,
Eq. quant2, Eq. quant3).  The search is checked against exact rational argmin, the
error bound of nearest rounding, and structural invariants; none of the checks below
re-uses the oracle's own search or its midpoint formula."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

QS = oracle.build_codebook(True)
QU = oracle.build_codebook(False)


def exact_argmin(q, x) -> int:
    fx = Fraction(float(x))
    d = [abs(Fraction(float(v)) - fx) for v in q]
    return d.index(min(d))               # first minimum


def neighbours(v, k=2):
    out = [np.float32(v)]
    lo = hi = np.float32(v)
    for _ in range(k):
        lo = np.nextafter(lo, np.float32(-np.inf)); hi = np.nextafter(hi, np.float32(np.inf))
        out += [lo, hi]
    return out


@pytest.mark.parametrize("q", [QS, QU], ids=["signed", "unsigned"])
def test_search_equals_exact_argmin_on_critical_points(q):
    pts = []
    for j in range(256):
        pts += neighbours(q[j])
        if j < 255:
            mid = (np.float64(q[j]) + np.float64(q[j + 1])) / 2
            pts += neighbours(np.float32(mid), 3)
    pts += [np.float32(v) for v in (-1.0, 1.0, 0.0, -0.0, 1e-30, -1e-30, 1e-45, -1e-45, 0.5, -0.5)]
    for x in pts:
        if abs(float(x)) > 1:
            continue
        e = exact_argmin(q, x)
        assert oracle.nearest_code(q, x) == e, (float(x), e)
        assert oracle.nearest_code_bruteforce(q, x) == e, (float(x), e)


@pytest.mark.parametrize("q", [QS, QU], ids=["signed", "unsigned"])
def test_search_equals_exact_argmin_random(q):
    rng = np.random.default_rng(7)
    xs = np.concatenate([rng.uniform(-1, 1, 1500), rng.standard_normal(500) * 1e-3,
                         10.0 ** rng.uniform(-9, 0, 500) * rng.choice([-1, 1], 500)]).astype(np.float32)
    if q is QU:
        xs = np.abs(xs)
    for x in xs:
        assert oracle.nearest_code(q, x) == exact_argmin(q, x)


def test_ties_keep_lower_index():
    # 0.5 * (Q_j + Q_j+1) is exactly representable for several neighbouring pairs
    hits = 0
    for q in (QS, QU):
        for j in range(255):
            mid = (np.float64(q[j]) + np.float64(q[j + 1])) / 2
            if np.float64(np.float32(mid)) == mid:
                hits += 1
                assert oracle.nearest_code(q, np.float32(mid)) == j
                assert oracle.nearest_code(q, np.nextafter(np.float32(mid), np.float32(2))) == j + 1
    assert hits > 10


@pytest.mark.parametrize("q", [QS, QU], ids=["signed", "unsigned"])
def test_codes_exact_monotone_and_half_gap_bound(q):
    for j in range(256):
        assert oracle.nearest_code(q, q[j]) == j
    rng = np.random.default_rng(11)
    xs = np.sort(rng.uniform(float(q[0]), 1, 4000).astype(np.float32))
    codes = np.array([oracle.nearest_code(q, x) for x in xs])
    assert np.all(np.diff(codes) >= 0)
    q64 = q.astype(np.float64)
    for x, c in zip(xs, codes):
        j = np.searchsorted(q64, np.float64(x), side="right") - 1
        j = min(max(j, 0), 254)
        gap = q64[j + 1] - q64[j]
        assert abs(q64[c] - np.float64(x)) <= gap / 2
    # below the lowest signed code (-1 is not representable): clamp, error <= 0.9/128
    if q is QS:
        for x in np.linspace(-1, float(q[0]), 50).astype(np.float32):
            assert oracle.nearest_code(q, x) == 0
            assert abs(float(q[0]) - float(x)) <= 0.9 / 128 + 1e-7


def test_absmax_blocks_and_ragged_tail():
    rng = np.random.default_rng(3)
    for n, B in ((1, 64), (63, 64), (64, 64), (65, 64), (1000, 256), (2048 * 3 + 512, 2048), (5000, 4096)):
        T = (rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 2)).astype(np.float32)
        TQ, N = oracle.quantize_blockwise(QS, T, B)
        nb = -(-n // B)
        assert N.shape == (nb,) and TQ.shape == (n,)
        for b in range(nb):
            blk = T[b * B:(b + 1) * B]
            assert N[b] == np.abs(blk).max()
            i = int(np.abs(blk).argmax())
            assert TQ[b * B + i] == (255 if blk[i] > 0 else 0)
            # element-wise definition: one binary32 division, then exact argmin
            for k in rng.integers(0, blk.size, 5):
                assert TQ[b * B + k] == exact_argmin(QS, np.float32(blk[k]) / np.float32(N[b]))


def test_block_independence():
    rng = np.random.default_rng(5)
    B, n = 256, 256 * 6 + 17
    T = rng.standard_normal(n).astype(np.float32)
    TQ0, N0 = oracle.quantize_blockwise(QS, T, B)
    T2 = T.copy(); T2[3 * B:4 * B] *= 37.0
    TQ1, N1 = oracle.quantize_blockwise(QS, T2, B)
    keep = np.ones(n, bool); keep[3 * B:4 * B] = False
    assert np.array_equal(TQ0[keep], TQ1[keep])
    assert np.array_equal(np.delete(N0, 3), np.delete(N1, 3)) and N1[3] != N0[3]


def test_zero_block_and_empty():
    T = np.zeros(300, np.float32); T[256:] = [1.0] * 44
    TQ, N = oracle.quantize_blockwise(QS, T, 256)
    assert N[0] == 0 and np.all(TQ[:256] == 127) and N[1] == 1 and np.all(TQ[256:] == 255)
    TQ, N = oracle.quantize_blockwise(QU, np.zeros(10, np.float32), 64)
    assert N[0] == 0 and np.all(TQ == 0)
    TQ, N = oracle.quantize_blockwise(QS, np.zeros(0, np.float32), 64)
    assert TQ.size == 0 and N.size == 0


def test_dequantize_is_one_multiply_and_roundtrip():
    rng = np.random.default_rng(9)
    n, B = 3000, 256
    TQ = rng.integers(0, 256, n).astype(np.uint8)
    N = (10.0 ** rng.uniform(-8, 3, -(-n // B))).astype(np.float32)
    for q in (QS, QU):
        TD = oracle.dequantize_blockwise(q, TQ, N, B)
        ref = q[TQ] * np.repeat(N, B)[:n]          # numpy binary32 multiply
        assert np.array_equal(TD, ref)
        # blocks that contain the code of +1 re-quantize to themselves
        TQ2 = TQ.copy(); TQ2[::B] = 255
        TD2 = oracle.dequantize_blockwise(q, TQ2, N, B)
        TQ3, N3 = oracle.quantize_blockwise(q, TD2, B)
        assert np.array_equal(N3, N) and np.array_equal(TQ3, TQ2)


def test_roundtrip_error_bound_on_tensor():
    """|T^D - T| <= N_b * (half the local codebook gap), plus the rounding of the
    division and of the multiply (a few ulp of N_b)."""
    rng = np.random.default_rng(13)
    n, B = 2048 * 4 + 100, 2048
    T = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    TQ, N = oracle.quantize_blockwise(QS, T, B)
    TD = oracle.dequantize_blockwise(QS, TQ, N, B)
    q64 = QS.astype(np.float64)
    Nrep = np.repeat(N.astype(np.float64), B)[:n]
    x = T.astype(np.float64) / Nrep
    j = np.clip(np.searchsorted(q64, x, side="right") - 1, 0, 254)
    half_gap = (q64[j + 1] - q64[j]) / 2
    below = x < q64[0]
    half_gap[below] = 0.9 / 128
    assert np.all(np.abs(TD.astype(np.float64) - T) <= Nrep * (half_gap + 4e-7))


@pytest.mark.parametrize("q", [QS, QU], ids=["signed", "unsigned"])
def test_normalization_is_one_correctly_rounded_division(q):
    """Eq. quant1 divides by N_b.  Blocks are built so that the quotient T/N falls on
    the two binary32 values that straddle a code midpoint: any other rounding of the
    quotient (a reciprocal multiply, a fused or truncated divide) flips codes here."""
    rng = np.random.default_rng(17)
    mids = (q[:-1].astype(np.float64) + q[1:].astype(np.float64)) / 2
    up = np.float32(mids)
    up = np.where(up.astype(np.float64) > mids, up, np.nextafter(up, np.float32(2)))   # first float above
    dn = np.nextafter(up, np.float32(-2))
    flips = 0
    for _ in range(120):
        N = np.float32(10.0 ** rng.uniform(-6, 3) * rng.uniform(1, 2))
        cand = []
        for xs in (up, dn):
            t = (xs * N).astype(np.float32)
            for d in (-1, 0, 1):
                tt = t.copy()
                for _ in range(abs(d)):
                    tt = np.nextafter(tt, np.float32(np.inf if d > 0 else -np.inf))
                cand.append(tt)
        T = np.concatenate([[N], np.concatenate(cand)]).astype(np.float32)
        T = T[np.abs(T) <= N]
        TQ, Nb = oracle.quantize_blockwise(q, T, 4096)
        assert Nb[0] == N
        x = T / N                                          # numpy: IEEE binary32 division
        ref = np.searchsorted(up, x, side="right")         # number of midpoints strictly below x
        assert np.array_equal(TQ, ref.astype(np.uint8))
        xr = T * (np.float32(1) / N)
        flips += int((np.searchsorted(up, xr, side="right") != ref).sum())
    assert flips > 50          # the construction does separate a reciprocal multiply from a division
