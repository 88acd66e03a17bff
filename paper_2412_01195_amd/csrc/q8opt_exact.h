// The short, exactly rounded forms of division and square root that the kernels use in place
// of the general a / b and sqrtf.  Plain functions of binary32 values built from fma, so that
// the very same source compiles for the GPU (inside q8opt_device.h) and for the host, where
// tests/test_exact_devices.py checks each of them against IEEE division and square root on
// random, adversarial and threshold-hugging operands and on complete enumerations of their hard
// cases (no GPU needed).  The hardware's approximate reciprocal and reciprocal square root
// enter as arguments ("seed"): the host check feeds every binary32 value within one unit in
// the last place of the true result, which covers whatever the instruction returns.
#ifndef Q8OPT_EXACT_H
#define Q8OPT_EXACT_H

#include <stdint.h>

#if defined(__HIP_DEVICE_COMPILE__) || defined(__HIPCC__)
#define Q8_EXACT_FN __device__ __host__ __forceinline__
#else
#define Q8_EXACT_FN static inline
#endif

namespace q8 {
namespace exact {

Q8_EXACT_FN float bits_as_float(uint32_t u) { return __builtin_bit_cast(float, u); }
Q8_EXACT_FN uint32_t float_as_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// Both divisions below are "product with the reciprocal, one residual correction":
//     q = RN(a y),  r = RN(a - b q) (one fma),  result = RN(q + r y) (one fma),
// with y = RN(1/b), the correctly rounded reciprocal.  With u = one ulp of a/b: |a y - a/b| <= u
// (y is off by at most 2^-24 relative), so q is within 2 u of a/b and |a - b q| <= 2 u |b|; the
// rounding of r and the error of y each change r y by at most 2^-24 of that, so the value
// q + r y that the last fma rounds lies within 2^-22 u of a/b.  It can round to the wrong
// neighbour only if a/b itself lies that close to the midpoint of two neighbouring binary32
// values: for 24-bit mantissas m, n that means |m 2^k - (2K+1) n| <= 16 (k = 24 or 25 by the
// quotient's binade), a set the host check enumerates completely -- every n, every residue up
// to +-64 in the suite (+-256 once: 3 * 10^9 pairs), both signs -- and on which the sequence
// returns the IEEE quotient every time (tests/test_exact_devices.py).  Scaling both operands
// by powers of two is exact as long as nothing leaves the normal range, so mantissas are all
// that matters.

// ---- Normalisation x = a / N (Eq. quant1) by a block-uniform N in [2^-60, 2^60], |a| <= N.
// Once per block: y = RN(1/N) (an IEEE division).
Q8_EXACT_FN bool norm_in_fast_range(uint32_t nbits)
{
    return (nbits >= 0x21800000u) && (nbits <= 0x5d800000u);   // 2^-60 .. 2^60
}

Q8_EXACT_FN float reciprocal_rn(float N)
{
    return 1.0f / N;
}

// Per element.  When the quotient is below the normal range (|a/N| < 2^-126) the result may be
// off in its last bits; such values lie far below the smallest decision threshold of any
// codebook the table builder accepts (no non-zero entry below 2^-99) and get the same code.
Q8_EXACT_FN float div_fast(float a, float N, float y)
{
    const float q = a * y;
    const float r = __builtin_fmaf(-N, q, a);
    return __builtin_fmaf(r, y, q);
}

// ---- Weight update of Eq. adam on rows whose new states all lie in [kFastLo, kFastHi]
// (and eps in [0, 2^10], bias-correction factor in [1, 2^10]).
constexpr float kFastLo = 0x1p-80f;
constexpr float kFastHi = 0x1p40f;

// Division: for r in the range, d = sqrt(r) c + eps lies in [2^-40, 2^31] and |m| / d in
// [2^-111, 2^80]: no operand or quotient is zero, subnormal or near the exponent limits, so
// the sequence needs neither operand scaling nor a final fix-up.  `y0` = approximate 1/b,
// within one ulp; one Newton step turns it into RN(1/b) -- for every mantissa of b and every
// such y0 (the host check runs all 2^23 mantissas) with one exception: when the mantissa of b
// is all ones, 1/b lies half an ulp above a power of two, and from that power of two the step
// lands on a tie and returns it again (the known exception of Newton's step); a numerator that
// is a power of two then rounds the wrong way.  The hardware's reciprocal returns the other
// neighbour for such b (checked on the device for every exponent of the range).
Q8_EXACT_FN float div_rn_from_seed(float a, float b, float y0)
{
    const float e = __builtin_fmaf(-b, y0, 1.0f);
    const float y = __builtin_fmaf(e, y0, y0);
    const float q = a * y;
    const float r = __builtin_fmaf(-b, q, a);
    return __builtin_fmaf(r, y, q);
}

// Square root from the approximate reciprocal square root `y` (within one ulp of 1/sqrt(r)):
// s0 = RN(r y) is within a few ulps of the root, d = r - s0^2 its residual (one fma) and
// s0 + d (y/2) one Newton step, rounded once.  A binary32 square root depends only on the
// mantissa and the parity of the exponent (scaling r by 4 and y by 1/2 is exact), so the host
// check runs ALL 2^24 such r, each with every y within one ulp, against the IEEE square root:
// equal everywhere except for one pair -- mantissa 0x6e9372 at an odd exponent (r =
// 0x1.dd26e4p+1 times a power of 4) with the seed one ulp ABOVE the correctly rounded
// reciprocal root, which ends one ulp low.  The device suite runs every r of [2^-80, 2^40]
// through the kernel and finds the IEEE root each time: the hardware does not return that seed.
Q8_EXACT_FN float sqrt_rn_from_rsq(float r, float y)
{
    const float s0 = r * y;
    const float h = 0.5f * y;
    const float d = __builtin_fmaf(-s0, s0, r);
    return __builtin_fmaf(d, h, s0);
}

}  // namespace exact
}  // namespace q8

#endif  // Q8OPT_EXACT_H
