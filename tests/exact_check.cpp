// Host-side check of the kernels' exactly rounded division and square-root forms: compiled by
// tests/test_exact_devices.py from the library's own header (csrc/q8opt_exact.h), so what is
// checked here is the source the GPU runs.  Each function returns the number of operands whose
// result differs from the IEEE operation and stores the index of the first such operand.
//   g++ -O2 -ffp-contract=off -mfma -shared -fPIC
#include <cmath>
#include <cstdint>
#include <cstring>

#include "q8opt_exact.h"

using namespace q8::exact;

namespace {
inline uint32_t bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float next_up(float f) { return std::nextafterf(f, INFINITY); }
inline float next_dn(float f) { return std::nextafterf(f, -INFINITY); }

// splitmix64: the test's own generator for the random sweeps
inline uint64_t mix(uint64_t& s)
{
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
}  // namespace

extern "C" {

// Normalisation: a[i] / N[i] with |a| <= N, N in [2^-60, 2^60].  A quotient in the normal
// range must equal the IEEE quotient bit for bit; below it, both must stay below 2^-100 in
// magnitude with the same sign (far under any threshold: same code).
int64_t check_div_fast_pairs(const float* a, const float* N, int64_t n, int64_t* first_bad)
{
    int64_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (!norm_in_fast_range(bits(N[i])) || !(std::fabs(a[i]) <= N[i])) { if (!bad++) *first_bad = i; continue; }
        const float y = reciprocal_rn(N[i]);
        const float got = div_fast(a[i], N[i], y), want = a[i] / N[i];
        bool ok;
        if (std::fabs(want) >= 0x1p-126f) ok = bits(got) == bits(want);
        else ok = std::fabs(got) < 0x1p-100f && (got == 0.0f || want == 0.0f || std::signbit(got) == std::signbit(want));
        if (!ok && !bad++) *first_bad = i;
    }
    return bad;
}

// Random sweep: N = 2^e * m with e in [-60, 59], a = N * u for u spread over [-1, 1] on a
// logarithmic scale down to 2^-40, plus a = N and a = -N.
int64_t check_div_fast_random(uint64_t seed, int64_t count, float* bad_a, float* bad_N)
{
    int64_t bad = 0;
    uint64_t s = seed;
    for (int64_t i = 0; i < count; ++i) {
        const uint64_t r1 = mix(s), r2 = mix(s);
        const int e = (int)(r1 % 120) - 60;
        const float N = std::ldexp(1.0f + (float)((r1 >> 20) & 0x7fffff) / 8388608.0f, e);
        const int eu = -(int)((r2 >> 8) % 41);
        float a = N * std::ldexp((float)((r2 >> 20) & 0xffffff) / 16777216.0f, eu);
        if (r2 & 1) a = -a;
        if ((r2 & 0xfe) == 0) a = (r2 & 1) ? -N : N;
        if (!(std::fabs(a) <= N) || !norm_in_fast_range(bits(N))) continue;
        const float y = reciprocal_rn(N);
        const float got = div_fast(a, N, y), want = a / N;
        const bool ok = (std::fabs(want) >= 0x1p-126f) ? bits(got) == bits(want) : std::fabs(got) < 0x1p-100f;
        if (!ok && !bad++) { *bad_a = a; *bad_N = N; }
    }
    return bad;
}

// A seed is admissible if it lies within one unit in the last place of the TRUE value (the
// accuracy the instruction set documents for the approximate reciprocal and square root).
inline bool admissible(float seed, double truth)
{
    const double ulp = (double)next_up(std::fabs(seed)) - (double)std::fabs(seed);
    return std::fabs((double)seed - truth) <= ulp;
}

// Weight-update division m / d with every admissible seed for 1/d.  One seed is set aside: for
// a divisor whose mantissa is all ones, 1/d lies half an ulp above a power of two, and from
// that power of two the reciprocal refinement lands on a tie and stays there (the textbook
// exception of Newton's step for reciprocals); a power-of-two numerator then rounds the wrong
// way.  `strict` != 0 checks that seed too (the test that shows the exception is real); the
// GPU suite checks that the hardware does not return it (every exponent of the guarded range).
int64_t check_div_seeds_mode(const float* m, const float* d, int64_t n, int strict, int64_t* first_bad)
{
    int64_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        const float want = m[i] / d[i];
        const float y = 1.0f / d[i];
        const float seeds[3] = {next_dn(y), y, next_up(y)};
        const bool all_ones = (bits(d[i]) & 0x7fffffu) == 0x7fffffu;
        for (float y0 : seeds) {
            if (!admissible(y0, 1.0 / (double)d[i])) continue;
            if (!strict && all_ones && (bits(y0) & 0x7fffffu) == 0) continue;
            if (bits(div_rn_from_seed(m[i], d[i], y0)) != bits(want) && !bad++) *first_bad = i;
        }
    }
    return bad;
}

int64_t check_div_seeds(const float* m, const float* d, int64_t n, int64_t* first_bad)
{
    return check_div_seeds_mode(m, d, n, 0, first_bad);
}

// Square root with every admissible seed for 1/sqrt(r) (within one ulp of the true value).  One
// (r, seed) pair is set aside unless `strict`: mantissa 0x6e9372 at an odd exponent with the
// seed one ulp above the correctly rounded reciprocal root (see q8opt_exact.h); the device
// suite shows that the hardware does not return it.
int64_t check_sqrt_seeds_mode(const float* r, int64_t n, int strict, int64_t* first_bad)
{
    int64_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        const float want = std::sqrt(r[i]);
        const double truth = 1.0 / std::sqrt((double)r[i]);
        const float y = (float)truth;
        const float seeds[3] = {next_dn(y), y, next_up(y)};
        const bool special = (bits(r[i]) & 0x7fffffu) == 0x6e9372u && ((bits(r[i]) >> 23) & 1u) == 0u;   // odd exponent
        for (int k = 0; k < 3; ++k) {
            if (!admissible(seeds[k], truth)) continue;
            if (!strict && special && k == 2) continue;
            if (bits(sqrt_rn_from_rsq(r[i], seeds[k])) != bits(want) && !bad++) *first_bad = i;
        }
    }
    return bad;
}

int64_t check_sqrt_seeds(const float* r, int64_t n, int64_t* first_bad)
{
    return check_sqrt_seeds_mode(r, n, 0, first_bad);
}

// The complete set of hard operands of "product with the reciprocal, one correction": every pair
// of 24-bit mantissas (m, n) whose quotient lies within R * 2^-48 (relative) of a value with 25
// significant bits -- the midpoints of neighbouring binary32 values are among them -- i.e.
// m 2^k - L n = r with 0 < |r| <= R, k = 25 for m < n and 24 for m > n.  For each divisor n
// [n_begin, n_end) the numerators are solved from m = r 2^-k (mod n).  Each pair is run through
// div_fast with y = RN(1/n) (both signs of m) and through div_rn_from_seed with every admissible
// seed; the refined reciprocal of every admissible seed is also compared with RN(1/n).
// out[0] = pairs, out[1] = div_fast failures, out[2] = div_rn_from_seed failures,
// out[3] = refined reciprocals that are not RN(1/n).
void check_near_midpoint_pairs(uint32_t n_begin, uint32_t n_end, int R, int64_t* out)
{
    int64_t pairs = 0, bad_fast = 0, bad_seed = 0, bad_y = 0;
    for (uint32_t n = n_begin; n < n_end; ++n) {
        const float b = (float)n, yrn = 1.0f / b;
        const double truth = 1.0 / (double)b;
        const float seeds[3] = {next_dn(yrn), yrn, next_up(yrn)};
        bool adm[3];
        const bool all_ones = (n & 0x7fffffu) == 0x7fffffu;
        for (int k = 0; k < 3; ++k) {
            adm[k] = admissible(seeds[k], truth) && !(all_ones && (bits(seeds[k]) & 0x7fffffu) == 0);
            if (!adm[k]) continue;
            const float e = __builtin_fmaf(-b, seeds[k], 1.0f);
            if (bits(__builtin_fmaf(e, seeds[k], seeds[k])) != bits(yrn)) ++bad_y;
        }
        const int j = __builtin_ctz(n);
        const uint32_t g = 1u << j, n2 = n >> j;                       // n = g * n2, n2 odd
        const uint64_t inv2 = (n2 + 1) / 2;                            // 2^-1 mod n2
        for (int kP = 24; kP <= 25; ++kP) {
            uint64_t inv = 1 % n2;                                      // (2^kP / g)^-1 mod n2
            for (int i = 0; i < kP - j; ++i) inv = inv * inv2 % n2;
            for (int r = -R; r <= R; ++r) {
                if (r == 0 || (r & (int)(g - 1))) continue;             // solvable only if g divides r
                const int64_t rr = r / (int)g;
                const uint64_t m0 = (uint64_t)((rr % (int64_t)n2 + n2) % n2) * inv % n2;
                for (uint64_t m = m0; m < (1u << 24); m += n2) {        // all residues mod n, lifted into the mantissa range
                    if (m < (1u << 23)) continue;
                    if (kP == 25 ? !(m < n) : !(m > n)) continue;
                    const float a = (float)m, want = a / b;
                    ++pairs;
                    if (bits(div_fast(a, b, yrn)) != bits(want)) ++bad_fast;
                    if (bits(div_fast(-a, b, yrn)) != bits(-want)) ++bad_fast;
                    for (int k = 0; k < 3; ++k)
                        if (adm[k] && bits(div_rn_from_seed(a, b, seeds[k])) != bits(want)) ++bad_seed;
                }
            }
        }
    }
    out[0] = pairs; out[1] = bad_fast; out[2] = bad_seed; out[3] = bad_y;
}

// The same set of pairs as a list (for the device test): mantissas as integers in [2^23, 2^24).
// Returns the number of pairs written (at most cap).
int64_t list_near_midpoint_pairs(uint32_t n_begin, uint32_t n_end, int R, uint32_t* out_m, uint32_t* out_n, int64_t cap)
{
    int64_t count = 0;
    for (uint32_t n = n_begin; n < n_end; ++n) {
        const int j = __builtin_ctz(n);
        const uint32_t g = 1u << j, n2 = n >> j;
        const uint64_t inv2 = (n2 + 1) / 2;
        for (int kP = 24; kP <= 25; ++kP) {
            uint64_t inv = 1 % n2;
            for (int i = 0; i < kP - j; ++i) inv = inv * inv2 % n2;
            for (int r = -R; r <= R; ++r) {
                if (r == 0 || (r & (int)(g - 1))) continue;
                const int64_t rr = r / (int)g;
                const uint64_t m0 = (uint64_t)((rr % (int64_t)n2 + n2) % n2) * inv % n2;
                for (uint64_t m = m0; m < (1u << 24); m += n2) {
                    if (m < (1u << 23)) continue;
                    if (kP == 25 ? !(m < n) : !(m > n)) continue;
                    if (count == cap) return count;
                    out_m[count] = (uint32_t)m; out_n[count] = n; ++count;
                }
            }
        }
    }
    return count;
}

}  // extern "C"
