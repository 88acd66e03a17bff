/*
 * q8_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, sequential CPU definition of the 8-bit optimizer-state method of the
 * paper (Sec. IV "Optimizer State Quantization"): block-wise dynamic-tree
 * quantization (Eq. quant1-quant3) wrapped around the SGD-momentum (Eq. sgd)
 * and Adam (Eq. adam) updates.  Only tests/, the smoke check and the benchmark's
 * cpu_baseline leg may build, load or call this file.  It shares no code, table
 * or constant with the HIP library and includes none of its headers.
 *
 * Arithmetic contract: every floating-point operation below is one IEEE-754
 * binary32 operation rounded to nearest-even, in the order written; build with
 *     gcc -O2 -ffp-contract=off -fno-fast-math
 * so that no multiply-add is fused and nothing is re-associated.  Denormals are
 * kept.  The codebook is evaluated in binary64 and rounded once to binary32.
 *
 * Pins (tests/test_oracle_*.py): codebook structure against an independent
 * rational-arithmetic bit-field decoder; nearest-code search against a 256-way
 * exact argmin; round-trip error bound; fp32-state updates against closed forms
 * and against an independently written recurrence, bit for bit, with and without
 * the two extension flags; the bias-correction scalars against exact rational
 * arithmetic.  Every function here has at least one such pin, and
 * tests/test_oracle_mutations.py plants single mistakes in a copy of this file
 * and checks that the pins catch each of them.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define ORACLE_FLAG_BIAS_CORRECTION 1   /* extension, not printed in Eq. adam */
#define ORACLE_FLAG_DECOUPLED_WD    2   /* extension: AdamW-style decay        */

/* ------------------------------------------------------------------------- */
/* Codebook Q^map (Sec. IV-B "Nearest value searching", dynamic-tree type).   */
/*                                                                           */
/* An 8-bit pattern reads: leading bit | run of E zero bits | indicator 1 |   */
/* F linear-fraction bits.  E is a decimal exponent, so the pattern encodes   */
/* a mantissa in [0.1, 1] divided by 10^E; the F fraction bits index 2^F      */
/* equal bins of [0.1, 1] and the value is the bin centre.                    */
/*   signed map   : leading bit = sign, 7 remaining bits, E = 0..6, F = 6-E   */
/*   unsigned map : leading bit = extra (most significant) fraction bit,      */
/*                  E = 0..6, F = 7-E                                         */
/* The two patterns whose 7 low bits hold no indicator encode 0.0 (leading    */
/* bit 0) and +1.0 (leading bit 1).  The stored code is the RANK of the value */
/* in ascending order, which is what a binary search needs.                   */
/* ------------------------------------------------------------------------- */
static double pattern_value(int pattern, int is_signed)
{
    int lead = (pattern >> 7) & 1;
    int low7 = pattern & 0x7f;
    if (low7 == 0)
        return lead ? 1.0 : 0.0;
    int E = 0;
    while (((low7 >> (6 - E)) & 1) == 0)
        ++E;                                   /* zeros before the indicator */
    int fbits_low = 6 - E;                     /* fraction bits after it     */
    int k = low7 & ((1 << fbits_low) - 1);
    int F = fbits_low;
    if (!is_signed) {                          /* leading bit joins fraction */
        k |= lead << fbits_low;
        F = fbits_low + 1;
    }
    double num = 0.9 * (double)(2 * k + 1);
    double frac = 0.1 + num / (double)(1 << (F + 1));
    double p10 = 1.0;
    for (int e = 0; e < E; ++e)
        p10 *= 10.0;
    double mag = frac / p10;
    return (is_signed && lead) ? -mag : mag;
}

int oracle_build_codebook(int is_signed, float *out256)
{
    float v[256];
    for (int p = 0; p < 256; ++p)
        v[p] = (float)pattern_value(p, is_signed);
    for (int i = 1; i < 256; ++i) {            /* insertion sort, ascending  */
        float x = v[i];
        int j = i - 1;
        while (j >= 0 && v[j] > x) {
            v[j + 1] = v[j];
            --j;
        }
        v[j + 1] = x;
    }
    for (int i = 0; i < 256; ++i)
        out256[i] = v[i];
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Nearest value (Eq. quant2): argmin_j |Q_j - x|, found by binary search.    */
/* The last decision compares x with the midpoint of the two bracketing codes */
/* exactly: both 2x and Q_j + Q_{j+1} are exact in binary64.  Equal distance  */
/* keeps the lower index (first minimum of the argmin).                       */
/* ------------------------------------------------------------------------- */
int oracle_nearest_code(const float *q, float x)
{
    if (!(x > q[0]))
        return 0;
    if (x >= q[255])
        return 255;
    int lo = 0, hi = 255;                      /* q[lo] <= x < q[hi]         */
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (q[mid] <= x)
            lo = mid;
        else
            hi = mid;
    }
    double twice = 2.0 * (double)x;
    double sum = (double)q[lo] + (double)q[hi];
    return (twice > sum) ? hi : lo;
}

/* Definition written out: scan all 256 codes, keep the first minimum.        */
int oracle_nearest_code_bruteforce(const float *q, float x)
{
    int best = 0;
    double bestd = fabs((double)q[0] - (double)x);
    for (int j = 1; j < 256; ++j) {
        double d = fabs((double)q[j] - (double)x);
        if (d < bestd) {
            bestd = d;
            best = j;
        }
    }
    return best;
}

/* ------------------------------------------------------------------------- */
/* Block-wise quantization (Sec. IV-B "Tensor chunking", Eq. quant1, quant2). */
/* The flattened tensor is cut into ceil(n/B) blocks; the last may be short.  */
/* An all-zero block stores N = 0 and the code of 0.0.                        */
/* ------------------------------------------------------------------------- */
static void quantize_block(const float *q, const float *T, int64_t len,
                           uint8_t *TQ, float *N_out)
{
    float N = 0.0f;
    for (int64_t i = 0; i < len; ++i) {
        float a = fabsf(T[i]);
        if (a > N)
            N = a;
    }
    *N_out = N;
    if (N == 0.0f) {
        uint8_t z = (uint8_t)oracle_nearest_code(q, 0.0f);
        for (int64_t i = 0; i < len; ++i)
            TQ[i] = z;
        return;
    }
    for (int64_t i = 0; i < len; ++i) {
        float x = T[i] / N;
        TQ[i] = (uint8_t)oracle_nearest_code(q, x);
    }
}

int oracle_quantize_blockwise(const float *q, const float *T, int64_t n, int B,
                              uint8_t *TQ, float *N)
{
    if (n < 0 || B <= 0)
        return -1;
    for (int64_t s = 0, b = 0; s < n; s += B, ++b) {
        int64_t len = (n - s < B) ? n - s : B;
        quantize_block(q, T + s, len, TQ + s, N + b);
    }
    return 0;
}

/* Dequantization (Eq. quant3): T^D_i = Q^map(T^Q_i) * N_b, one multiply.     */
int oracle_dequantize_blockwise(const float *q, const uint8_t *TQ, const float *N,
                                int64_t n, int B, float *TD)
{
    if (n < 0 || B <= 0)
        return -1;
    for (int64_t i = 0; i < n; ++i)
        TD[i] = q[TQ[i]] * N[i / B];
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Scalars derived from the hyper-parameters.  1 - beta1 and 1 - beta2 are    */
/* binary32 subtractions (Eq. adam as printed needs nothing else).            */
/*                                                                           */
/* Extensions outside Eq. adam (the paper trains its DF-ResNets with AdamW,   */
/* weight decay 0.05, Sec. V "Training settings", but prints neither the      */
/* decay nor a bias correction):                                              */
/*   bias correction  : the step is alpha / (1 - beta1^t) and the root of r   */
/*                      is multiplied by 1 / sqrt(1 - beta2^t); both scalars   */
/*                      are evaluated in binary64 (beta^t by the C library's  */
/*                      pow) and rounded once to binary32;                    */
/*   decoupled decay  : w <- w - (alpha * wd) * w before the step, with       */
/*                      alpha * wd one binary32 product.                      */
/* ------------------------------------------------------------------------- */
typedef struct {
    float alpha, beta1, beta2, eps, wd;
    float omb1, omb2;        /* 1 - beta1, 1 - beta2, binary32 subtraction     */
    float alpha_t, isbc2;    /* bias-corrected step and 1/sqrt(1 - beta2^t)    */
    float alpha_wd;          /* alpha * wd for decoupled decay                 */
    int flags;
} adam_scalars;

static adam_scalars adam_prepare(float alpha, float beta1, float beta2, float eps,
                                 float wd, int64_t t, int flags)
{
    adam_scalars s;
    s.alpha = alpha; s.beta1 = beta1; s.beta2 = beta2; s.eps = eps; s.wd = wd;
    s.omb1 = 1.0f - beta1;
    s.omb2 = 1.0f - beta2;
    s.flags = flags;
    s.alpha_t = alpha;
    s.isbc2 = 1.0f;
    if (flags & ORACLE_FLAG_BIAS_CORRECTION) {
        double bc1 = 1.0 - pow((double)beta1, (double)t);
        double bc2 = 1.0 - pow((double)beta2, (double)t);
        s.alpha_t = (float)((double)alpha / bc1);
        s.isbc2 = (float)(1.0 / sqrt(bc2));
    }
    s.alpha_wd = alpha * wd;
    return s;
}

/* The derived scalars, for the tests that pin them: out = {1-beta1, 1-beta2,  */
/* alpha_t, isbc2, alpha*wd}.                                                 */
int oracle_adam_scalars(float alpha, float beta1, float beta2, float eps, float wd,
                        int64_t t, int flags, float *out5)
{
    adam_scalars s = adam_prepare(alpha, beta1, beta2, eps, wd, t, flags);
    out5[0] = s.omb1; out5[1] = s.omb2; out5[2] = s.alpha_t; out5[3] = s.isbc2; out5[4] = s.alpha_wd;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* One element of Eq. adam, from 32-bit previous states.  As printed in the   */
/* paper there is no bias-correction term; (1-beta2) g^2 is ((1-beta2) g) g.  */
/* Coupled decay (g + wd*w) is applied only when wd != 0.  Every statement is */
/* one rounded binary32 operation, also in the two extensions: with bias      */
/* correction the root is first scaled (one product), then eps is added;      */
/* decoupled decay shrinks w (one product, one difference) before the step    */
/* is subtracted.                                                             */
/* ------------------------------------------------------------------------- */
static void adam_element(const adam_scalars *s, float *w, float g,
                         float m_prev, float r_prev, float *m_new, float *r_new)
{
    float wv = *w;
    if (s->wd != 0.0f && !(s->flags & ORACLE_FLAG_DECOUPLED_WD)) {
        float t0 = s->wd * wv;
        g = g + t0;
    }
    float t1 = s->beta1 * m_prev;
    float t2 = s->omb1 * g;
    float m = t1 + t2;
    float t3 = s->beta2 * r_prev;
    float t4 = s->omb2 * g;
    float t5 = t4 * g;
    float r = t3 + t5;
    float root = sqrtf(r);
    float d, u, t6;
    if (s->flags & ORACLE_FLAG_BIAS_CORRECTION) {
        float rs = root * s->isbc2;
        d = rs + s->eps;
        u = m / d;
        t6 = s->alpha_t * u;
    } else {
        d = root + s->eps;
        u = m / d;
        t6 = s->alpha * u;
    }
    if (s->wd != 0.0f && (s->flags & ORACLE_FLAG_DECOUPLED_WD)) {
        float t7 = s->alpha_wd * wv;
        wv = wv - t7;
    }
    *w = wv - t6;
    *m_new = m;
    *r_new = r;
}

/* One element of Eq. sgd; m_0 = g_0 follows from a zero previous state.      */
static void sgd_element(float alpha, float beta, float wd, float *w, float g,
                        float m_prev, float *m_new)
{
    float wv = *w;
    if (wd != 0.0f) {
        float t0 = wd * wv;
        g = g + t0;
    }
    float t1 = beta * m_prev;
    float m = t1 + g;
    float t2 = alpha * m;
    *w = wv - t2;
    *m_new = m;
}

/* ------------------------------------------------------------------------- */
/* 32-bit-state updates (quantization bypassed; also the path of tensors too  */
/* small to be worth quantizing).                                             */
/* ------------------------------------------------------------------------- */
int oracle_adam32_step(float *w, const float *g, float *m, float *r, int64_t n,
                       float alpha, float beta1, float beta2, float eps,
                       float wd, int64_t t, int flags)
{
    if (n < 0)
        return -1;
    adam_scalars s = adam_prepare(alpha, beta1, beta2, eps, wd, t, flags);
    for (int64_t i = 0; i < n; ++i)
        adam_element(&s, &w[i], g[i], m[i], r[i], &m[i], &r[i]);
    return 0;
}

int oracle_sgd32_step(float *w, const float *g, float *m, int64_t n,
                      float alpha, float beta, float wd)
{
    if (n < 0)
        return -1;
    for (int64_t i = 0; i < n; ++i)
        sgd_element(alpha, beta, wd, &w[i], g[i], m[i], &m[i]);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* 8-bit steps (Sec. IV-B last paragraph; order from Sec. I): states go       */
/* 8-bit -> 32-bit, the weights are updated with the new 32-bit states, and   */
/* the new states are quantized block by block.                               */
/* ------------------------------------------------------------------------- */
#define ORACLE_MAX_B 65536

int oracle_adam8bit_step(float *w, const float *g,
                         uint8_t *m_q, uint8_t *r_q, float *N_m, float *N_r,
                         const float *q_signed, const float *q_unsigned,
                         int64_t n, int B,
                         float alpha, float beta1, float beta2, float eps,
                         float wd, int64_t t, int flags)
{
    static _Thread_local float mbuf[ORACLE_MAX_B], rbuf[ORACLE_MAX_B];
    if (n < 0 || B <= 0 || B > ORACLE_MAX_B)
        return -1;
    adam_scalars s = adam_prepare(alpha, beta1, beta2, eps, wd, t, flags);
    for (int64_t st = 0, b = 0; st < n; st += B, ++b) {
        int64_t len = (n - st < B) ? n - st : B;
        for (int64_t i = 0; i < len; ++i) {
            float m_prev = q_signed[m_q[st + i]] * N_m[b];
            float r_prev = q_unsigned[r_q[st + i]] * N_r[b];
            adam_element(&s, &w[st + i], g[st + i], m_prev, r_prev, &mbuf[i], &rbuf[i]);
        }
        quantize_block(q_signed, mbuf, len, m_q + st, N_m + b);
        quantize_block(q_unsigned, rbuf, len, r_q + st, N_r + b);
    }
    return 0;
}

/* For the parity report: the normalized new states x = m / N_m', y = r / N_r'  */
/* of ONE block (len <= B entries), exactly as oracle_adam8bit_step forms them   */
/* before the nearest-value search; nothing is modified.  (0 where N' = 0.)      */
int oracle_adam8bit_block_normalized(const float *w, const float *g,
                                     const uint8_t *m_q, const uint8_t *r_q, float N_m, float N_r,
                                     const float *q_signed, const float *q_unsigned, int len,
                                     float alpha, float beta1, float beta2, float eps,
                                     float wd, int64_t t, int flags, float *x_out, float *y_out)
{
    if (len < 0 || len > ORACLE_MAX_B)
        return -1;
    adam_scalars s = adam_prepare(alpha, beta1, beta2, eps, wd, t, flags);
    float Nm_new = 0.0f, Nr_new = 0.0f;
    for (int i = 0; i < len; ++i) {
        float m_prev = q_signed[m_q[i]] * N_m;
        float r_prev = q_unsigned[r_q[i]] * N_r;
        float wv = w[i];
        adam_element(&s, &wv, g[i], m_prev, r_prev, &x_out[i], &y_out[i]);
        if (fabsf(x_out[i]) > Nm_new)
            Nm_new = fabsf(x_out[i]);
        if (fabsf(y_out[i]) > Nr_new)
            Nr_new = fabsf(y_out[i]);
    }
    for (int i = 0; i < len; ++i) {
        x_out[i] = (Nm_new == 0.0f) ? 0.0f : x_out[i] / Nm_new;
        y_out[i] = (Nr_new == 0.0f) ? 0.0f : y_out[i] / Nr_new;
    }
    return 0;
}

int oracle_sgd8bit_step(float *w, const float *g, uint8_t *m_q, float *N_m,
                        const float *q_signed, int64_t n, int B,
                        float alpha, float beta, float wd)
{
    static _Thread_local float mbuf[ORACLE_MAX_B];
    if (n < 0 || B <= 0 || B > ORACLE_MAX_B)
        return -1;
    for (int64_t st = 0, b = 0; st < n; st += B, ++b) {
        int64_t len = (n - st < B) ? n - st : B;
        for (int64_t i = 0; i < len; ++i) {
            float m_prev = q_signed[m_q[st + i]] * N_m[b];
            sgd_element(alpha, beta, wd, &w[st + i], g[st + i], m_prev, &mbuf[i]);
        }
        quantize_block(q_signed, mbuf, len, m_q + st, N_m + b);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Extension outside the paper: weights and gradients stored as bfloat16      */
/* (the upper 16 bits of a binary32: 1 sign, 8 exponent, 7 fraction bits).    */
/* A stored value is widened exactly, the step runs in binary32 exactly as    */
/* above, and the new weight is rounded to nearest-even bfloat16.  The 8-bit  */
/* states and their block maxima are unaffected by the storage type.          */
/* ------------------------------------------------------------------------- */
float oracle_bf16_to_f32(uint16_t h)
{
    union { uint32_t u; float f; } v;
    v.u = (uint32_t)h << 16;
    return v.f;
}

/* Round to nearest, ties to the even 16-bit pattern: the 16 discarded bits    */
/* are compared with one half (0x8000).  Overflow carries into the exponent   */
/* and ends at infinity, as IEEE rounding requires; NaN stays NaN (quiet).    */
uint16_t oracle_f32_to_bf16(float f)
{
    union { uint32_t u; float f; } v;
    v.f = f;
    uint32_t hi = v.u >> 16, lo = v.u & 0xffffu;
    if ((v.u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)(hi | 0x0040u);
    if (lo > 0x8000u || (lo == 0x8000u && (hi & 1u)))
        hi += 1;
    return (uint16_t)hi;
}

/* IEEE binary16 (1 sign, 5 exponent, 10 fraction bits) storage: same contract as    */
/* bfloat16 above -- exact widening, one round-to-nearest-even of the new weight.    */
float oracle_f16_to_f32(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, f = h & 0x3ff;
    double v;
    if (e == 0x1f)
        v = f ? (double)NAN : (double)INFINITY;
    else if (e == 0)
        v = ldexp((double)f, -24);                     /* subnormal: f * 2^-24        */
    else
        v = ldexp((double)(1024 + f), e - 25);         /* (1 + f/1024) * 2^(e-15)     */
    return (float)(sign ? -v : v);                     /* every binary16 is a binary32 */
}

/* Nearest binary16 to a finite binary32, ties to even: scale |x| so that one unit  */
/* is the spacing of binary16 at that magnitude (2^-24 below 2^-14, else 2^(e-10)),  */
/* round the scaled value to an integer with ties to even, and rebuild the pattern;  */
/* a carry out of the fraction moves to the next exponent, past 65504 to infinity.   */
uint16_t oracle_f32_to_f16(float x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0;
    double a = fabs((double)x);
    if (isnan(x))
        return (uint16_t)(sign | 0x7e00u);
    if (isinf(x))
        return (uint16_t)(sign | 0x7c00u);
    int e;                                             /* a = m * 2^e, m in [0.5, 1)   */
    (void)frexp(a, &e);
    int E = e - 1;                                     /* a in [2^E, 2^(E+1))          */
    if (a == 0.0 || E < -14)
        E = -14;                                       /* subnormal spacing 2^-24      */
    double units = ldexp(a, 10 - E);                   /* exact: a power-of-two scale  */
    double fl = floor(units), frac = units - fl;
    long k = (long)fl;
    if (frac > 0.5 || (frac == 0.5 && (k & 1)))
        k += 1;
    /* k in [0, 2048]: value = k * 2^(E-10) */
    if (k == 2048) {                                   /* carried into the next binade */
        k = 1024;
        E += 1;
    }
    if (k < 1024)                                      /* subnormal (only when E = -14) */
        return (uint16_t)(sign | (uint16_t)k);
    if (E > 15)
        return (uint16_t)(sign | 0x7c00u);
    return (uint16_t)(sign | (uint16_t)((E + 15) << 10) | (uint16_t)(k - 1024));
}

enum { STORE_BF16 = 0, STORE_F16 = 1 };

static float widen(uint16_t h, int kind)
{
    return kind == STORE_F16 ? oracle_f16_to_f32(h) : oracle_bf16_to_f32(h);
}

static uint16_t narrow(float x, int kind)
{
    return kind == STORE_F16 ? oracle_f32_to_f16(x) : oracle_f32_to_bf16(x);
}

static int adam8bit_step_lowp(uint16_t *w, const uint16_t *g, int kind,
                              uint8_t *m_q, uint8_t *r_q, float *N_m, float *N_r,
                              const float *q_signed, const float *q_unsigned,
                              int64_t n, int B,
                              float alpha, float beta1, float beta2, float eps,
                              float wd, int64_t t, int flags)
{
    static _Thread_local float mbuf[ORACLE_MAX_B], rbuf[ORACLE_MAX_B];
    if (n < 0 || B <= 0 || B > ORACLE_MAX_B)
        return -1;
    adam_scalars s = adam_prepare(alpha, beta1, beta2, eps, wd, t, flags);
    for (int64_t st = 0, b = 0; st < n; st += B, ++b) {
        int64_t len = (n - st < B) ? n - st : B;
        for (int64_t i = 0; i < len; ++i) {
            float m_prev = q_signed[m_q[st + i]] * N_m[b];
            float r_prev = q_unsigned[r_q[st + i]] * N_r[b];
            float w32 = widen(w[st + i], kind);
            adam_element(&s, &w32, widen(g[st + i], kind), m_prev, r_prev, &mbuf[i], &rbuf[i]);
            w[st + i] = narrow(w32, kind);
        }
        quantize_block(q_signed, mbuf, len, m_q + st, N_m + b);
        quantize_block(q_unsigned, rbuf, len, r_q + st, N_r + b);
    }
    return 0;
}

static int sgd8bit_step_lowp(uint16_t *w, const uint16_t *g, int kind, uint8_t *m_q, float *N_m,
                             const float *q_signed, int64_t n, int B,
                             float alpha, float beta, float wd)
{
    static _Thread_local float mbuf[ORACLE_MAX_B];
    if (n < 0 || B <= 0 || B > ORACLE_MAX_B)
        return -1;
    for (int64_t st = 0, b = 0; st < n; st += B, ++b) {
        int64_t len = (n - st < B) ? n - st : B;
        for (int64_t i = 0; i < len; ++i) {
            float m_prev = q_signed[m_q[st + i]] * N_m[b];
            float w32 = widen(w[st + i], kind);
            sgd_element(alpha, beta, wd, &w32, widen(g[st + i], kind), m_prev, &mbuf[i]);
            w[st + i] = narrow(w32, kind);
        }
        quantize_block(q_signed, mbuf, len, m_q + st, N_m + b);
    }
    return 0;
}

int oracle_adam8bit_step_bf16(uint16_t *w, const uint16_t *g,
                              uint8_t *m_q, uint8_t *r_q, float *N_m, float *N_r,
                              const float *q_signed, const float *q_unsigned, int64_t n, int B,
                              float alpha, float beta1, float beta2, float eps, float wd, int64_t t, int flags)
{
    return adam8bit_step_lowp(w, g, STORE_BF16, m_q, r_q, N_m, N_r, q_signed, q_unsigned, n, B,
                              alpha, beta1, beta2, eps, wd, t, flags);
}

int oracle_adam8bit_step_f16(uint16_t *w, const uint16_t *g,
                             uint8_t *m_q, uint8_t *r_q, float *N_m, float *N_r,
                             const float *q_signed, const float *q_unsigned, int64_t n, int B,
                             float alpha, float beta1, float beta2, float eps, float wd, int64_t t, int flags)
{
    return adam8bit_step_lowp(w, g, STORE_F16, m_q, r_q, N_m, N_r, q_signed, q_unsigned, n, B,
                              alpha, beta1, beta2, eps, wd, t, flags);
}

int oracle_sgd8bit_step_bf16(uint16_t *w, const uint16_t *g, uint8_t *m_q, float *N_m,
                             const float *q_signed, int64_t n, int B, float alpha, float beta, float wd)
{
    return sgd8bit_step_lowp(w, g, STORE_BF16, m_q, N_m, q_signed, n, B, alpha, beta, wd);
}

int oracle_sgd8bit_step_f16(uint16_t *w, const uint16_t *g, uint8_t *m_q, float *N_m,
                            const float *q_signed, int64_t n, int B, float alpha, float beta, float wd)
{
    return sgd8bit_step_lowp(w, g, STORE_F16, m_q, N_m, q_signed, n, B, alpha, beta, wd);
}
