/* Driver for the sanitizer run of tests/test_sanitizers.py: calls every entry point of the CPU
 * oracle (linked in as source) on small and ragged inputs whose buffers are allocated with
 * exactly the documented sizes, so that AddressSanitizer sees any access past them and
 * UndefinedBehaviorSanitizer any shift, overflow or conversion fault. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_build_codebook(int is_signed, float *out256);
int oracle_nearest_code(const float *q, float x);
int oracle_nearest_code_bruteforce(const float *q, float x);
int oracle_quantize_blockwise(const float *q, const float *T, int64_t n, int B, uint8_t *TQ, float *N);
int oracle_dequantize_blockwise(const float *q, const uint8_t *TQ, const float *N, int64_t n, int B, float *TD);
int oracle_adam32_step(float *w, const float *g, float *m, float *r, int64_t n, float alpha, float beta1, float beta2,
                       float eps, float wd, int64_t t, int flags);
int oracle_sgd32_step(float *w, const float *g, float *m, int64_t n, float alpha, float beta, float wd);
int oracle_adam_scalars(float alpha, float beta1, float beta2, float eps, float wd, int64_t t, int flags, float *out5);
int oracle_adam8bit_step(float *w, const float *g, uint8_t *m_q, uint8_t *r_q, float *N_m, float *N_r,
                         const float *qs, const float *qu, int64_t n, int B, float alpha, float beta1, float beta2,
                         float eps, float wd, int64_t t, int flags);
int oracle_sgd8bit_step(float *w, const float *g, uint8_t *m_q, float *N_m, const float *qs, int64_t n, int B,
                        float alpha, float beta, float wd);
int oracle_adam8bit_block_normalized(const float *w, const float *g, const uint8_t *m_q, const uint8_t *r_q, float N_m,
                                     float N_r, const float *qs, const float *qu, int len, float alpha, float beta1,
                                     float beta2, float eps, float wd, int64_t t, int flags, float *x, float *y);
int oracle_adam8bit_step_bf16(uint16_t *w, const uint16_t *g, uint8_t *m_q, uint8_t *r_q, float *N_m, float *N_r,
                              const float *qs, const float *qu, int64_t n, int B, float alpha, float beta1, float beta2,
                              float eps, float wd, int64_t t, int flags);
int oracle_adam8bit_step_f16(uint16_t *w, const uint16_t *g, uint8_t *m_q, uint8_t *r_q, float *N_m, float *N_r,
                             const float *qs, const float *qu, int64_t n, int B, float alpha, float beta1, float beta2,
                             float eps, float wd, int64_t t, int flags);
int oracle_sgd8bit_step_bf16(uint16_t *w, const uint16_t *g, uint8_t *m_q, float *N_m, const float *qs, int64_t n, int B,
                             float alpha, float beta, float wd);
int oracle_sgd8bit_step_f16(uint16_t *w, const uint16_t *g, uint8_t *m_q, float *N_m, const float *qs, int64_t n, int B,
                            float alpha, float beta, float wd);
float oracle_bf16_to_f32(uint16_t h);
uint16_t oracle_f32_to_bf16(float f);
float oracle_f16_to_f32(uint16_t h);
uint16_t oracle_f32_to_f16(float f);

static uint64_t state = 12345;
static double uni(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0;
}

int main(void)
{
    float qs[256], qu[256];
    oracle_build_codebook(1, qs);
    oracle_build_codebook(0, qu);
    long checks = 0;
    for (int i = -300; i <= 300; ++i) {
        float x = (float)i / 300.0f;
        if (oracle_nearest_code(qs, x) != oracle_nearest_code_bruteforce(qs, x)) return 2;
        if (oracle_nearest_code(qu, x) != oracle_nearest_code_bruteforce(qu, x)) return 2;
        ++checks;
    }
    const int sizes[] = {0, 1, 5, 63, 64, 65, 255, 256, 257, 2047, 2048, 2049, 5000};
    const int blocks[] = {64, 256, 2048, 4096};
    for (unsigned si = 0; si < sizeof sizes / sizeof *sizes; ++si)
        for (unsigned bi = 0; bi < sizeof blocks / sizeof *blocks; ++bi) {
            const int64_t n = sizes[si];
            const int B = blocks[bi];
            const int64_t nb = (n + B - 1) / B;
            float *w = malloc(sizeof(float) * (n ? n : 1)), *g = malloc(sizeof(float) * (n ? n : 1));
            float *m = calloc(n ? n : 1, sizeof(float)), *r = calloc(n ? n : 1, sizeof(float));
            float *T = malloc(sizeof(float) * (n ? n : 1));
            uint8_t *mq = malloc(n ? n : 1), *rq = malloc(n ? n : 1);
            float *Nm = calloc(nb ? nb : 1, sizeof(float)), *Nr = calloc(nb ? nb : 1, sizeof(float));
            uint16_t *wh = malloc(2 * (n ? n : 1)), *gh = malloc(2 * (n ? n : 1));
            float *x = malloc(sizeof(float) * B), *y = malloc(sizeof(float) * B);
            memset(mq, 127, n ? n : 1);
            memset(rq, 0, n ? n : 1);
            for (int64_t i = 0; i < n; ++i) {
                w[i] = (float)(0.2 * uni() - 0.1);
                g[i] = (float)(2e-3 * uni() - 1e-3);
            }
            for (int t = 1; t <= 3; ++t) {
                for (int flags = 0; flags < 4; ++flags) {
                    oracle_adam8bit_step(w, g, mq, rq, Nm, Nr, qs, qu, n, B, 1e-3f, 0.9f, 0.999f, 1e-8f, flags ? 0.05f : 0.0f, t, flags);
                    oracle_adam32_step(w, g, m, r, n, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, t, flags);
                }
                oracle_sgd8bit_step(w, g, mq, Nm, qs, n, B, 0.1f, 0.9f, 1e-4f);
                oracle_sgd32_step(w, g, m, n, 0.1f, 0.9f, 1e-4f);
                if (n > 0) {
                    const int len = (int)(n < B ? n : B);
                    oracle_adam8bit_block_normalized(w, g, mq, rq, Nm[0], Nr[0], qs, qu, len, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.0f, t, 0, x, y);
                }
            }
            oracle_quantize_blockwise(qs, w, n, B, mq, Nm);
            oracle_dequantize_blockwise(qs, mq, Nm, n, B, T);
            for (int64_t i = 0; i < n; ++i) {
                wh[i] = oracle_f32_to_bf16(w[i]);
                gh[i] = oracle_f32_to_bf16(g[i]);
            }
            memset(rq, 0, n ? n : 1);
            oracle_adam8bit_step_bf16(wh, gh, mq, rq, Nm, Nr, qs, qu, n, B, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.0f, 1, 0);
            oracle_sgd8bit_step_bf16(wh, gh, mq, Nm, qs, n, B, 0.1f, 0.9f, 1e-4f);
            for (int64_t i = 0; i < n; ++i) {
                wh[i] = oracle_f32_to_f16(w[i]);
                gh[i] = oracle_f32_to_f16(g[i]);
            }
            oracle_adam8bit_step_f16(wh, gh, mq, rq, Nm, Nr, qs, qu, n, B, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.0f, 2, 3);
            oracle_sgd8bit_step_f16(wh, gh, mq, Nm, qs, n, B, 0.1f, 0.9f, 0.0f);
            free(w); free(g); free(m); free(r); free(T); free(mq); free(rq); free(Nm); free(Nr); free(wh); free(gh); free(x); free(y);
            ++checks;
        }
    for (uint32_t h = 0; h < 65536; ++h) {          /* every 16-bit pattern through both conversions */
        float a = oracle_bf16_to_f32((uint16_t)h), b = oracle_f16_to_f32((uint16_t)h);
        if (a == a && oracle_f32_to_bf16(a) != h) return 3;
        if (b == b && oracle_f32_to_f16(b) != h) return 4;
    }
    const float extremes[] = {0.0f, -0.0f, 1e-45f, -1e-45f, 65504.0f, 65520.0f, 1e30f, -3.4e38f, 5.96e-8f, 2.98e-8f};
    for (unsigned i = 0; i < sizeof extremes / sizeof *extremes; ++i) {
        (void)oracle_f32_to_f16(extremes[i]);
        (void)oracle_f32_to_bf16(extremes[i]);
    }
    float s5[5];
    oracle_adam_scalars(1e-3f, 0.9f, 0.999f, 1e-8f, 0.05f, 1000000000000ll, 3, s5);
    printf("oracle sanitizer driver: %ld cases ok\n", checks);
    return 0;
}
