/*
 * Sanitizer driver for the CPU oracle (test infrastructure, like the oracle itself).
 *
 * Built together with w4a8_oracle.c under -fsanitize=address,undefined and run as a plain executable on the host,
 * it calls every exported function of the oracle on small ragged shapes whose buffers are heap blocks of exactly the
 * documented size, so that an index that leaves an array, a signed overflow or a misaligned access in the oracle
 * aborts the run.  The few relations checked on the way are between independent functions of the oracle (pack and
 * unpack, the int4 sum against the int8 sum over the unpacked codes, the unsigned storage against the signed one,
 * the fine-grained sum with one group against the per-channel path); the pins against the paper live in the Python
 * tests, not here.
 *
 *   gcc -O1 -g -fno-omit-frame-pointer -fsanitize=address,undefined -fno-sanitize-recover=all -ffp-contract=off \
 *       -o oracle_selftest selftest.c w4a8_oracle.c -lm && ./oracle_selftest
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_half_to_float(const uint16_t *h, float *f, size_t n);
void oracle_float_to_half(const float *f, uint16_t *h, size_t n);
void oracle_double_to_half(const double *d, uint16_t *h, size_t n);
int oracle_pack_w4(const int8_t *wq, uint8_t *wp, int N, int K);
void oracle_unpack_w4(const uint8_t *wp, int8_t *wq, int N, int K);
int oracle_nibble_in_high_half_as_int8(unsigned nib);
void oracle_quantize_act(const uint16_t *x_half, int8_t *xq, float *s_a, int M, int K);
void oracle_quantize_weights_rtn(const uint16_t *w_half, int8_t *wq, float *s_w, int N, int K);
void oracle_quantize_weights_clip(const uint16_t *w_half, const float *gamma, const float *beta, int8_t *wq, float *s_w,
                                  int N, int K);
void oracle_gemm_acc_i32(const int8_t *xq, const uint8_t *wp, int32_t *acc, int M, int N, int K);
void oracle_gemm_acc_i32_u4(const int8_t *xq, const uint8_t *up, int32_t *acc, int M, int N, int K);
void oracle_gemm_acc_i32_w8(const int8_t *xq, const int8_t *w8, int32_t *acc, int M, int N, int K);
void oracle_quantize_weights_rtn8(const uint16_t *w_half, int8_t *wq, float *s_w, int N, int K);
void oracle_epilogue(const int32_t *acc, const float *s_a, const float *s_w, float *y32, uint16_t *out_half, int M, int N);
int oracle_gemm(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w, int32_t *acc, float *y32,
                uint16_t *out_half, int M, int N, int K);
int oracle_quantize_weights_groups(const uint16_t *w_half, int group, int8_t *wq, float *s_g, int N, int K);
int oracle_gemm_fine_grained(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_g, int group,
                             double *y64, float *y32, uint16_t *out_half, double *mag, int M, int N, int K);
void oracle_silu_mul(const uint16_t *gate_up_half, double *y64, uint16_t *h_half, int M, int I);
void oracle_add_rmsnorm(const uint16_t *x_half, const uint16_t *res_half, const uint16_t *gamma_half, double eps,
                        uint16_t *r_half, double *y64, uint16_t *y_half, int M, int K);
int oracle_num_threads(void);

static int failures;

#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            ++failures;                                   \
            fprintf(stderr, "selftest: " __VA_ARGS__);    \
            fprintf(stderr, " (%s:%d)\n", __FILE__, __LINE__); \
        }                                                 \
    } while (0)

/* exact-size heap block: one byte past it is the sanitizer's red zone */
static void *block(size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p) { fprintf(stderr, "selftest: out of memory\n"); exit(2); }
    memset(p, 0xA5, bytes);
    return p;
}

static uint32_t lcg_state = 2311u;
static uint32_t lcg(void) { lcg_state = lcg_state * 1664525u + 1013904223u; return lcg_state >> 8; }

/* finite fp16 values of mixed magnitude, with exact zeros, from the generator above */
static void fill_half(uint16_t *h, size_t n, int allow_big)
{
    float *f = (float *)block(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) {
        uint32_t r = lcg();
        float v = ((int)(r % 2001) - 1000) / 1000.0f;
        if (r % 17 == 0) v = 0.0f;
        if (allow_big && r % 29 == 0) v *= 60.0f;
        f[i] = v;
    }
    oracle_float_to_half(f, h, n);
    free(f);
}

static void one_shape(int M, int N, int K, int group)
{
    const size_t mk = (size_t)M * K, nk = (size_t)N * K, mn = (size_t)M * N;
    uint16_t *x = (uint16_t *)block(mk * 2), *w = (uint16_t *)block(nk * 2);
    fill_half(x, mk, 1);
    fill_half(w, nk, 0);
    if (M > 1) memset(x + (size_t)(M - 1) * K, 0, (size_t)K * 2);   /* an all-zero token */

    int8_t *xq = (int8_t *)block(mk);
    float *s_a = (float *)block((size_t)M * 4);
    oracle_quantize_act(x, xq, s_a, M, K);
    for (size_t i = 0; i < mk; ++i) CHECK(xq[i] >= -127, "activation code %d below -127", xq[i]);
    if (M > 1) CHECK(s_a[M - 1] == 0.0f, "all-zero token has scale %g", s_a[M - 1]);

    int8_t *wq = (int8_t *)block(nk), *wq_back = (int8_t *)block(nk), *wq_clip = (int8_t *)block(nk);
    float *s_w = (float *)block((size_t)N * 4), *s_clip = (float *)block((size_t)N * 4);
    float *gamma = (float *)block((size_t)N * 4), *beta = (float *)block((size_t)N * 4);
    oracle_quantize_weights_rtn(w, wq, s_w, N, K);
    for (int n = 0; n < N; ++n) { gamma[n] = 0.5f + (lcg() % 50) / 100.0f; beta[n] = 0.5f + (lcg() % 50) / 100.0f; }
    oracle_quantize_weights_clip(w, gamma, beta, wq_clip, s_clip, N, K);
    oracle_quantize_weights_clip(w, NULL, NULL, wq_back, s_clip, N, K);
    CHECK(memcmp(wq, wq_back, nk) == 0, "clipping with gamma = beta = 1 differs from round-to-nearest");
    for (size_t i = 0; i < nk; ++i) CHECK(wq_clip[i] >= -8 && wq_clip[i] <= 7, "clipped code %d out of range", wq_clip[i]);

    uint8_t *wp = (uint8_t *)block(nk / 2), *up = (uint8_t *)block(nk / 2);
    CHECK(oracle_pack_w4(wq, wp, N, K) == 0, "pack refused in-range codes");
    oracle_unpack_w4(wp, wq_back, N, K);
    CHECK(memcmp(wq, wq_back, nk) == 0, "unpack(pack(w)) != w");
    for (size_t i = 0; i < nk / 2; ++i) up[i] = (uint8_t)(wp[i] ^ 0x88u);   /* u = w + 8 in both nibbles */

    int32_t *acc = (int32_t *)block(mn * 4), *acc_u = (int32_t *)block(mn * 4), *acc_8 = (int32_t *)block(mn * 4);
    oracle_gemm_acc_i32(xq, wp, acc, M, N, K);
    oracle_gemm_acc_i32_u4(xq, up, acc_u, M, N, K);
    oracle_gemm_acc_i32_w8(xq, wq, acc_8, M, N, K);
    CHECK(memcmp(acc, acc_u, mn * 4) == 0, "unsigned storage gives other sums than the signed one");
    CHECK(memcmp(acc, acc_8, mn * 4) == 0, "int4 sums differ from the int8 GEMM over the unpacked codes");

    float *y32 = (float *)block(mn * 4), *y32_b = (float *)block(mn * 4);
    uint16_t *out = (uint16_t *)block(mn * 2), *out_b = (uint16_t *)block(mn * 2);
    oracle_epilogue(acc, s_a, s_w, y32, out, M, N);
    oracle_epilogue(acc, s_a, s_w, NULL, NULL, M, N);
    CHECK(oracle_gemm(xq, s_a, wp, s_w, NULL, y32_b, out_b, M, N, K) == 0, "gemm failed");
    CHECK(memcmp(y32, y32_b, mn * 4) == 0 && memcmp(out, out_b, mn * 2) == 0, "gemm != acc + epilogue");
    CHECK(oracle_gemm(xq, s_a, wp, s_w, acc_u, NULL, NULL, M, N, K) == 0, "gemm with no outputs failed");

    int8_t *w8 = (int8_t *)block(nk);
    float *s_w8 = (float *)block((size_t)N * 4);
    oracle_quantize_weights_rtn8(w, w8, s_w8, N, K);
    oracle_gemm_acc_i32_w8(xq, w8, acc_8, M, N, K);

    if (group > 0 && K % group == 0) {
        const int G = K / group;
        float *s_g = (float *)block((size_t)G * N * 4);
        double *y64 = (double *)block(mn * 8), *mag = (double *)block(mn * 8);
        CHECK(oracle_quantize_weights_groups(w, group, wq_back, s_g, N, K) == 0, "group quantiser refused K %% group == 0");
        CHECK(oracle_pack_w4(wq_back, up, N, K) == 0, "pack refused group codes");
        CHECK(oracle_gemm_fine_grained(xq, s_a, up, s_g, group, y64, y32_b, out_b, mag, M, N, K) == 0, "fine-grained gemm failed");
        CHECK(oracle_gemm_fine_grained(xq, s_a, up, s_g, group, NULL, NULL, NULL, NULL, M, N, K) == 0, "fine-grained, no outputs");
        for (size_t i = 0; i < mn; ++i) CHECK(fabs(y64[i]) <= mag[i] * (1 + 1e-12) + 1e-300, "|y| above its magnitude bound");
        /* one group spanning all of K is the per-channel recipe */
        CHECK(oracle_quantize_weights_groups(w, K, wq_back, s_clip, N, K) == 0, "group = K refused");
        CHECK(memcmp(wq, wq_back, nk) == 0, "one group over K differs from the per-channel quantiser");
        CHECK(oracle_quantize_weights_groups(w, K + 1, wq_back, s_clip, N, K) != 0, "group that does not divide K accepted");
        free(s_g); free(y64); free(mag);
    }

    free(x); free(w); free(xq); free(s_a); free(wq); free(wq_back); free(wq_clip); free(s_w); free(s_clip);
    free(gamma); free(beta); free(wp); free(up); free(acc); free(acc_u); free(acc_8); free(y32); free(y32_b);
    free(out); free(out_b); free(w8); free(s_w8);
}

int main(void)
{
    /* conversions over every fp16 bit pattern: finite values survive half -> float -> half unchanged */
    {
        const size_t n = 65536;
        uint16_t *h = (uint16_t *)block(n * 2), *back = (uint16_t *)block(n * 2);
        float *f = (float *)block(n * 4);
        double *d = (double *)block(n * 8);
        for (size_t i = 0; i < n; ++i) h[i] = (uint16_t)i;
        oracle_half_to_float(h, f, n);
        oracle_float_to_half(f, back, n);
        for (size_t i = 0; i < n; ++i)
            if ((i & 0x7C00u) != 0x7C00u) CHECK(back[i] == h[i], "fp16 %04zx does not round-trip through float", i);
        for (size_t i = 0; i < n; ++i) d[i] = isfinite(f[i]) ? (double)f[i] * (1.0 + 1e-9) : 0.0;
        oracle_double_to_half(d, back, n);
        free(h); free(back); free(f); free(d);
    }
    for (unsigned nib = 0; nib < 16; ++nib) {
        int v = oracle_nibble_in_high_half_as_int8(nib);
        CHECK(v == 16 * (nib >= 8 ? (int)nib - 16 : (int)nib), "nibble %u in the high half reads %d", nib, v);
    }
    {
        int8_t bad[2] = {8, 0};
        uint8_t byte[1];
        CHECK(oracle_pack_w4(bad, byte, 1, 2) != 0, "pack accepted the code 8");
    }
    one_shape(1, 1, 2, 2);
    one_shape(3, 5, 8, 4);
    one_shape(7, 33, 130, 26);
    one_shape(2, 17, 256, 128);
    one_shape(5, 40, 384, 128);
    {
        const int M = 3, I = 11;
        uint16_t *gu = (uint16_t *)block((size_t)M * 2 * I * 2), *h = (uint16_t *)block((size_t)M * I * 2);
        double *y = (double *)block((size_t)M * I * 8);
        fill_half(gu, (size_t)M * 2 * I, 1);
        oracle_silu_mul(gu, y, h, M, I);
        oracle_silu_mul(gu, NULL, NULL, M, I);
        for (int i = 0; i < M * I; ++i) CHECK(isfinite(y[i]), "silu(gate) * up is not finite");
        free(gu); free(h); free(y);
    }
    {
        const int M = 3, K = 37;
        uint16_t *x = (uint16_t *)block((size_t)M * K * 2), *res = (uint16_t *)block((size_t)M * K * 2);
        uint16_t *g = (uint16_t *)block((size_t)K * 2), *r = (uint16_t *)block((size_t)M * K * 2), *yh = (uint16_t *)block((size_t)M * K * 2);
        double *y = (double *)block((size_t)M * K * 8);
        fill_half(x, (size_t)M * K, 2);
        fill_half(res, (size_t)M * K, 3);
        fill_half(g, (size_t)K, 4);
        oracle_add_rmsnorm(x, res, g, 1e-5, r, y, yh, M, K);
        oracle_add_rmsnorm(x, NULL, g, 1e-5, r, NULL, NULL, M, K);
        for (int i = 0; i < M * K; ++i) CHECK(isfinite(y[i]), "RMSNorm value is not finite");
        free(x); free(res); free(g); free(r); free(yh); free(y);
    }
    CHECK(oracle_num_threads() >= 1, "thread count below one");
    if (failures) { fprintf(stderr, "oracle selftest: %d check(s) failed\n", failures); return 1; }
    puts("oracle selftest ok");
    return 0;
}
