/*
 * CPU oracle for the W4A8 linear path (per-token int8 activations x per-channel
 * int4 weights, int32 accumulation, dequantisation after the GEMM).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is a plain, slow,
 * definition-level implementation used only to check the GPU kernels and to
 * report a CPU baseline.  It shares no code, header, table or helper with the
 * HIP library and must never be called from it.
 *
 * Everything here is the *definition* written out as nested loops:
 *   - no blocking, no fusion, no reordering of the k sum,
 *   - no "times sixteen" trick for the GEMM: the nibble is sign-extended to its
 *     true value and multiplied as is, so that the GPU's high-nibble placement
 *     and later division by 16 (Sec. 5.3 "Reusing the sign bit", App. A.1) is
 *     checked against the plain result,
 *   - fp32 arithmetic is IEEE single precision (x86-64 SSE, no -ffast-math),
 *     fp16 conversions are written out bit by bit with round-half-to-even.
 *
 * Passages followed: Fig. 2 caption (X is M x K, s_a per token, s per weight
 * channel); Sec. 3 Eq. (2),(3) with z = 0 (symmetric quantise / dequantise);
 * Sec. 4.2 Eq. (6),(7) (sum over k, then one dequantisation with
 * S_ij = S_a_i * S_w_j); Sec. 5.1 Eq. (8),(9) with N = 4 bits and
 * gamma = beta = 1; Sec. 5.3 and App. A.1 (signed int4 kept as the low
 * nibble of its two's complement; int32 accumulator).
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 * low nibble = even k; weights stored N rows x K/2 bytes; activation range
 * [-127,127] with scale absmax/127; rounding is round-half-to-even; the
 * quantiser divides (x / s_a) in fp32; an all-zero token gets s_a = 0 and
 * zero codes; the scale product s_a*s_w is rounded to fp32 first, then
 * multiplied by float(acc); the output is that fp32 value rounded once to fp16.
 *
 * Build:  gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC -o liboracle.so w4a8_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ fp16 */

/* IEEE binary16 bits -> double (exact). */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24); /* subnormal or zero */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + f), e - 25);
    }
    return sign ? -v : v;
}

/* double -> IEEE binary16 bits, one rounding, round-half-to-even, gradual
 * underflow, overflow to infinity.  Scalings by powers of two are exact in
 * double and nearbyint() rounds half to even in the default rounding mode. */
static uint16_t double_to_half_bits(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v)) return 0x7e00u;
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u); /* midpoint to 2^16 rounds to inf */
    if (a < ldexp(1.0, -14)) {
        /* subnormal range: spacing 2^-24; result 1024 is the smallest normal */
        int q = (int)nearbyint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)q);
    }
    int ex;
    (void)frexp(a, &ex); /* a = f * 2^ex, f in [0.5,1) */
    int e = ex - 1;      /* a in [2^e, 2^(e+1)) */
    int q = (int)nearbyint(ldexp(a, 10 - e)); /* in [1024, 2048] */
    if (q == 2048) { q = 1024; e += 1; }
    return (uint16_t)(sign | (uint16_t)(((e + 15) << 10) + (q - 1024)));
}

void oracle_half_to_float(const uint16_t *h, float *f, size_t n)
{
    for (size_t i = 0; i < n; ++i) f[i] = (float)half_bits_to_double(h[i]);
}

void oracle_float_to_half(const float *f, uint16_t *h, size_t n)
{
    for (size_t i = 0; i < n; ++i) h[i] = double_to_half_bits((double)f[i]);
}

void oracle_double_to_half(const double *d, uint16_t *h, size_t n)
{
    for (size_t i = 0; i < n; ++i) h[i] = double_to_half_bits(d[i]);
}

/* ------------------------------------------------------- int4 pack/unpack */

/* True value of a stored nibble: the low four bits of the two's complement of
 * a number in [-8,7] (App. A.1: -7 = 1111 1001 is stored as 1001). */
static int nibble_value(unsigned nib)
{
    nib &= 15u;
    return nib >= 8u ? (int)nib - 16 : (int)nib;
}

/* wq[N][K] values in [-8,7]  ->  wp[N][K/2]; byte j of a row holds k = 2j in
 * its low nibble and k = 2j+1 in its high nibble.  Returns -1 if a value is
 * out of range or K is odd. */
int oracle_pack_w4(const int8_t *wq, uint8_t *wp, int N, int K)
{
    if (K % 2) return -1;
    for (int n = 0; n < N; ++n) {
        for (int j = 0; j < K / 2; ++j) {
            int lo = wq[(size_t)n * K + 2 * j];
            int hi = wq[(size_t)n * K + 2 * j + 1];
            if (lo < -8 || lo > 7 || hi < -8 || hi > 7) return -1;
            wp[(size_t)n * (K / 2) + j] =
                (uint8_t)(((unsigned)lo & 15u) | (((unsigned)hi & 15u) << 4));
        }
    }
    return 0;
}

void oracle_unpack_w4(const uint8_t *wp, int8_t *wq, int N, int K)
{
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            unsigned b = wp[(size_t)n * (K / 2) + (k >> 1)];
            unsigned nib = (k & 1) ? (b >> 4) : (b & 15u);
            wq[(size_t)n * K + k] = (int8_t)nibble_value(nib);
        }
    }
}

/* The paper's on-device conversion, kept here only so the tests can pin the
 * worked example of App. A.1 (nibble 1001 in the high half of a byte reads as
 * -112 = 16 * -7).  The oracle's GEMM never uses it. */
int oracle_nibble_in_high_half_as_int8(unsigned nib)
{
    uint8_t byte = (uint8_t)((nib & 15u) << 4);
    return (int)(int8_t)byte;
}

/* ----------------------------------------------------------- quantisers */

/* Per-token symmetric 8-bit quantisation (Sec. 3, "per token"; Eq. (2) with
 * z = 0): one scale per row of X. */
void oracle_quantize_act(const uint16_t *x_half, int8_t *xq, float *s_a, int M, int K)
{
    for (int m = 0; m < M; ++m) {
        float amax = 0.0f;
        for (int k = 0; k < K; ++k) {
            float v = (float)half_bits_to_double(x_half[(size_t)m * K + k]);
            float a = fabsf(v);
            if (a > amax) amax = a;
        }
        if (amax == 0.0f) {
            s_a[m] = 0.0f;
            for (int k = 0; k < K; ++k) xq[(size_t)m * K + k] = 0;
            continue;
        }
        float scale = amax / 127.0f; /* one correctly rounded fp32 division */
        s_a[m] = scale;
        for (int k = 0; k < K; ++k) {
            float v = (float)half_bits_to_double(x_half[(size_t)m * K + k]);
            float q = v / scale;     /* Eq. (2): x / scale, fp32 */
            float r = nearbyintf(q);          /* round half to even */
            if (r > 127.0f) r = 127.0f;
            if (r < -127.0f) r = -127.0f;
            xq[(size_t)m * K + k] = (int8_t)r;
        }
    }
}

/* Per-output-channel symmetric 4-bit round-to-nearest (Eq. (8),(9) with
 * N = 4 bits, gamma = beta = 1): S = max|W_row| / 7, codes clamped to [-8,7].
 * Offline step; the harness uses it to make int4 weights from fp16 ones. */
void oracle_quantize_weights_rtn(const uint16_t *w_half, int8_t *wq, float *s_w, int N, int K)
{
    for (int n = 0; n < N; ++n) {
        float wmax = -INFINITY, wmin = INFINITY;
        for (int k = 0; k < K; ++k) {
            float v = (float)half_bits_to_double(w_half[(size_t)n * K + k]);
            if (v > wmax) wmax = v;
            if (v < wmin) wmin = v;
        }
        float top = fabsf(wmax) > fabsf(wmin) ? fabsf(wmax) : fabsf(wmin);
        if (top == 0.0f) {
            s_w[n] = 0.0f;
            for (int k = 0; k < K; ++k) wq[(size_t)n * K + k] = 0;
            continue;
        }
        float scale = top / 7.0f;
        s_w[n] = scale;
        for (int k = 0; k < K; ++k) {
            float v = (float)half_bits_to_double(w_half[(size_t)n * K + k]);
            float q = v / scale;
            float r = nearbyintf(q);
            if (r > 7.0f) r = 7.0f;
            if (r < -8.0f) r = -8.0f;
            wq[(size_t)n * K + k] = (int8_t)r;
        }
    }
}

/* The same with the clipping strengths of Eq. (9) given per output channel:
 *   S = max(|gamma * max(W_row)|, |beta * min(W_row)|) / 7,  codes = clamp(rne(W / S), -8, 7)   (Eq. (8)).
 * Values outside the clipped range saturate, so -8 does occur here.  gamma or beta may be NULL (= 1). */
void oracle_quantize_weights_clip(const uint16_t *w_half, const float *gamma, const float *beta, int8_t *wq, float *s_w,
                                  int N, int K)
{
    for (int n = 0; n < N; ++n) {
        float wmax = -INFINITY, wmin = INFINITY;
        for (int k = 0; k < K; ++k) {
            float v = (float)half_bits_to_double(w_half[(size_t)n * K + k]);
            if (v > wmax) wmax = v;
            if (v < wmin) wmin = v;
        }
        float g = gamma ? gamma[n] : 1.0f, b = beta ? beta[n] : 1.0f;
        float up = fabsf(g * wmax), down = fabsf(b * wmin);
        float top = up > down ? up : down;
        if (top == 0.0f) {
            s_w[n] = 0.0f;
            for (int k = 0; k < K; ++k) wq[(size_t)n * K + k] = 0;
            continue;
        }
        float scale = top / 7.0f;
        s_w[n] = scale;
        for (int k = 0; k < K; ++k) {
            float v = (float)half_bits_to_double(w_half[(size_t)n * K + k]);
            float q = v / scale;
            float r = nearbyintf(q);
            if (r > 7.0f) r = 7.0f;
            if (r < -8.0f) r = -8.0f;
            wq[(size_t)n * K + k] = (int8_t)r;
        }
    }
}

/* ------------------------------------------------------------------ GEMM */

/* acc[m][n] = sum_k xq[m][k] * W_q[n][k]   (Eq. (6), the sum inside Dq).
 * int32 accumulation as the paper states; the caller keeps K small enough
 * (|acc| <= 128*8*K) that int32 cannot overflow. */
void oracle_gemm_acc_i32(const int8_t *xq, const uint8_t *wp, int32_t *acc, int M, int N, int K)
{
#pragma omp parallel
    {
        int8_t *wrow = (int8_t *)malloc((size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            for (int k = 0; k < K; ++k) {
                unsigned b = wp[(size_t)n * (K / 2) + (k >> 1)];
                unsigned nib = (k & 1) ? (b >> 4) : (b & 15u);
                wrow[k] = (int8_t)nibble_value(nib);
            }
            for (int m = 0; m < M; ++m) {
                int32_t s = 0;
                for (int k = 0; k < K; ++k)
                    s += (int32_t)xq[(size_t)m * K + k] * (int32_t)wrow[k];
                acc[(size_t)m * N + n] = s;
            }
        }
        free(wrow);
    }
}

/* The "vanilla" unsigned storage the paper compares against (Sec. 5.3, App. A.1, Fig. 4(b)): offline 8 is added to
 * every signed code so that it lies in [0, 15], the nibble stored is that unsigned value u, and the device subtracts
 * 8 again before multiplying:  acc[m][n] = sum_k xq[m][k] * (u[n][k] - 8).  Same packing order as the signed format. */
void oracle_gemm_acc_i32_u4(const int8_t *xq, const uint8_t *up, int32_t *acc, int M, int N, int K)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            int32_t s = 0;
            for (int k = 0; k < K; ++k) {
                unsigned b = up[(size_t)n * (K / 2) + (k >> 1)];
                int u = (int)((k & 1) ? (b >> 4) : (b & 15u));
                s += (int32_t)xq[(size_t)m * K + k] * (int32_t)(u - 8);
            }
            acc[(size_t)m * N + n] = s;
        }
    }
}

/* The W8A8 counterpart (the paper's own comparison point, Table 4): the same sum with int8 weight codes
 * w8[N][K] stored one per byte.  |acc| <= 128 * 128 * K, inside int32 for K <= 65536. */
void oracle_gemm_acc_i32_w8(const int8_t *xq, const int8_t *w8, int32_t *acc, int M, int N, int K)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            int32_t s = 0;
            for (int k = 0; k < K; ++k)
                s += (int32_t)xq[(size_t)m * K + k] * (int32_t)w8[(size_t)n * K + k];
            acc[(size_t)m * N + n] = s;
        }
    }
}

/* Per-output-channel symmetric 8-bit round-to-nearest (Eq. (8),(9) with N = 8 bits, gamma = beta = 1):
 * S = max|W_row| / 127, codes clamped to [-128, 127] (with this S the clamp never acts). */
void oracle_quantize_weights_rtn8(const uint16_t *w_half, int8_t *wq, float *s_w, int N, int K)
{
    for (int n = 0; n < N; ++n) {
        float top = 0.0f;
        for (int k = 0; k < K; ++k) {
            float v = fabsf((float)half_bits_to_double(w_half[(size_t)n * K + k]));
            if (v > top) top = v;
        }
        if (top == 0.0f) {
            s_w[n] = 0.0f;
            for (int k = 0; k < K; ++k) wq[(size_t)n * K + k] = 0;
            continue;
        }
        float scale = top / 127.0f;
        s_w[n] = scale;
        for (int k = 0; k < K; ++k) {
            float v = (float)half_bits_to_double(w_half[(size_t)n * K + k]);
            float r = nearbyintf(v / scale);
            if (r > 127.0f) r = 127.0f;
            if (r < -128.0f) r = -128.0f;
            wq[(size_t)n * K + k] = (int8_t)r;
        }
    }
}

/* y32[m][n] = float(acc[m][n]) * (s_a[m] * s_w[n])   (Eq. (6),(7); Eq. (3), z = 0)
 * out_half  = y32 rounded once to fp16.  Either output pointer may be NULL. */
void oracle_epilogue(const int32_t *acc, const float *s_a, const float *s_w,
                     float *y32, uint16_t *out_half, int M, int N)
{
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            float s_ij = s_a[m] * s_w[n];              /* Eq. (7), one fp32 rounding */
            float y = (float)acc[(size_t)m * N + n] * s_ij; /* int32->fp32 RNE, fp32 mul */
            if (y32) y32[(size_t)m * N + n] = y;
            if (out_half) out_half[(size_t)m * N + n] = double_to_half_bits((double)y);
        }
    }
}

/* Whole quantised linear: acc, then epilogue.  acc may be NULL (scratch is
 * allocated), y32 / out_half may be NULL. */
int oracle_gemm(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w,
                int32_t *acc, float *y32, uint16_t *out_half, int M, int N, int K)
{
    int32_t *a = acc ? acc : (int32_t *)malloc((size_t)M * N * sizeof(int32_t));
    if (!a) return -1;
    oracle_gemm_acc_i32(xq, wp, a, M, N, K);
    oracle_epilogue(a, s_a, s_w, y32, out_half, M, N);
    if (!acc) free(a);
    return 0;
}

/* ------------------------------------------------- fine-grained comparison */

/* Group-wise symmetric 4-bit round-to-nearest (the "g128" recipes of Table 1, Sec. 3): every run of `group`
 * consecutive k of an output channel has its own scale S = max|W| / 7 over that run (Eq. (8),(9) with gamma = beta
 * = 1 applied per group).  s_g is stored group-major: s_g[g * N + n].  K must be a multiple of group. */
int oracle_quantize_weights_groups(const uint16_t *w_half, int group, int8_t *wq, float *s_g, int N, int K)
{
    if (group <= 0 || K % group) return -1;
    for (int n = 0; n < N; ++n) {
        for (int g = 0; g < K / group; ++g) {
            const uint16_t *src = w_half + (size_t)n * K + (size_t)g * group;
            int8_t *dst = wq + (size_t)n * K + (size_t)g * group;
            float top = 0.0f;
            for (int k = 0; k < group; ++k) {
                float v = fabsf((float)half_bits_to_double(src[k]));
                if (v > top) top = v;
            }
            float scale = top / 7.0f;
            s_g[(size_t)g * N + n] = top == 0.0f ? 0.0f : scale;
            for (int k = 0; k < group; ++k) {
                float r = 0.0f;
                if (top != 0.0f) {
                    r = nearbyintf((float)half_bits_to_double(src[k]) / scale);
                    if (r > 7.0f) r = 7.0f;
                    if (r < -8.0f) r = -8.0f;
                }
                dst[k] = (int8_t)r;
            }
        }
    }
    return 0;
}

/* The fine-grained W4A8 product the paper sets its per-channel kernel against (Eq. (5), Fig. 2(b), Sec. 7.2):
 *     O[m][n] = sum_g Dq( sum_{k in group g} xq[m][k] * W_q[n][k],  s_a[m],  s_g[g][n] ),
 * an exact integer sum per group, made floating point and scaled group by group.
 *   y64  : the definition in fp64, s_a[m] * sum_g (acc_g * s_g[g][n]);
 *   y32  : the same in the fp32 arithmetic the paper names for O, in this order: f = 0; for g ascending
 *          f = fma(float(acc_g), s_g[g][n], f); y = f * s_a[m]   (the per-token factor is common to all groups
 *          and is applied once, after the sum);
 *   out_half : y32 rounded once to fp16;
 *   mag  : s_a[m] * sum_g |acc_g| * s_g[g][n] in fp64, the size a rounding-error bound is relative to.
 * Any output pointer may be NULL.  K must be a multiple of group. */
int oracle_gemm_fine_grained(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_g, int group,
                             double *y64, float *y32, uint16_t *out_half, double *mag, int M, int N, int K)
{
    if (group <= 0 || K % group) return -1;
    const int G = K / group;
#pragma omp parallel
    {
        int8_t *wrow = (int8_t *)malloc((size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            for (int k = 0; k < K; ++k) {
                unsigned b = wp[(size_t)n * (K / 2) + (k >> 1)];
                wrow[k] = (int8_t)nibble_value((k & 1) ? (b >> 4) : (b & 15u));
            }
            for (int m = 0; m < M; ++m) {
                double d = 0.0, a = 0.0;
                float f = 0.0f;
                for (int g = 0; g < G; ++g) {
                    int32_t s = 0;
                    for (int k = g * group; k < (g + 1) * group; ++k)
                        s += (int32_t)xq[(size_t)m * K + k] * (int32_t)wrow[k];
                    float sc = s_g[(size_t)g * N + n];
                    d += (double)s * (double)sc;
                    a += fabs((double)s) * fabs((double)sc);
                    f = fmaf((float)s, sc, f);
                }
                float y = f * s_a[m];
                size_t o = (size_t)m * N + n;
                if (y64) y64[o] = (double)s_a[m] * d;
                if (y32) y32[o] = y;
                if (out_half) out_half[o] = double_to_half_bits((double)y);
                if (mag) mag[o] = fabs((double)s_a[m]) * a;
            }
        }
        free(wrow);
    }
    return 0;
}

/* ------------------------------------------------------------- layer glue */

/* h[m][i] = silu(gate[m][i]) * up[m][i], gate = columns [0,I), up = columns
 * [I,2I) of gate_up[M][2I] (fp16).  Evaluated in fp64 from the exact fp16
 * inputs; y64 gets the fp64 value, h_half that value rounded once to fp16. */
void oracle_silu_mul(const uint16_t *gate_up_half, double *y64, uint16_t *h_half, int M, int I)
{
    for (int m = 0; m < M; ++m) {
        for (int i = 0; i < I; ++i) {
            double g = half_bits_to_double(gate_up_half[(size_t)m * 2 * I + i]);
            double u = half_bits_to_double(gate_up_half[(size_t)m * 2 * I + I + i]);
            double y = g / (1.0 + exp(-g)) * u;
            if (y64) y64[(size_t)m * I + i] = y;
            if (h_half) h_half[(size_t)m * I + i] = double_to_half_bits(y);
        }
    }
}

/* The operator in front of a gated MLP's first linear in a pre-norm decoder layer, whose output the per-token
 * quantiser consumes (the engine of Sec. 6.1 fuses the quantiser into such neighbours; the norm itself is LLaMA's
 * RMSNorm, not the paper's):
 *   r[m][k] = fp16( fp32(res[m][k]) + fp32(x[m][k]) )         one fp32 addition, one rounding to fp16; r = x if res is NULL
 *   y[m][k] = r[m][k] / sqrt( mean_k r[m][k]^2 + eps ) * g[k]
 * evaluated in fp64 from the fp16 values r and g; y64 gets the fp64 value, y_half that value rounded once to fp16. */
void oracle_add_rmsnorm(const uint16_t *x_half, const uint16_t *res_half, const uint16_t *gamma_half, double eps,
                        uint16_t *r_half, double *y64, uint16_t *y_half, int M, int K)
{
    for (int m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int k = 0; k < K; ++k) {
            uint16_t rb = x_half[(size_t)m * K + k];
            if (res_half) {
                float sum = (float)half_bits_to_double(res_half[(size_t)m * K + k]) + (float)half_bits_to_double(rb);
                rb = double_to_half_bits((double)sum);
            }
            r_half[(size_t)m * K + k] = rb;
            double r = half_bits_to_double(rb);
            ss += r * r;
        }
        double inv = 1.0 / sqrt(ss / (double)K + eps);
        for (int k = 0; k < K; ++k) {
            double y = half_bits_to_double(r_half[(size_t)m * K + k]) * inv * half_bits_to_double(gamma_half[k]);
            if (y64) y64[(size_t)m * K + k] = y;
            if (y_half) y_half[(size_t)m * K + k] = double_to_half_bits(y);
        }
    }
}

#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the OpenMP loops above will use (1 when built without OpenMP). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
