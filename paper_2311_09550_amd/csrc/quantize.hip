// Row-wise kernels around the GEMM: the per-token activation quantiser, the
// offline per-channel weight quantiser + packer, the SiLU*up glue, and the
// glue fused with the quantiser that follows it.  All are one pass over HBM;
// a workgroup owns one row.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

constexpr int kRowThreads = 256;
constexpr int kCache = 8;  // 16-byte chunks a thread keeps in registers between the two passes (K <= 16384)
constexpr int kFewRows = 128;  // token counts up to which the activation quantiser spreads a row over 1024 threads
constexpr int kSomeRows = 256;  // ... and over 512 threads (measured: 3-5 % faster than 256 threads up to 256 rows, 5 % slower at 512)

// maximum over the workgroup; every thread gets the result.  NONNEG: the values are absolute values (the wave's step
// then runs in the vector ALU instead of through six shuffles)
template <int THREADS = kRowThreads, bool NONNEG = false>
__device__ __forceinline__ float block_max(float v, float *scratch) {
    if constexpr (NONNEG) {
        v = wave_max_nonneg(v);
    } else {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    float m = scratch[0];
#pragma unroll
    for (int w = 1; w < THREADS / 64; ++w) m = fmaxf(m, scratch[w]);
    return m;
}

// fp16( silu(gate) * up ) for eight gate / up pairs, fp32 arithmetic, as four words of two fp16 each.
// silu(g) = g / (1 + e^-g) with the hardware's exp2 and reciprocal (about 1 ulp of fp32 each): the result carries a
// few ulps of fp32 error, three orders of magnitude below the fp16 rounding that follows, and the kernel stays
// bandwidth-bound (the correctly rounded library exp and division cost some 35 vector operations per element and made
// it compute-bound).  exp2 overflows to +inf for very negative g, the reciprocal of that is 0: silu(-65504) = -0.
__device__ __forceinline__ v4u silu_mul8(v4u gv, v4u uv) {
    v4u o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float y[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const float gt = e ? hi_half(gv[j]) : lo_half(gv[j]);
            const float up = e ? hi_half(uv[j]) : lo_half(uv[j]);
            y[e] = silu_mul_f32(gt, up);
        }
        o[j] = pack_f16x2(y[0], y[1]);
    }
    return o;
}

}  // namespace

// Per-token symmetric int8 quantisation (Sec. 3 "per token"; Eq. (2), z = 0).
// Rows of x are ldx elements apart (ldx = K for a dense matrix; more when x is a column slice of a wider one).
// Loads and stores carry the non-temporal hint: a row is read once and its codes are written once (measured at
// M = 1024 .. 2048, K = 5120: 8 to 11 % off the kernel's time, nothing lost at small M; the GEMM that reads the codes
// next is not slowed).  A row per wave or per two waves, several rows to a workgroup, was slower at every M tried.
// THREADS, CACHE: threads per row and chunks a thread keeps between the passes.  256 x 8 where the rows fill the chip;
// for a few rows (token generation) 1024 x 2, which shortens each thread's share of the one row its compute unit has;
// 512 x 4 in between.
template <int THREADS, int CACHE>
__global__ __launch_bounds__(THREADS, THREADS <= 256 ? 8 : 1) void quantize_act_kernel(const uint16_t *__restrict__ x, int8_t *__restrict__ xq,
                                                              float *__restrict__ s_a, int K, long long ldx) {
    constexpr int kRowThreads = THREADS, kCache = CACHE;  // shadow the file-scope defaults
    __shared__ float scratch[kRowThreads / 64];
    const int m = blockIdx.x;
    const int chunks = K >> 3;  // 8 fp16 = 16 bytes
    const v4u *src = (const v4u *)(x + (size_t)m * (size_t)ldx);

    v4u cache[kCache];
    unsigned amax2 = 0u;
#pragma unroll
    for (int i = 0; i < kCache; ++i) {
        const int c = threadIdx.x + i * kRowThreads;
        cache[i] = v4u{0, 0, 0, 0};
        if (c < chunks) cache[i] = __builtin_nontemporal_load(src + c);
        amax2 = absmax8_packed(cache[i], amax2);
    }
    for (int c = threadIdx.x + kCache * kRowThreads; c < chunks; c += kRowThreads) amax2 = absmax8_packed(src[c], amax2);
    float amax = block_max<kRowThreads, true>(absmax_packed_value(amax2), scratch);

    const RowQuantizer rq(amax, 127.0f, -127.f, 127.f);
    if (threadIdx.x == 0) s_a[m] = rq.scale;  // amax == 0 gives scale 0
    const bool zero_row = amax == 0.f;

    v2u *dst = (v2u *)(xq + (size_t)m * K);
    auto emit = [&](int c, v4u v) {
        v2u o = v2u{0, 0};
        if (!zero_row) {
            float xf[8];
            halves8(v, xf);
            o = rq.packed8_own_max(xf);
        }
        __builtin_nontemporal_store(o, dst + c);
    };
#pragma unroll
    for (int i = 0; i < kCache; ++i) {
        const int c = threadIdx.x + i * kRowThreads;
        if (c < chunks) emit(c, cache[i]);
    }
    for (int c = threadIdx.x + kCache * kRowThreads; c < chunks; c += kRowThreads) emit(c, src[c]);
}

// Per-output-channel symmetric int4 round-to-nearest (Eq. (8),(9), 4 bits, gamma = beta = 1)
// followed by the nibble packing of App. A.1 (low nibble = even k).
__global__ __launch_bounds__(kRowThreads, 8) void quantize_weights_kernel(const uint16_t *__restrict__ w, uint8_t *__restrict__ wp,
                                                                       float *__restrict__ s_w, int K) {
    __shared__ float scratch[kRowThreads / 64];
    const int n = blockIdx.x;
    const int chunks = K >> 3;
    const v4u *src = (const v4u *)(w + (size_t)n * K);

    unsigned amax2 = 0u;
    for (int c = threadIdx.x; c < chunks; c += kRowThreads) amax2 = absmax8_packed(src[c], amax2);
    float amax = block_max<kRowThreads, true>(absmax_packed_value(amax2), scratch);

    const RowQuantizer rq(amax, 7.0f, -8.f, 7.f);
    if (threadIdx.x == 0) s_w[n] = rq.scale;
    const bool zero_row = amax == 0.f;

    unsigned *dst = (unsigned *)(wp + (size_t)n * (K >> 1));
    for (int c = threadIdx.x; c < chunks; c += kRowThreads) {
        unsigned o = 0;
        if (!zero_row) {
            float xf[8];
            int q[8];
            halves8(src[c], xf);
            rq.codes8(xf, q);
#pragma unroll
            for (int j = 0; j < 4; ++j) o |= (unsigned)((q[2 * j] & 15) | ((q[2 * j + 1] & 15) << 4)) << (8 * j);
        }
        dst[c] = o;
    }
}

// The same with the clipping strengths of Eq. (9) per output channel: S = max(|gamma max(W)|, |beta min(W)|) / 7.
// Values outside the clipped range saturate at -8 / 7 (Eq. (8)).  gamma / beta may be NULL (= 1).
__global__ __launch_bounds__(kRowThreads, 8) void quantize_weights_clip_kernel(const uint16_t *__restrict__ w,
                                                                            const float *__restrict__ gamma,
                                                                            const float *__restrict__ beta,
                                                                            uint8_t *__restrict__ wp, float *__restrict__ s_w,
                                                                            int K) {
    __shared__ float scratch_hi[kRowThreads / 64];
    __shared__ float scratch_lo[kRowThreads / 64];
    const int n = blockIdx.x;
    const int chunks = K >> 3;
    const v4u *src = (const v4u *)(w + (size_t)n * K);

    float hi = -INFINITY, neg_lo = -INFINITY;  // max(W) and max(-W) = -min(W)
    for (int c = threadIdx.x; c < chunks; c += kRowThreads) {
        float xf[8];
        halves8(src[c], xf);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            hi = fmaxf(hi, xf[j]);
            neg_lo = fmaxf(neg_lo, -xf[j]);
        }
    }
    hi = block_max(hi, scratch_hi);
    neg_lo = block_max(neg_lo, scratch_lo);
    const float g = gamma ? gamma[n] : 1.0f, b = beta ? beta[n] : 1.0f;
    const float top = fmaxf(fabsf(g * hi), fabsf(b * -neg_lo));

    const RowQuantizer rq(top, 7.0f, -8.f, 7.f);
    if (threadIdx.x == 0) s_w[n] = rq.scale;
    const bool zero_row = top == 0.f;

    unsigned *dst = (unsigned *)(wp + (size_t)n * (K >> 1));
    for (int c = threadIdx.x; c < chunks; c += kRowThreads) {
        unsigned o = 0;
        if (!zero_row) {
            float xf[8];
            int q[8];
            halves8(src[c], xf);
            rq.codes8(xf, q);
#pragma unroll
            for (int j = 0; j < 4; ++j) o |= (unsigned)((q[2 * j] & 15) | ((q[2 * j + 1] & 15) << 4)) << (8 * j);
        }
        dst[c] = o;
    }
}

// h = fp16( silu(gate) * up ), gate = columns [0,I), up = columns [I,2I) of a row of gate_up.
__global__ __launch_bounds__(kRowThreads) void silu_mul_kernel(const uint16_t *__restrict__ gate_up, uint16_t *__restrict__ h,
                                                               int I) {
    const int m = blockIdx.y;
    const int c = blockIdx.x * kRowThreads + threadIdx.x;  // 8 outputs per thread
    if (c >= (I >> 3)) return;
    const v4u gv = *((const v4u *)(gate_up + (size_t)m * 2 * I) + c);
    const v4u uv = *((const v4u *)(gate_up + (size_t)m * 2 * I + I) + c);
    *((v4u *)(h + (size_t)m * I) + c) = silu_mul8(gv, uv);
}

// The glue and the quantiser behind it in one pass: h = fp16(silu(gate) * up) is formed in registers (the same
// arithmetic as silu_mul_kernel, so the same fp16 bits), then quantised per token exactly as quantize_act_kernel
// would quantise it.  The fp16 intermediate never goes to memory.  A row is spread over 1024 threads so that a
// thread holds at most two chunks of h (I <= 16384); longer rows recompute h in the second pass.  (Measured at
// M = 1024, I = 13824, cold input: 512 threads with four chunks each, two workgroups per compute unit, are 4 % slower;
// non-temporal loads and stores change nothing, in isolation or inside the layer's step.)
constexpr int kFusedThreads = 1024;
constexpr int kFusedCache = 2;

__global__ __launch_bounds__(kFusedThreads) void silu_mul_quantize_kernel(const uint16_t *__restrict__ gate_up,
                                                                          int8_t *__restrict__ xq, float *__restrict__ s_a,
                                                                          int I) {
    __shared__ float scratch[kFusedThreads / 64];
    const int m = blockIdx.x;
    const int chunks = I >> 3;
    const v4u *gate = (const v4u *)(gate_up + (size_t)m * 2 * I);
    const v4u *up = (const v4u *)(gate_up + (size_t)m * 2 * I + I);

    v4u cache[kFusedCache];
    unsigned amax2 = 0u;
#pragma unroll
    for (int i = 0; i < kFusedCache; ++i) {
        const int c = threadIdx.x + i * kFusedThreads;
        cache[i] = v4u{0, 0, 0, 0};
        if (c < chunks) cache[i] = silu_mul8(gate[c], up[c]);
        amax2 = absmax8_packed(cache[i], amax2);
    }
    for (int c = threadIdx.x + kFusedCache * kFusedThreads; c < chunks; c += kFusedThreads)
        amax2 = absmax8_packed(silu_mul8(gate[c], up[c]), amax2);
    const float amax = block_max<kFusedThreads, true>(absmax_packed_value(amax2), scratch);

    const RowQuantizer rq(amax, 127.0f, -127.f, 127.f);
    if (threadIdx.x == 0) s_a[m] = rq.scale;
    const bool zero_row = amax == 0.f;

    v2u *dst = (v2u *)(xq + (size_t)m * I);
    auto emit = [&](int c, v4u v) {
        v2u o = v2u{0, 0};
        if (!zero_row) {
            float xf[8];
            halves8(v, xf);
            o = rq.packed8_own_max(xf);
        }
        dst[c] = o;
    };
#pragma unroll
    for (int i = 0; i < kFusedCache; ++i) {
        const int c = threadIdx.x + i * kFusedThreads;
        if (c < chunks) emit(c, cache[i]);
    }
    for (int c = threadIdx.x + kFusedCache * kFusedThreads; c < chunks; c += kFusedThreads)
        emit(c, silu_mul8(gate[c], up[c]));
}

// Residual add, RMSNorm and the per-token quantiser in one pass over a row (the quantiser fused into the operator in
// front of it, Sec. 6.1; the norm is LLaMA's):
//   r = fp16(fp32(res) + fp32(x))  (r = x without a residual),  y = fp16(fp32(r) * rsqrt(mean r^2 + eps) * fp32(g)),
//   (xq, s_a) = the per-token quantiser of quantize_act_kernel applied to y.
// The mean of squares is an fp32 sum (per thread, then over the workgroup), the reciprocal square root a correctly
// rounded square root and division.  r and y are written where the caller wants them (the residual stream goes on; y
// is for inspection), otherwise the only traffic is x, res, g in and the codes out.  A thread keeps its chunks of the
// row in registers (K <= 16384); longer rows take what is beyond from r as written, or from the inputs again, with the
// same bits.  THREADS x CACHE as for the quantiser: 1024 x 2 for a few rows, 256 x 8 where the rows fill the chip.

template <int kNormThreads, int kNormCache>
__global__ __launch_bounds__(kNormThreads) void add_rmsnorm_quantize_kernel(const uint16_t *x, const uint16_t *res,
                                                                          const uint16_t *__restrict__ gamma, float eps,
                                                                          uint16_t *r_out, uint16_t *__restrict__ y_out,
                                                                          int8_t *__restrict__ xq, float *__restrict__ s_a,
                                                                          int K) {
    __shared__ float scratch[kNormThreads / 64];
    __shared__ float scratch_sum[kNormThreads / 64];
    const int m = blockIdx.x;
    const int chunks = K >> 3;
    const v4u *xs = (const v4u *)(x + (size_t)m * K);
    const v4u *rs = res ? (const v4u *)(res + (size_t)m * K) : nullptr;
    const v4u *gs = (const v4u *)gamma;
    auto r_chunk = [&](int c) { return rs ? add_halves8(rs[c], xs[c]) : xs[c]; };
    // what the later passes take for a chunk beyond the registers: r as written (r_out may be x or res themselves, which
    // this thread has then overwritten), else the same sum again
    auto r_again = [&](int c) { return r_out ? ((const v4u *)(r_out + (size_t)m * K))[c] : r_chunk(c); };

    v4u cache[kNormCache];
    float ss = 0.f;
    auto add_squares = [&](v4u r) { ss = add_squares8(r, ss); };
#pragma unroll
    for (int i = 0; i < kNormCache; ++i) {
        const int c = threadIdx.x + i * kNormThreads;
        cache[i] = v4u{0, 0, 0, 0};
        if (c < chunks) {
            cache[i] = r_chunk(c);
            if (r_out) ((v4u *)(r_out + (size_t)m * K))[c] = cache[i];
        }
        add_squares(cache[i]);
    }
    for (int c = threadIdx.x + kNormCache * kNormThreads; c < chunks; c += kNormThreads) {
        const v4u r = r_chunk(c);
        if (r_out) ((v4u *)(r_out + (size_t)m * K))[c] = r;
        add_squares(r);
    }
    // sum over the workgroup: DPP steps inside the wave, the waves' sums in wave order
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) scratch_sum[threadIdx.x >> 6] = ss;
    __syncthreads();
    float total = 0.f;
#pragma unroll
    for (int w = 0; w < kNormThreads / 64; ++w) total += scratch_sum[w];
    const float inv = rms_inverse(total, K, eps);
    auto y_chunk = [&](int c, v4u r) { return norm_scale8(r, inv, gs[c]); };
    unsigned amax2 = 0u;
#pragma unroll
    for (int i = 0; i < kNormCache; ++i) {
        const int c = threadIdx.x + i * kNormThreads;
        if (c < chunks) cache[i] = y_chunk(c, cache[i]);  // from here on the cache holds y
        amax2 = absmax8_packed(cache[i], amax2);
    }
    for (int c = threadIdx.x + kNormCache * kNormThreads; c < chunks; c += kNormThreads)
        amax2 = absmax8_packed(y_chunk(c, r_again(c)), amax2);
    const float amax = block_max<kNormThreads, true>(absmax_packed_value(amax2), scratch);

    const RowQuantizer rq(amax, 127.0f, -127.f, 127.f);
    if (threadIdx.x == 0) s_a[m] = rq.scale;
    const bool zero_row = amax == 0.f;
    v2u *dst = (v2u *)(xq + (size_t)m * K);
    auto emit = [&](int c, v4u y) {
        if (y_out) ((v4u *)(y_out + (size_t)m * K))[c] = y;
        v2u o = v2u{0, 0};
        if (!zero_row) {
            float yf[8];
            halves8(y, yf);
            o = rq.packed8_own_max(yf);
        }
        dst[c] = o;
    };
#pragma unroll
    for (int i = 0; i < kNormCache; ++i) {
        const int c = threadIdx.x + i * kNormThreads;
        if (c < chunks) emit(c, cache[i]);
    }
    for (int c = threadIdx.x + kNormCache * kNormThreads; c < chunks; c += kNormThreads) emit(c, y_chunk(c, r_again(c)));
}

hipError_t launch_add_rmsnorm_quantize(const void *x, const void *res, const void *gamma, float eps, void *r_out, void *y_out,
                                       int8_t *xq, float *s_a, int M, int K, hipStream_t stream) {
    if (M <= kFewRows)
        hipLaunchKernelGGL((add_rmsnorm_quantize_kernel<1024, 2>), dim3(M), dim3(1024), 0, stream, (const uint16_t *)x,
                           (const uint16_t *)res, (const uint16_t *)gamma, eps, (uint16_t *)r_out, (uint16_t *)y_out, xq, s_a, K);
    else
        hipLaunchKernelGGL((add_rmsnorm_quantize_kernel<kRowThreads, kCache>), dim3(M), dim3(kRowThreads), 0, stream,
                           (const uint16_t *)x, (const uint16_t *)res, (const uint16_t *)gamma, eps, (uint16_t *)r_out,
                           (uint16_t *)y_out, xq, s_a, K);
    return hipGetLastError();
}

hipError_t launch_quantize_act(const void *x, long long ldx, int8_t *xq, float *s_a, int M, int K, hipStream_t stream) {
    // up to half a row per compute unit the rows are spread over four times the threads
    if (M <= kFewRows)
        hipLaunchKernelGGL((quantize_act_kernel<1024, 2>), dim3(M), dim3(1024), 0, stream, (const uint16_t *)x, xq, s_a, K, ldx);
    else if (M <= kSomeRows)
        hipLaunchKernelGGL((quantize_act_kernel<512, 4>), dim3(M), dim3(512), 0, stream, (const uint16_t *)x, xq, s_a, K, ldx);
    else
        hipLaunchKernelGGL((quantize_act_kernel<kRowThreads, kCache>), dim3(M), dim3(kRowThreads), 0, stream, (const uint16_t *)x,
                           xq, s_a, K, ldx);
    return hipGetLastError();
}

hipError_t launch_quantize_weights(const void *w, uint8_t *wp, float *s_w, int N, int K, hipStream_t stream) {
    hipLaunchKernelGGL(quantize_weights_kernel, dim3(N), dim3(kRowThreads), 0, stream, (const uint16_t *)w, wp, s_w, K);
    return hipGetLastError();
}

hipError_t launch_quantize_weights_clip(const void *w, const float *gamma, const float *beta, uint8_t *wp, float *s_w, int N,
                                        int K, hipStream_t stream) {
    hipLaunchKernelGGL(quantize_weights_clip_kernel, dim3(N), dim3(kRowThreads), 0, stream, (const uint16_t *)w, gamma, beta,
                       wp, s_w, K);
    return hipGetLastError();
}

hipError_t launch_silu_mul(const void *gate_up, void *h, int M, int I, hipStream_t stream) {
    const int chunks = I >> 3;
    dim3 grid((chunks + kRowThreads - 1) / kRowThreads, M);
    hipLaunchKernelGGL(silu_mul_kernel, grid, dim3(kRowThreads), 0, stream, (const uint16_t *)gate_up, (uint16_t *)h, I);
    return hipGetLastError();
}

hipError_t launch_silu_mul_quantize(const void *gate_up, int8_t *xq, float *s_a, int M, int I, hipStream_t stream) {
    hipLaunchKernelGGL(silu_mul_quantize_kernel, dim3(M), dim3(kFusedThreads), 0, stream, (const uint16_t *)gate_up, xq, s_a, I);
    return hipGetLastError();
}

}  // namespace w4a8
