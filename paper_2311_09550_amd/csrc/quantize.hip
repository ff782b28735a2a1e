// Row-wise kernels around the GEMM: the per-token activation quantiser, the
// offline per-channel weight quantiser + packer, and the SiLU*up glue.
// All three are one pass over HBM; a workgroup owns one row.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

constexpr int kRowThreads = 256;
constexpr int kCache = 8;  // 16-byte chunks a thread keeps in registers between the two passes (K <= 16384)

__device__ __forceinline__ float half_bits_to_float(unsigned short h) { return __half2float(__ushort_as_half(h)); }

// absolute maximum of eight fp16 values held in four words
__device__ __forceinline__ float absmax8(v4u c, float m) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        m = fmaxf(m, fabsf(half_bits_to_float((unsigned short)(c[j] & 0xFFFFu))));
        m = fmaxf(m, fabsf(half_bits_to_float((unsigned short)(c[j] >> 16))));
    }
    return m;
}

// maximum over the workgroup; every thread gets the result
__device__ __forceinline__ float block_max(float v, float *scratch) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    float m = scratch[0];
#pragma unroll
    for (int w = 1; w < kRowThreads / 64; ++w) m = fmaxf(m, scratch[w]);
    return m;
}

// Eq. (2) with zero point 0: divide by the scale in fp32 (IEEE division), round half to even, clamp.
__device__ __forceinline__ int quant_code(float x, float scale, float lo, float hi) {
    float q = __fdiv_rn(x, scale);
    q = rintf(q);
    q = fminf(fmaxf(q, lo), hi);
    return (int)q;
}

}  // namespace

// Per-token symmetric int8 quantisation (Sec. 3 "per token"; Eq. (2), z = 0).
__global__ __launch_bounds__(kRowThreads) void quantize_act_kernel(const uint16_t *__restrict__ x, int8_t *__restrict__ xq,
                                                                   float *__restrict__ s_a, int K) {
    __shared__ float scratch[kRowThreads / 64];
    const int m = blockIdx.x;
    const int chunks = K >> 3;  // 8 fp16 = 16 bytes
    const v4u *src = (const v4u *)(x + (size_t)m * K);

    v4u cache[kCache];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < kCache; ++i) {
        const int c = threadIdx.x + i * kRowThreads;
        cache[i] = v4u{0, 0, 0, 0};
        if (c < chunks) cache[i] = src[c];
        amax = absmax8(cache[i], amax);
    }
    for (int c = threadIdx.x + kCache * kRowThreads; c < chunks; c += kRowThreads) amax = absmax8(src[c], amax);
    amax = block_max(amax, scratch);

    const float scale = __fdiv_rn(amax, 127.0f);
    if (threadIdx.x == 0) s_a[m] = scale;  // amax == 0 gives scale 0
    const bool zero_row = amax == 0.f;

    v2u *dst = (v2u *)(xq + (size_t)m * K);
    auto emit = [&](int c, v4u v) {
        v2u o = v2u{0, 0};
        if (!zero_row) {
            int q[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                q[2 * j] = quant_code(half_bits_to_float((unsigned short)(v[j] & 0xFFFFu)), scale, -127.f, 127.f);
                q[2 * j + 1] = quant_code(half_bits_to_float((unsigned short)(v[j] >> 16)), scale, -127.f, 127.f);
            }
            o.x = (q[0] & 255) | ((q[1] & 255) << 8) | ((q[2] & 255) << 16) | ((unsigned)(q[3] & 255) << 24);
            o.y = (q[4] & 255) | ((q[5] & 255) << 8) | ((q[6] & 255) << 16) | ((unsigned)(q[7] & 255) << 24);
        }
        dst[c] = o;
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
__global__ __launch_bounds__(kRowThreads) void quantize_weights_kernel(const uint16_t *__restrict__ w, uint8_t *__restrict__ wp,
                                                                       float *__restrict__ s_w, int K) {
    __shared__ float scratch[kRowThreads / 64];
    const int n = blockIdx.x;
    const int chunks = K >> 3;
    const v4u *src = (const v4u *)(w + (size_t)n * K);

    float amax = 0.f;
    for (int c = threadIdx.x; c < chunks; c += kRowThreads) amax = absmax8(src[c], amax);
    amax = block_max(amax, scratch);

    const float scale = __fdiv_rn(amax, 7.0f);
    if (threadIdx.x == 0) s_w[n] = scale;
    const bool zero_row = amax == 0.f;

    unsigned *dst = (unsigned *)(wp + (size_t)n * (K >> 1));
    for (int c = threadIdx.x; c < chunks; c += kRowThreads) {
        const v4u v = src[c];
        unsigned o = 0;
        if (!zero_row) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int q0 = quant_code(half_bits_to_float((unsigned short)(v[j] & 0xFFFFu)), scale, -8.f, 7.f);
                const int q1 = quant_code(half_bits_to_float((unsigned short)(v[j] >> 16)), scale, -8.f, 7.f);
                o |= (unsigned)((q0 & 15) | ((q1 & 15) << 4)) << (8 * j);
            }
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
    v4u o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float y[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const float gt = half_bits_to_float((unsigned short)(e ? gv[j] >> 16 : gv[j] & 0xFFFFu));
            const float up = half_bits_to_float((unsigned short)(e ? uv[j] >> 16 : uv[j] & 0xFFFFu));
            y[e] = __fdiv_rn(gt, 1.0f + expf(-gt)) * up;
        }
        o[j] = pack_f16x2(y[0], y[1]);
    }
    *((v4u *)(h + (size_t)m * I) + c) = o;
}

hipError_t launch_quantize_act(const void *x, int8_t *xq, float *s_a, int M, int K, hipStream_t stream) {
    hipLaunchKernelGGL(quantize_act_kernel, dim3(M), dim3(kRowThreads), 0, stream, (const uint16_t *)x, xq, s_a, K);
    return hipGetLastError();
}

hipError_t launch_quantize_weights(const void *w, uint8_t *wp, float *s_w, int N, int K, hipStream_t stream) {
    hipLaunchKernelGGL(quantize_weights_kernel, dim3(N), dim3(kRowThreads), 0, stream, (const uint16_t *)w, wp, s_w, K);
    return hipGetLastError();
}

hipError_t launch_silu_mul(const void *gate_up, void *h, int M, int I, hipStream_t stream) {
    const int chunks = I >> 3;
    dim3 grid((chunks + kRowThreads - 1) / kRowThreads, M);
    hipLaunchKernelGGL(silu_mul_kernel, grid, dim3(kRowThreads), 0, stream, (const uint16_t *)gate_up, (uint16_t *)h, I);
    return hipGetLastError();
}

}  // namespace w4a8
