// Two probes that measure what the chip sustains, for the measurements to be read against: a read-only streaming
// reduction (achievable HBM read rate) and a register-resident int8 MFMA loop (achievable matrix-core rate, which on
// this chip depends on the operand values through power management).  They compute nothing the library's callers use.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ unsigned mix(unsigned x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// Every thread walks the buffer with a grid-wide stride, four 16-byte loads in flight; the xor of everything read is
// kept so that the loads cannot be dropped (it is stored only if it equals a value it practically never takes).
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const v4u *__restrict__ src, unsigned long long n16,
                                                                unsigned *__restrict__ sink) {
    const unsigned long long stride = (unsigned long long)gridDim.x * 256ull;
    unsigned acc = 0;
    for (unsigned long long i = (unsigned long long)blockIdx.x * 256ull + threadIdx.x; i < n16; i += 4 * stride) {
        v4u v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const unsigned long long j = i + u * stride;
            v[u] = j < n16 ? src[j] : v4u{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;
}

// The same reduction with the access pattern, the loads in flight per thread and the load instruction as template
// arguments, to find the read rate the chip really sustains and the pattern that reaches it:
//   PATTERN 0: grid-wide stride (all workgroups sweep the buffer together), global loads;
//           1: every workgroup owns one contiguous run of the buffer, global loads;
//           2, 3: the patterns 0, 1 with bounds-checked buffer loads (what the weight-streaming kernels use);
//           4, 5: the patterns 2, 3 with the non-temporal cache policy.
//   U loads of 16 bytes per thread are issued before the first one is used.
template <int PATTERN, int U>
__global__ __launch_bounds__(256) void probe_read_pattern_kernel(const v4u *__restrict__ src, unsigned long long n16,
                                                                 unsigned *__restrict__ sink) {
    constexpr bool kOwnRun = (PATTERN & 1) != 0;
    constexpr bool kBuffer = PATTERN >= 2;
    constexpr int kAux = PATTERN >= 4 ? 2 : 0;
    // a workgroup's share: everything (stride = the whole grid) or its own run (stride = the workgroup)
    const unsigned long long per = (n16 + gridDim.x - 1) / gridDim.x;
    const unsigned long long begin = kOwnRun ? per * blockIdx.x : 0ull;
    const unsigned long long end = kOwnRun ? (begin + per < n16 ? begin + per : n16) : n16;
    const unsigned long long stride = kOwnRun ? 256ull : (unsigned long long)gridDim.x * 256ull;
    const unsigned long long first = begin + (kOwnRun ? 0ull : (unsigned long long)blockIdx.x * 256ull) + threadIdx.x;
    // buffer loads address at most 4 GiB from their base: the probe's buffers are smaller
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)src, 0, (unsigned)(n16 * 16ull > 0xFFFFFFF0ull ? 0xFFFFFFF0ull : n16 * 16ull),
                                          0x00020000);
    unsigned acc = 0;
    for (unsigned long long i = first; i < end; i += U * stride) {
        v4u v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long j = i + u * stride;
            if (kBuffer)
                v[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, j < end ? (unsigned)(j * 16ull) : 0xFFFFFFF0u, 0, kAux);
            else
                v[u] = j < end ? src[j] : v4u{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;
}

// What one compute unit can pull in when part of what it reads sits in L2 and part comes from memory: one workgroup
// of 4 waves per compute unit, 16 loads of 16 bytes per thread in flight, `cold` read once (each workgroup its own
// run, non-temporal), `hot` (small, shared by all workgroups) read over and over.
//   MODE 0: every wave alternates cold and hot loads; 1: waves 0, 1 read cold, waves 2, 3 hot; 2: cold only; 3: hot only.
// Per iteration a workgroup reads 4096 chunks of 16 bytes: 2048 + 2048 in the mixed modes.
template <int MODE>
__global__ __launch_bounds__(256) void probe_mixed_read_kernel(const v4u *__restrict__ cold, unsigned cold_chunks_per_wg,
                                                               const v4u *__restrict__ hot, unsigned hot_chunks,
                                                               unsigned *__restrict__ sink) {
    const unsigned tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const v4u *own = cold + (size_t)blockIdx.x * cold_chunks_per_wg;
    constexpr int kLoads = 16;
    constexpr unsigned kColdPerIter = MODE == 2 ? 4096u : 2048u;
    const unsigned iters = cold_chunks_per_wg / kColdPerIter;
    v4u acc = v4u{0u, 0u, 0u, 0u};
    for (unsigned it = 0; it < iters; ++it) {
        v4u v[kLoads];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            bool from_cold;
            unsigned idx;  // within this iteration's cold (or hot) part
            if (MODE == 0) {
                from_cold = (j & 1) == 0;
                idx = (unsigned)(j >> 1) * 256u + tid;
            } else if (MODE == 1) {
                from_cold = wave < 2;
                idx = (unsigned)j * 128u + (wave & 1u) * 64u + lane;
            } else {
                from_cold = MODE == 2;
                idx = (unsigned)j * 256u + tid;
            }
            if (from_cold) {
                const unsigned k = it * kColdPerIter + idx;
                v[j] = __builtin_nontemporal_load(own + (k < cold_chunks_per_wg ? k : 0u));
            } else {
                v[j] = hot[(it * 4096u + idx + blockIdx.x * 1024u) % hot_chunks];
            }
        }
#pragma unroll
        for (int j = 0; j < kLoads; ++j) acc ^= v[j];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;
}

// 8 independent 32x32x32 int8 MFMAs per iteration on register operands (the operand shapes of the large-M kernel:
// 4 activation-like and 2 weight-like fragments).  pattern 0: small constants; 1: random bytes for the activations and
// random multiples of 16 for the weights, i.e. what the W4A8 kernel feeds the matrix cores.
__global__ __launch_bounds__(256, 2) void probe_mfma_i8_kernel(int *__restrict__ sink, int iters, int pattern) {
    v4i a[4], b[2];
    const unsigned t = threadIdx.x + blockIdx.x * 256u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) a[i][j] = pattern == 0 ? i + j : (int)mix(t * 64 + i * 4 + j + 1);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) b[i][j] = pattern == 0 ? i + j + 1 : (int)(mix(t * 64 + 32 + i * 4 + j + 1) & 0xF0F0F0F0u);
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int m = 0; m < 4; ++m)
                acc[n * 4 + m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[n], a[m], acc[n * 4 + m], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    if (s == 0x12345) sink[0] = s;
}

}  // namespace

hipError_t launch_probe_stream_read(const void *src, size_t bytes, unsigned *sink, int workgroups, hipStream_t stream) {
    hipLaunchKernelGGL(probe_stream_read_kernel, dim3(workgroups), dim3(256), 0, stream, (const v4u *)src,
                       (unsigned long long)(bytes / 16), sink);
    return hipGetLastError();
}

template <int PATTERN>
static hipError_t launch_read_pattern(const v4u *src, unsigned long long n16, unsigned *sink, int loads, int workgroups,
                                      hipStream_t stream) {
    switch (loads) {
        case 4: hipLaunchKernelGGL((probe_read_pattern_kernel<PATTERN, 4>), dim3(workgroups), dim3(256), 0, stream, src, n16, sink); break;
        case 8: hipLaunchKernelGGL((probe_read_pattern_kernel<PATTERN, 8>), dim3(workgroups), dim3(256), 0, stream, src, n16, sink); break;
        case 16: hipLaunchKernelGGL((probe_read_pattern_kernel<PATTERN, 16>), dim3(workgroups), dim3(256), 0, stream, src, n16, sink); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_probe_mixed_read(const void *cold, unsigned cold_chunks_per_wg, const void *hot, unsigned hot_chunks,
                                   unsigned *sink, int mode, int workgroups, hipStream_t stream) {
    const v4u *c = (const v4u *)cold, *h = (const v4u *)hot;
    switch (mode) {
        case 0: hipLaunchKernelGGL(probe_mixed_read_kernel<0>, dim3(workgroups), dim3(256), 0, stream, c, cold_chunks_per_wg, h, hot_chunks, sink); break;
        case 1: hipLaunchKernelGGL(probe_mixed_read_kernel<1>, dim3(workgroups), dim3(256), 0, stream, c, cold_chunks_per_wg, h, hot_chunks, sink); break;
        case 2: hipLaunchKernelGGL(probe_mixed_read_kernel<2>, dim3(workgroups), dim3(256), 0, stream, c, cold_chunks_per_wg, h, hot_chunks, sink); break;
        case 3: hipLaunchKernelGGL(probe_mixed_read_kernel<3>, dim3(workgroups), dim3(256), 0, stream, c, cold_chunks_per_wg, h, hot_chunks, sink); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_probe_read_pattern(const void *src, size_t bytes, unsigned *sink, int pattern, int loads, int workgroups,
                                     hipStream_t stream) {
    const v4u *s = (const v4u *)src;
    const unsigned long long n16 = bytes / 16;
    switch (pattern) {
        case 0: return launch_read_pattern<0>(s, n16, sink, loads, workgroups, stream);
        case 1: return launch_read_pattern<1>(s, n16, sink, loads, workgroups, stream);
        case 2: return launch_read_pattern<2>(s, n16, sink, loads, workgroups, stream);
        case 3: return launch_read_pattern<3>(s, n16, sink, loads, workgroups, stream);
        case 4: return launch_read_pattern<4>(s, n16, sink, loads, workgroups, stream);
        case 5: return launch_read_pattern<5>(s, n16, sink, loads, workgroups, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_probe_mfma_i8(int *sink, int workgroups, int iters, int pattern, hipStream_t stream) {
    hipLaunchKernelGGL(probe_mfma_i8_kernel, dim3(workgroups), dim3(256), 0, stream, sink, iters, pattern);
    return hipGetLastError();
}

}  // namespace w4a8
