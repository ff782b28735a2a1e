// Weight-streaming W4A8 GEMM for small M (the self-decoding stage, which the
// paper calls memory-intensive: Sec. 4.1).  Time goes to reading the packed
// weights once from HBM, so the kernel is built around that stream:
//
//   * a workgroup owns 16*T output channels (rows of Wp) and one K slice;
//   * its waves take interleaved 128-wide k steps, so that at any moment the
//     workgroup reads a contiguous run of every row;
//   * a lane loads 16 packed bytes (32 weights) straight from global memory
//     into registers, converts them with the sign-bit placement of Sec. 5.3
//     and feeds two 16x16x64 int8 MFMAs; activations (a few KB, cache
//     resident) are loaded the same way and byte-permuted to the same k order;
//   * partial sums of the waves meet in LDS; partial sums of K slices handled
//     by different workgroups meet in the workspace, where the last workgroup
//     to arrive adds them up (integer sums: any order gives the same bits);
//   * the dequantisation of Eq. (6),(7) is applied once, by whoever holds the
//     complete sum.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

template <int MT, int T, int WAVES, int U, bool ACC_OUT>
__global__ __launch_bounds__(WAVES * 64) void gemm_decode_kernel(DecodeArgs p) {
    constexpr int kThreads = WAVES * 64;
    __shared__ v4i red[WAVES * MT * T * 64];
    __shared__ int last_flag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 15;   // row of the 16-row operand tile
    const int g = lane >> 4;   // K group of the lane
    const int n0 = blockIdx.x * (16 * T);
    const int split = blockIdx.y;

    // k steps (128 wide) of this workgroup's K slice
    const int ks_total = (p.K + 127) >> 7;
    const int ks_per = (ks_total + p.splits - 1) / p.splits;
    const int ks_begin = split * ks_per;
    const int ks_end = min(ks_total, ks_begin + ks_per);

    const size_t w_stride = (size_t)(p.K >> 1);
    const uint8_t *wrow[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        int n = min(n0 + 16 * t + r, p.N - 1);  // rows past N are read (clamped) and never written
        wrow[t] = p.wp + (size_t)n * w_stride + 16 * g;
    }
    const int8_t *xrow[MT];
    bool xvalid[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int m = 16 * mt + r;
        xvalid[mt] = m < p.M;
        xrow[mt] = p.xq + (size_t)min(m, p.M - 1) * p.K + 32 * g;
    }

    v4i acc[MT][T];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t) acc[mt][t] = v4i{0, 0, 0, 0};

    for (int ks0 = ks_begin + wave; ks0 < ks_end; ks0 += WAVES * U) {
        v4u wreg[U][T];
        v4u xreg[U][MT][2];
        // issue every load of the U steps before the first use
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ks = ks0 + u * WAVES;
            const bool live = ks < ks_end && (ks * 128 + 32 * g) < p.K;  // K % 32 == 0: a lane's group is all in or all out
#pragma unroll
            for (int t = 0; t < T; ++t) {
                wreg[u][t] = v4u{0, 0, 0, 0};
                if (live) wreg[u][t] = *(const v4u *)(wrow[t] + (size_t)ks * 64);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                xreg[u][mt][0] = v4u{0, 0, 0, 0};
                xreg[u][mt][1] = v4u{0, 0, 0, 0};
                if (live && xvalid[mt]) {
                    const v4u *px = (const v4u *)(xrow[mt] + (size_t)ks * 128);
                    xreg[u][mt][0] = px[0];
                    xreg[u][mt][1] = px[1];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i xop[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) xop[mt] = x_operand(xreg[u][mt][h]);
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    v4i wop = h == 0 ? w_operand(wreg[u][t].x, wreg[u][t].y)
                                     : w_operand(wreg[u][t].z, wreg[u][t].w);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt][t] = mfma_i8_16x16x64(wop, xop[mt], acc[mt][t]);
                }
            }
        }
    }

    // combine the waves' partial sums
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t) red[((wave * MT + mt) * T + t) * 64 + lane] = acc[mt][t];
    __syncthreads();

    // one (mt, t, lane) item = four consecutive n of one m
    constexpr int kItems = MT * T * 64;
    const bool vec_ok = (p.N & 3) == 0;

    if (p.splits > 1) {
        for (int it = tid; it < kItems; it += kThreads) {
            v4i s = red[it];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) s += red[w * kItems + it];
            const int l = it & 63, t = (it >> 6) % T, mt = (it >> 6) / T;
            const int m = 16 * mt + (l & 15);
            const int n = n0 + 16 * t + 4 * (l >> 4);
            if (m < p.M) {
                int *dst = p.partials + ((size_t)split * p.M + m) * p.N + n;
                if (vec_ok && n + 3 < p.N) {
                    *(v4i *)dst = s;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (n + j < p.N) dst[j] = s[j];
                }
            }
        }
        __threadfence();  // publish this workgroup's partial sums device-wide
        __syncthreads();
        if (tid == 0) {
            int old = atomicAdd(p.counters + blockIdx.x, 1);
            last_flag = (old == p.splits - 1);
        }
        __syncthreads();
        if (!last_flag) return;
        __threadfence();  // see the other workgroups' partial sums
    }

    for (int it = tid; it < kItems; it += kThreads) {
        const int l = it & 63, t = (it >> 6) % T, mt = (it >> 6) / T;
        const int m = 16 * mt + (l & 15);
        const int n = n0 + 16 * t + 4 * (l >> 4);
        if (m >= p.M || n >= p.N) continue;
        v4i s;
        if (p.splits > 1) {
            s = v4i{0, 0, 0, 0};
            for (int sp = 0; sp < p.splits; ++sp) {
                const int *src = p.partials + ((size_t)sp * p.M + m) * p.N + n;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < p.N) s[j] += __hip_atomic_load(src + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else {
            s = red[it];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) s += red[w * kItems + it];
        }
        if (ACC_OUT) {
            int *dst = p.acc_out + (size_t)m * p.N + n;
            v4i v = v4i{s.x >> 4, s.y >> 4, s.z >> 4, s.w >> 4};  // exact: every sum is a multiple of 16
            if (vec_ok && n + 3 < p.N) {
                *(v4i *)dst = v;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < p.N) dst[j] = v[j];
            }
        } else {
            const float sa = p.s_a[m];
            unsigned short *dst = (unsigned short *)p.out + (size_t)m * p.N + n;
            if (vec_ok && n + 3 < p.N) {
                const float4 sw = *(const float4 *)(p.s_w + n);
                v2u o;
                o.x = pack_f16x2(dequant(s.x, sa, sw.x), dequant(s.y, sa, sw.y));
                o.y = pack_f16x2(dequant(s.z, sa, sw.z), dequant(s.w, sa, sw.w));
                *(v2u *)dst = o;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < p.N) dst[j] = f32_to_f16_bits(dequant(s[j], sa, p.s_w[n + j]));
            }
        }
    }
    if (p.splits > 1 && tid == 0) atomicExch(p.counters + blockIdx.x, 0);  // leave the counter ready for the next call
}

template <int MT, int T, int WAVES, int U>
static hipError_t launch_one(const DecodeArgs &p, bool acc_out, hipStream_t stream) {
    dim3 grid((p.N + 16 * T - 1) / (16 * T), p.splits);
    dim3 block(WAVES * 64);
    if (acc_out)
        hipLaunchKernelGGL((gemm_decode_kernel<MT, T, WAVES, U, true>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((gemm_decode_kernel<MT, T, WAVES, U, false>), grid, block, 0, stream, p);
    return hipGetLastError();
}

// Rows of X handled by one MFMA column tile: MT = ceil(M/16), at most 4.
hipError_t launch_gemm_decode(const DecodeArgs &p, bool acc_out, const DecodeShape &s, hipStream_t stream) {
    const int mt = (p.M + 15) / 16;
#define W4A8_CASE(MT_, T_, WV_, U_)                                                    \
    if (mt == MT_ && s.row_tiles == T_ && s.waves == WV_)                                 \
        return launch_one<MT_, T_, WV_, U_>(p, acc_out, stream);
    W4A8_CASE(1, 1, 8, 4)
    W4A8_CASE(1, 2, 8, 4)
    W4A8_CASE(1, 4, 8, 2)
    W4A8_CASE(1, 1, 4, 4)
    W4A8_CASE(1, 2, 4, 4)
    W4A8_CASE(1, 4, 4, 2)
    W4A8_CASE(2, 1, 8, 4)
    W4A8_CASE(2, 2, 8, 2)
    W4A8_CASE(2, 1, 4, 4)
    W4A8_CASE(2, 2, 4, 2)
    W4A8_CASE(3, 1, 8, 2)
    W4A8_CASE(3, 2, 8, 2)
    W4A8_CASE(3, 1, 4, 2)
    W4A8_CASE(3, 2, 4, 2)
    W4A8_CASE(4, 1, 8, 2)
    W4A8_CASE(4, 1, 4, 2)
    W4A8_CASE(4, 2, 4, 2)
#undef W4A8_CASE
    return hipErrorInvalidConfiguration;
}

}  // namespace w4a8
