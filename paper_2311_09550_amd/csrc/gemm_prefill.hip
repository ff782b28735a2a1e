// LDS-staged W4A8 GEMM for large M (the context-decoding stage, which the paper
// calls computationally intensive: Sec. 4.1).  Time goes to the int8 matrix
// cores, so the kernel is built to keep them fed:
//
//   * v_mfma_i32_32x32x32_i8 is the instruction that reaches the chip's int8
//     peak (the 16x16x64 form issues at roughly half that rate), so an output
//     tile is made of 32 x 32 MFMA tiles;
//   * a workgroup of WM x WN waves owns a (32*MTW*WM) x (32*NTW*WN) output tile
//     and walks K in steps of 128;
//   * both operands are staged in LDS through registers, double buffered, one
//     barrier per step.  Activations are byte-permuted once on their way into
//     LDS; weights stay PACKED in LDS (half the bytes, half the LDS traffic)
//     and are converted in registers right before the MFMA with the sign-bit
//     placement of Sec. 5.3 -- the fused conversion of Fig. 4(c);
//   * 16-byte LDS slots are XOR-swizzled by the row so that the rows one
//     ds_read_b128 touches fall into different banks;
//   * workgroup ids are remapped so that each XCD (one L2 each) works on a
//     contiguous range of weight slabs and on all M tiles of a slab together;
//   * the epilogue applies Eq. (6),(7) to the finished int32 sums and writes fp16.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = kPrefillBK;  // 128 activations = 128 bytes of A, 64 bytes of packed B per row

// D(32x32,int32) += A(32x32,int8) * B(32x32,int8).  Lane l supplies row (l & 31) of A and column (l & 31) of B,
// 16 bytes of K group (l >> 5); it receives D[8*(v/4) + 4*(l >> 5) + (v%4)][l & 31] in register v.
__device__ __forceinline__ v16i mfma_i8_32x32x32(v4i a, v4i b, v16i c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

// 16-byte slots of a 128-byte activation row / a 64-byte packed weight row, swizzled so that 8 as well as 16
// consecutive rows reading the same logical slot hit different banks.
__device__ __forceinline__ int a_slot(int row, int col) {
    return row * 128 + ((col ^ (((row >> 1) & 7) ^ ((row & 1) << 2))) << 4);
}
__device__ __forceinline__ int b_slot(int row, int col) {
    return row * 64 + ((col ^ (((row >> 2) & 3) ^ (((row >> 1) & 1) << 1))) << 4);
}

}  // namespace

template <int MTW, int NTW, int WM, int WN, bool ACC_OUT>
__global__ __launch_bounds__(64 * WM * WN, 2) void gemm_prefill_kernel(PrefillArgs p) {
    constexpr int kThreads = 64 * WM * WN;
    constexpr int BM = 32 * MTW * WM;
    constexpr int BN = 32 * NTW * WN;
    constexpr int A_CHUNKS = BM * 8;  // 16-byte chunks per k step
    constexpr int B_CHUNKS = BN * 4;
    constexpr int A_PER = (A_CHUNKS + kThreads - 1) / kThreads;
    constexpr int B_PER = (B_CHUNKS + kThreads - 1) / kThreads;
    __shared__ __attribute__((aligned(16))) uint8_t lds_a[2][BM * 128];
    __shared__ __attribute__((aligned(16))) uint8_t lds_b[2][BN * 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN;  // wave row (M direction)
    const int wn = wave % WN;  // wave column (N direction)
    const int idx = lane & 31;
    const int g = lane >> 5;

    // XCD-aware tile order: workgroup b runs on XCD (b & 7); give each XCD a contiguous run of tiles,
    // M tiles of one weight slab adjacent.
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_n = logical / p.tiles_m;
    const int tile_m = logical - tile_n * p.tiles_m;
    const int bm0 = tile_m * BM;
    const int bn0 = tile_n * BN;

    const int kt_total = (p.K + kBK - 1) / kBK;

    // Both operands are fetched with buffer loads whose per-lane byte offsets do not depend on the k step (the step
    // enters as the scalar offset), so the loop spends no vector instructions on addresses or bounds: a chunk of a
    // row past M or N sits at an offset beyond the buffer, which reads as zero.  Only a last, partial k step
    // (K % 128 != 0) needs its own offsets, with the chunks past K sent beyond the buffer as well.
    constexpr unsigned kNowhere = 0xFFFFFFF0u;
    const __amdgpu_buffer_rsrc_t a_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.xq, 0, (unsigned)((size_t)p.M * p.K), 0x00020000);
    const __amdgpu_buffer_rsrc_t b_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, (unsigned)((size_t)p.N * (p.K >> 1)), 0x00020000);
    const int k_last = (kt_total - 1) * kBK;  // first k of the last step
    unsigned a_off[A_PER], a_off_last[A_PER], b_off[B_PER], b_off_last[B_PER];
    int a_dst[A_PER], b_dst[B_PER];  // LDS destinations of this thread's chunks (the same for every step)
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int c = tid + i * kThreads;
        const int row = c >> 3, col = c & 7;
        const int m = bm0 + row;
        const bool ok = c < A_CHUNKS && m < p.M;
        a_off[i] = ok ? (unsigned)m * (unsigned)p.K + col * 16 : kNowhere;
        a_off_last[i] = (ok && k_last + col * 16 < p.K) ? a_off[i] : kNowhere;
        a_dst[i] = a_slot(row, col);
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
        const int c = tid + i * kThreads;
        const int row = c >> 2, col = c & 3;
        const int n = bn0 + row;
        const bool ok = c < B_CHUNKS && n < p.N;
        b_off[i] = ok ? (unsigned)n * (unsigned)(p.K >> 1) + col * 16 : kNowhere;
        b_off_last[i] = (ok && k_last + col * 32 < p.K) ? b_off[i] : kNowhere;
        b_dst[i] = b_slot(row, col);
    }

    v4u areg[A_PER];
    v4u breg[B_PER];

    auto load_global = [&](int kt) {
        if (kt + 1 < kt_total) {  // uniform: not the last step
#pragma unroll
            for (int i = 0; i < A_PER; ++i) areg[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, a_off[i], kt * kBK, 0);
#pragma unroll
            for (int i = 0; i < B_PER; ++i) breg[i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, b_off[i], kt * (kBK / 2), 0);
        } else {
#pragma unroll
            for (int i = 0; i < A_PER; ++i) areg[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, a_off_last[i], kt * kBK, 0);
#pragma unroll
            for (int i = 0; i < B_PER; ++i)
                breg[i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, b_off_last[i], kt * (kBK / 2), 0);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i)
            if (tid + i * kThreads < A_CHUNKS) *(v4i *)(&lds_a[buf][a_dst[i]]) = x_operand(areg[i]);
#pragma unroll
        for (int i = 0; i < B_PER; ++i)
            if (tid + i * kThreads < B_CHUNKS) *(v4u *)(&lds_b[buf][b_dst[i]]) = breg[i];
    };

    v16i acc[MTW][NTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int t = 0; t < NTW; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][t][v] = 0;

    const int a_row0 = wm * (32 * MTW) + idx;
    const int b_row0 = wn * (32 * NTW) + idx;

    // A k step of 128 is four MFMA steps of 32: step j = 2s + h.  Lane group g holds the 32 weights of 16-byte chunk
    // (2s + g) of the packed row; their halves h = 0, 1 feed one MFMA step each, against activation chunk 2*(2s+g)+h.
    // The LDS reads run one MFMA step ahead of the MFMAs that use them, and the hand-over to the next k step (LDS
    // store, barrier, first reads from the new buffer) sits in front of the last MFMA step, whose operands are already
    // in registers: LDS latency and the barrier are covered by matrix work instead of being waited for.
    auto read_x = [&](v4i(&dst)[MTW], int buf, int j) {
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
            dst[mt] = *(const v4i *)(&lds_a[buf][a_slot(a_row0 + 32 * mt, 2 * (2 * (j >> 1) + g) + (j & 1))]);
    };
    auto read_w = [&](v4u(&dst)[NTW], int buf, int s) {
#pragma unroll
        for (int t = 0; t < NTW; ++t) dst[t] = *(const v4u *)(&lds_b[buf][b_slot(b_row0 + 32 * t, 2 * s + g)]);
    };
    auto mfma_step = [&](const v4i(&x)[MTW], const v4u(&w)[NTW], int h) {
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
            const v4i wop = h == 0 ? w_operand(w[t].x, w[t].y) : w_operand(w[t].z, w[t].w);
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) acc[mt][t] = mfma_i8_32x32x32(wop, x[mt], acc[mt][t]);
        }
    };

    load_global(0);
    store_lds(0);
    __syncthreads();

    v4i x0[MTW], x1[MTW];
    v4u w0[NTW], w1[NTW];
    read_x(x0, 0, 0);
    read_w(w0, 0, 0);
    int buf = 0;
    for (int kt = 0; kt < kt_total; ++kt) {
        const bool more = kt + 1 < kt_total;
        if (more) load_global(kt + 1);

        read_x(x1, buf, 1);
        mfma_step(x0, w0, 0);  // step 0
        read_x(x0, buf, 2);
        read_w(w1, buf, 1);
        mfma_step(x1, w0, 1);  // step 1
        read_x(x1, buf, 3);
        mfma_step(x0, w1, 0);  // step 2
        if (more) {
            store_lds(buf ^ 1);
            __syncthreads();
            read_x(x0, buf ^ 1, 0);
            read_w(w0, buf ^ 1, 0);
        }
        mfma_step(x1, w1, 1);  // step 3
        buf ^= 1;
    }

    // epilogue: lane holds, per (mt, t, quad), four consecutive n of one m
    const bool vec_ok = (p.ldc & 3) == 0;
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int m = bm0 + wm * (32 * MTW) + 32 * mt + idx;
        if (m >= p.M) continue;
        const float sa = ACC_OUT ? 0.f : p.s_a[m];
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = bn0 + wn * (32 * NTW) + 32 * t + 8 * q + 4 * g;
                if (n >= p.N) continue;
                const v4i s = v4i{acc[mt][t][4 * q], acc[mt][t][4 * q + 1], acc[mt][t][4 * q + 2], acc[mt][t][4 * q + 3]};
                if (ACC_OUT) {
                    int *dst = p.acc_out + (size_t)m * p.ldc + n;
                    const v4i v = v4i{s.x >> 4, s.y >> 4, s.z >> 4, s.w >> 4};  // exact: every sum is a multiple of 16
                    if (vec_ok && n + 3 < p.N) {
                        *(v4i *)dst = v;
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (n + j < p.N) dst[j] = v[j];
                    }
                } else {
                    unsigned short *dst = (unsigned short *)p.out + (size_t)m * p.ldc + n;
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
        }
    }
}

template <int MTW, int NTW, int WM, int WN>
static hipError_t launch_tile(PrefillArgs p, bool acc_out, hipStream_t stream) {
    constexpr int BM = 32 * MTW * WM, BN = 32 * NTW * WN;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    const int total = p.tiles_m * p.tiles_n;
    dim3 grid(8 * ((total + 7) / 8));
    dim3 block(64 * WM * WN);
    if (acc_out)
        hipLaunchKernelGGL((gemm_prefill_kernel<MTW, NTW, WM, WN, true>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((gemm_prefill_kernel<MTW, NTW, WM, WN, false>), grid, block, 0, stream, p);
    return hipGetLastError();
}

static hipError_t launch_slice(const PrefillArgs &p, bool acc_out, int tile, hipStream_t stream) {
    switch (tile) {
        case kPrefillTile128x256: return launch_tile<4, 2, 1, 4>(p, acc_out, stream);
        case kPrefillTile128x128: return launch_tile<2, 2, 2, 2>(p, acc_out, stream);
        case kPrefillTile128x160: return launch_tile<1, 5, 4, 1>(p, acc_out, stream);
        case kPrefillTile128x256Square: return launch_tile<2, 4, 2, 2>(p, acc_out, stream);
        default: return hipErrorInvalidConfiguration;
    }
}

// The kernel addresses its operands with 32-bit byte offsets; a problem whose activation or weight matrix is
// larger than that is cut into row slices of M and N, one launch each (the slices write disjoint parts of the output).
hipError_t launch_gemm_prefill(const PrefillArgs &p, bool acc_out, int tile, hipStream_t stream) {
    const long long kMaxBytes = 0xF0000000ll;
    long long m_rows = kMaxBytes / p.K, n_rows = kMaxBytes / (p.K >> 1);
    m_rows -= m_rows % 256;
    n_rows -= n_rows % 1280;  // a multiple of every tile width
    for (long long n0 = 0; n0 < p.N; n0 += n_rows) {
        for (long long m0 = 0; m0 < p.M; m0 += m_rows) {
            PrefillArgs q = p;
            q.M = (int)((p.M - m0) < m_rows ? (p.M - m0) : m_rows);
            q.N = (int)((p.N - n0) < n_rows ? (p.N - n0) : n_rows);
            q.xq = p.xq + (size_t)m0 * p.K;
            q.wp = p.wp + (size_t)n0 * (p.K >> 1);
            if (p.s_a) q.s_a = p.s_a + m0;
            if (p.s_w) q.s_w = p.s_w + n0;
            if (p.out) q.out = (unsigned short *)p.out + (size_t)m0 * p.ldc + n0;
            if (p.acc_out) q.acc_out = p.acc_out + (size_t)m0 * p.ldc + n0;
            const hipError_t e = tile >= kPrefillDma128x256 ? launch_prefill_dma_slice(q, acc_out, tile, stream)
                                                            : launch_slice(q, acc_out, tile, stream);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace w4a8
