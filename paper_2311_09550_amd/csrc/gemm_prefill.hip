// LDS-staged W4A8 GEMM for large M (the context-decoding stage, which the paper
// calls computationally intensive: Sec. 4.1).  Time goes to the int8 matrix
// cores, so the kernel is built to keep them fed:
//
//   * a workgroup of four waves (2 x 2) owns a (32*MTW) x (32*NTW) output tile
//     and walks K in steps of 128;
//   * both operands are staged in LDS through registers, double buffered, one
//     barrier per step.  Activations are byte-permuted once on their way into
//     LDS; weights stay PACKED in LDS (half the bytes, half the LDS traffic)
//     and are converted in registers right before the MFMA with the sign-bit
//     placement of Sec. 5.3 -- the fused conversion of Fig. 4(c);
//   * 16-byte LDS slots are XOR-swizzled by the row so that the 16 rows a
//     ds_read_b128 touches fall into different banks;
//   * workgroup ids are remapped so that each XCD (one L2 each) works on a
//     contiguous range of weight slabs and on all M tiles of a slab together;
//   * the epilogue applies Eq. (6),(7) to the finished int32 sums and writes fp16.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

constexpr int kThreads = 256;
constexpr int kBK = kPrefillBK;  // 128 activations = 128 bytes of A, 64 bytes of packed B per row

template <int MTW, int NTW>
struct Tile {
    static constexpr int BM = 32 * MTW;
    static constexpr int BN = 32 * NTW;
    static constexpr int A_BYTES = BM * 128;
    static constexpr int B_BYTES = BN * 64;
    static constexpr int A_CHUNKS = BM * 8;  // 16-byte chunks per k step
    static constexpr int B_CHUNKS = BN * 4;
    static constexpr int A_PER_THREAD = (A_CHUNKS + kThreads - 1) / kThreads;
    static constexpr int B_PER_THREAD = (B_CHUNKS + kThreads - 1) / kThreads;
};

__device__ __forceinline__ int a_slot(int row, int col) { return row * 128 + ((col ^ (row & 7)) << 4); }
__device__ __forceinline__ int b_slot(int row, int col) { return row * 64 + ((col ^ ((row >> 1) & 3)) << 4); }

}  // namespace

template <int MTW, int NTW, bool ACC_OUT>
__global__ __launch_bounds__(kThreads) void gemm_prefill_kernel(PrefillArgs p) {
    using TL = Tile<MTW, NTW>;
    __shared__ __attribute__((aligned(16))) uint8_t lds_a[2][TL::A_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t lds_b[2][TL::B_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1;  // wave row (M direction)
    const int wn = wave & 1;   // wave column (N direction)
    const int r = lane & 15;
    const int g = lane >> 4;

    // XCD-aware tile order: workgroup b runs on XCD (b & 7); give each XCD a contiguous run of tiles,
    // M tiles of one weight slab adjacent.
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_n = logical / p.tiles_m;
    const int tile_m = logical - tile_n * p.tiles_m;
    const int bm0 = tile_m * TL::BM;
    const int bn0 = tile_n * TL::BN;

    const int kt_total = (p.K + kBK - 1) / kBK;

    v4u areg[TL::A_PER_THREAD];
    v4u breg[TL::B_PER_THREAD];

    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < TL::A_PER_THREAD; ++i) {
            const int c = tid + i * kThreads;
            const int row = c >> 3, col = c & 7;
            const int m = bm0 + row, k = kt * kBK + col * 16;
            areg[i] = v4u{0, 0, 0, 0};
            if (c < TL::A_CHUNKS && m < p.M && k < p.K) areg[i] = *(const v4u *)(p.xq + (size_t)m * p.K + k);
        }
#pragma unroll
        for (int i = 0; i < TL::B_PER_THREAD; ++i) {
            const int c = tid + i * kThreads;
            const int row = c >> 2, col = c & 3;
            const int n = bn0 + row, kb = kt * (kBK / 2) + col * 16;
            breg[i] = v4u{0, 0, 0, 0};
            if (c < TL::B_CHUNKS && n < p.N && 2 * kb < p.K) breg[i] = *(const v4u *)(p.wp + (size_t)n * (p.K >> 1) + kb);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TL::A_PER_THREAD; ++i) {
            const int c = tid + i * kThreads;
            if (c < TL::A_CHUNKS) *(v4i *)(&lds_a[buf][a_slot(c >> 3, c & 7)]) = x_operand(areg[i]);
        }
#pragma unroll
        for (int i = 0; i < TL::B_PER_THREAD; ++i) {
            const int c = tid + i * kThreads;
            if (c < TL::B_CHUNKS) *(v4u *)(&lds_b[buf][b_slot(c >> 2, c & 3)]) = breg[i];
        }
    };

    v4i acc[MTW][NTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int t = 0; t < NTW; ++t) acc[mt][t] = v4i{0, 0, 0, 0};

    const int a_row0 = wm * (16 * MTW) + r;
    const int b_row0 = wn * (16 * NTW) + r;

    load_global(0);
    store_lds(0);
    __syncthreads();

    int buf = 0;
    for (int kt = 0; kt < kt_total; ++kt) {
        const bool more = kt + 1 < kt_total;
        if (more) load_global(kt + 1);

        v4u wpk[NTW];
#pragma unroll
        for (int t = 0; t < NTW; ++t) wpk[t] = *(const v4u *)(&lds_b[buf][b_slot(b_row0 + 16 * t, g)]);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4i xop[MTW];
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) xop[mt] = *(const v4i *)(&lds_a[buf][a_slot(a_row0 + 16 * mt, 2 * g + h)]);
#pragma unroll
            for (int t = 0; t < NTW; ++t) {
                const v4i wop = h == 0 ? w_operand(wpk[t].x, wpk[t].y) : w_operand(wpk[t].z, wpk[t].w);
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt) acc[mt][t] = mfma_i8_16x16x64(wop, xop[mt], acc[mt][t]);
            }
        }

        if (more) store_lds(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // epilogue: lane holds, per (mt, t), four consecutive n of one m
    const bool vec_ok = (p.N & 3) == 0;
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int m = bm0 + wm * (16 * MTW) + 16 * mt + r;
        if (m >= p.M) continue;
        const float sa = ACC_OUT ? 0.f : p.s_a[m];
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
            const int n = bn0 + wn * (16 * NTW) + 16 * t + 4 * g;
            if (n >= p.N) continue;
            const v4i s = acc[mt][t];
            if (ACC_OUT) {
                int *dst = p.acc_out + (size_t)m * p.N + n;
                const v4i v = v4i{s.x >> 4, s.y >> 4, s.z >> 4, s.w >> 4};
                if (vec_ok && n + 3 < p.N) {
                    *(v4i *)dst = v;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (n + j < p.N) dst[j] = v[j];
                }
            } else {
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
    }
}

hipError_t launch_gemm_prefill(const PrefillArgs &p, bool acc_out, hipStream_t stream) {
    const int total = p.tiles_m * p.tiles_n;
    dim3 grid(8 * ((total + 7) / 8));
    dim3 block(kThreads);
    if (acc_out)
        hipLaunchKernelGGL((gemm_prefill_kernel<4, 8, true>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((gemm_prefill_kernel<4, 8, false>), grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace w4a8
