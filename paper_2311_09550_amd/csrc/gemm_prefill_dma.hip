// LDS-staged W4A8 GEMM for large M, operands brought into LDS by the memory pipeline itself.
//
// Same tiling and arithmetic as gemm_prefill_kernel (32x32x32 int8 MFMA tiles, packed weights in LDS, fused
// conversion of Fig. 4(c), dequantising epilogue of Eq. (6),(7)); what differs is how a k step reaches LDS:
//
//   * `buffer_load_dwordx4 ... lds` writes 64 lanes x 16 bytes straight into LDS (base + lane*16), so there is no
//     register staging, no ds_write and no wait for global data in front of a store.  Four stages of 64 k each form a
//     ring; the loads of stage t+3 are issued while stage t is multiplied, which covers L2 as well as HBM latency;
//   * the XOR swizzle that keeps ds_read_b128 free of bank conflicts is applied on the GLOBAL side: lane (row, slot)
//     fetches the chunk that belongs into that physical slot, so the linear LDS image is already swizzled;
//   * the activation bytes are permuted to the weights' even/odd k order after the LDS read (they cannot be touched
//     on the way in any more);
//   * one barrier per stage, placed between the stage's two MFMA steps; the reads for the next MFMA step are always
//     issued before the current step's MFMAs.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;

constexpr int kStageK = 64;  // k per stage: 64 bytes of an activation row, 32 bytes of a packed weight row
constexpr int kStages = 4;

__device__ __forceinline__ v16i mfma32(v4i a, v4i b, v16i c) { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }

// swizzles of the 16-byte slots of a 64-byte activation row (4 slots) and a 32-byte weight row (2 slots): 8 as well
// as 16 consecutive rows reading the same logical slot fall into different banks
__device__ __forceinline__ int fa(int row) { return ((row >> 2) & 3) ^ (((row >> 1) & 1) << 1); }
__device__ __forceinline__ int fb(int row) { return ((row >> 3) & 1) ^ ((row >> 2) & 1); }

// s_waitcnt that waits for the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

}  // namespace

template <int MTW, int NTW, int WM, int WN, bool ACC_OUT>
__global__ __launch_bounds__(64 * WM * WN, 2) void gemm_prefill_dma_kernel(PrefillArgs p) {
    constexpr int kWaves = WM * WN;
    constexpr int BM = 32 * MTW * WM;
    constexpr int BN = 32 * NTW * WN;
    constexpr int A_LOADS = (BM / 16 + kWaves - 1) / kWaves;  // wave loads (16 rows x 64 B) per wave and stage
    constexpr int B_LOADS = (BN / 32 + kWaves - 1) / kWaves;  // wave loads (32 rows x 32 B) per wave and stage
    constexpr int kLoads = A_LOADS + B_LOADS;                 // the same for every wave: the waits count on it
    constexpr int A_STAGE = A_LOADS * kWaves * 1024;
    constexpr int B_STAGE = B_LOADS * kWaves * 1024;
    __shared__ __attribute__((aligned(1024))) uint8_t lds_a[kStages][A_STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t lds_b[kStages][B_STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int idx = lane & 31;
    const int g = lane >> 5;

    // XCD-aware tile order (see gemm_prefill_kernel)
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_n = logical / p.tiles_m;
    const int tile_m = logical - tile_n * p.tiles_m;
    const int bm0 = tile_m * BM;
    const int bn0 = tile_n * BN;

    const int st_total = (p.K + kStageK - 1) / kStageK;  // stages to walk
    const int k_last = (st_total - 1) * kStageK;

    constexpr unsigned kNowhere = 0xFFFFFFF0u;
    // buffer resources (base, no stride, size in bytes, raw 32-bit format) for the two operands, kept in scalar registers
    auto make_rsrc = [](const void *base, size_t bytes) {
        const unsigned long long b = (unsigned long long)base;
        v4i r;
        r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)b);
        r.y = __builtin_amdgcn_readfirstlane((int)(unsigned)((b >> 32) & 0xFFFFu));
        r.z = __builtin_amdgcn_readfirstlane((int)(unsigned)bytes);
        r.w = 0x00020000;
        return r;
    };
    const v4i a_rsrc = make_rsrc(p.xq, (size_t)p.M * p.K);
    const v4i b_rsrc = make_rsrc(p.wp, (size_t)p.N * (p.K >> 1));

    // Per-lane byte offsets of this wave's loads (independent of the stage, which enters as the scalar offset).
    // Wave load L of the activation tile covers rows 16L .. 16L+15: lane -> row 16L + lane/4, physical slot lane%4.
    // Wave load L of the weight tile covers rows 32L .. 32L+31: lane -> row 32L + lane/2, physical slot lane%2.
    unsigned a_off[A_LOADS], a_off_last[A_LOADS], b_off[B_LOADS], b_off_last[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int row = 16 * (i * kWaves + wave) + (lane >> 2);
        const int col = (lane & 3) ^ fa(row);
        const int m = bm0 + row;
        const bool ok = row < BM && m < p.M;
        a_off[i] = ok ? (unsigned)m * (unsigned)p.K + col * 16 : kNowhere;
        a_off_last[i] = (ok && k_last + col * 16 < p.K) ? a_off[i] : kNowhere;
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        const int row = 32 * (i * kWaves + wave) + (lane >> 1);
        const int col = (lane & 1) ^ fb(row);
        const int n = bn0 + row;
        const bool ok = row < BN && n < p.N;
        b_off[i] = ok ? (unsigned)n * (unsigned)(p.K >> 1) + col * 16 : kNowhere;
        b_off_last[i] = (ok && k_last + col * 32 < p.K) ? b_off[i] : kNowhere;
    }

    // issue the kLoads loads of stage st into ring slot st % kStages (nothing is issued past the last stage, so
    // that the outstanding-load count the waits rely on is the same arithmetic for every stage: see below)
    // The load is written in assembly on purpose: the compiler orders LDS reads after every LDS-writing load it knows
    // of (it cannot tell the ring slots apart) and would wait for the stage just requested before each fragment read.
    // Here the ordering is explicit instead: wait_vmcnt + barrier before a slot is read, barrier before it is refilled.
    auto dma16 = [](const v4i &rsrc, unsigned lds_addr, unsigned voffset, int soffset) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
                     : "memory", "m0");
    };
    auto lds_addr = [](const void *ptr) { return (unsigned)(unsigned long long)(lds_ptr_t)ptr; };
    auto issue = [&](int st) {
        const int slot = st & (kStages - 1);
        const bool last = st + 1 >= st_total;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            dma16(a_rsrc, __builtin_amdgcn_readfirstlane(lds_addr(&lds_a[slot][(i * kWaves + wave) * 1024])),
                  last ? a_off_last[i] : a_off[i], st * kStageK);
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            dma16(b_rsrc, __builtin_amdgcn_readfirstlane(lds_addr(&lds_b[slot][(i * kWaves + wave) * 1024])),
                  last ? b_off_last[i] : b_off[i], st * (kStageK / 2));
    };

    v16i acc[MTW][NTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int t = 0; t < NTW; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][t][v] = 0;

    // LDS addresses of this lane's fragments (stage-independent part)
    int xa[MTW][2], wa[NTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int row = wm * (32 * MTW) + 32 * mt + idx;
#pragma unroll
        for (int h = 0; h < 2; ++h) xa[mt][h] = row * 64 + (((2 * g + h) ^ fa(row)) << 4);
    }
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        const int row = wn * (32 * NTW) + 32 * t + idx;
        wa[t] = row * 32 + ((g ^ fb(row)) << 4);
    }
    auto read_x = [&](v4u(&dst)[MTW], int slot, int h) {
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) dst[mt] = *(const v4u *)(&lds_a[slot][xa[mt][h]]);
    };
    auto read_w = [&](v4u(&dst)[NTW], int slot) {
#pragma unroll
        for (int t = 0; t < NTW; ++t) dst[t] = *(const v4u *)(&lds_b[slot][wa[t]]);
    };
    auto mfma_step = [&](const v4u(&x)[MTW], const v4u(&w)[NTW], int h) {
        v4i xop[MTW];
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) xop[mt] = x_operand(x[mt]);
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
            const v4i wop = h == 0 ? w_operand(w[t].x, w[t].y) : w_operand(w[t].z, w[t].w);
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) acc[mt][t] = mfma32(wop, xop[mt], acc[mt][t]);
        }
    };

    // Prologue: stages 0 .. kStages-2 go out; stage 0 must have landed (in every wave) before the first read.
#pragma unroll
    for (int s = 0; s < kStages - 1; ++s)
        if (s < st_total) issue(s);
    // Loads return in order, so "at most n outstanding" means all but the youngest n have landed.  Stages past the
    // end are simply not issued; waiting for fewer outstanding loads than necessary is always safe, so the waits below
    // use the count that holds in the steady state and fall back to "all landed" near the end.
    if (st_total >= kStages - 1)
        wait_vmcnt<(kStages - 2) * kLoads>();
    else
        wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();

    v4u x0[MTW], x1[MTW], w0[NTW], w1[NTW];
    read_x(x0, 0, 0);
    read_w(w0, 0);
    // one stage: w_cur holds its weights, w_nxt receives those of the following stage
    auto stage = [&](int st, const v4u(&w_cur)[NTW], v4u(&w_nxt)[NTW]) {
        const int slot = st & (kStages - 1);
        const int next = (st + 1) & (kStages - 1);
        // step 0 of this stage; the second half of its activations is fetched meanwhile
        read_x(x1, slot, 1);
        mfma_step(x0, w_cur, 0);
        // stage st+1 has to be in LDS, for every wave, before its first fragments are read; every wave is also done
        // reading stage st-1 (its last reads were waited for before its MFMAs), so that slot can be refilled
        if (st + 2 < st_total)
            wait_vmcnt<(kStages - 3) * kLoads>();  // stage st+2 may still be in flight
        else
            wait_vmcnt<0>();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        if (st + kStages - 1 < st_total) issue(st + kStages - 1);
        if (st + 1 < st_total) {
            read_x(x0, next, 0);
            read_w(w_nxt, next);
        }
        mfma_step(x1, w_cur, 1);
    };
    for (int st = 0; st < st_total; st += 2) {
        stage(st, w0, w1);
        if (st + 1 < st_total) stage(st + 1, w1, w0);
    }
    wait_vmcnt<0>();

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
static hipError_t launch_dma_tile(PrefillArgs p, bool acc_out, hipStream_t stream) {
    constexpr int BM = 32 * MTW * WM, BN = 32 * NTW * WN;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    const int total = p.tiles_m * p.tiles_n;
    dim3 grid(8 * ((total + 7) / 8));
    dim3 block(64 * WM * WN);
    if (acc_out)
        hipLaunchKernelGGL((gemm_prefill_dma_kernel<MTW, NTW, WM, WN, true>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((gemm_prefill_dma_kernel<MTW, NTW, WM, WN, false>), grid, block, 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_prefill_dma_slice(const PrefillArgs &p, bool acc_out, int tile, hipStream_t stream) {
    switch (tile) {
        case kPrefillDma128x256: return launch_dma_tile<4, 2, 1, 4>(p, acc_out, stream);
        case kPrefillDma128x256Square: return launch_dma_tile<2, 4, 2, 2>(p, acc_out, stream);
        case kPrefillDma128x160: return launch_dma_tile<1, 5, 4, 1>(p, acc_out, stream);
        case kPrefillDma128x128: return launch_dma_tile<2, 2, 2, 2>(p, acc_out, stream);
        default: return hipErrorInvalidConfiguration;
    }
}

}  // namespace w4a8
