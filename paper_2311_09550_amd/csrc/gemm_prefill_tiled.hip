// W4A8 GEMM for large M over weights in the tiled layout, and the kernel that produces that layout.
//
// Why another layout: for large M the kernel is bound by how fast a compute unit can pull its operand tiles out of
// L2.  A wave-wide 16-byte-per-lane load that touches 16 or 32 different cache lines (what a k slice of a row-major
// operand amounts to) moves well under half the bytes per cycle of one that touches 8 whole lines.  The activations
// can be read in whole lines as they are (a stage is 128 k = one 128-byte line per row).  The packed weights cannot
// (128 k of a row are 64 bytes), but they are static, so they are reordered once, after quantisation (the paper also
// fixes the weight format offline, Sec. 5.3), into 2 KB blocks that a stage consumes whole:
//
//   block (nb, kb) = output channels 32 nb .. 32 nb + 31, k = 128 kb .. 128 kb + 127, at byte ((nb * KB) + kb) * 2048,
//                    KB = ceil(K / 128); rows past N and k past K hold zero codes;
//   inside a block: 16-byte chunk (c, r), c = 0..3, r = 0..31, at (c * 32 + r) * 16 holds the 32 codes
//                    k = 128 kb + 32 c .. + 31 of channel 32 nb + r;
//   inside a dword (8 codes k0..k7): nibbles, low to high, hold k0 k4 k1 k5 k2 k6 k3 k7, so that
//                    (w << 4) & 0xF0F0F0F0 is {16 k0 .. 16 k3} and w & 0xF0F0F0F0 is {16 k4 .. 16 k7} as int8:
//                    the conversion of Fig. 4(c) then lands in the activations' natural k order and the
//                    activation bytes need no shuffling at all.
//
// The 32 lanes of an MFMA operand read 512 consecutive bytes of a block: no LDS bank conflicts, no swizzle.
//
// Kernel structure: a ring of STAGES stages of 128 k in LDS, filled by LDS-direct buffer loads (1 KB per wave
// instruction: 8 activation rows x 128 B, or half a weight block).  Stage t + STAGES is requested as soon as every
// wave has taken its last fragment of stage t, so STAGES - 1 stages are in flight while one is being multiplied.
// One workgroup barrier per stage; fragments for the next MFMA step are always read during the current one.
#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;

constexpr int kStageK = kTiledBlockK;

__device__ __forceinline__ v16i mfma32(v4i a, v4i b, v16i c) { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }

// Swizzle of the eight 16-byte slots of a 128-byte activation row in LDS: 8 as well as 16 consecutive rows reading
// the same logical slot fall into different banks.
__device__ __forceinline__ int fx(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// The same for the unsigned storage: each nibble holds u = w + 8 and the subtraction happens here, on four bytes at
// a time: (u + 0x78) ^ 0x80 is u - 8 as a two's-complement byte, and u + 0x78 <= 0x87 never carries into the next byte.
__device__ __forceinline__ v4i u_operand_tiled(unsigned w0, unsigned w1) {
    auto minus8 = [](unsigned bytes) { return (int)((bytes + 0x78787878u) ^ 0x80808080u); };
    v4i r;
    r.x = minus8(w0 & 0x0F0F0F0Fu);
    r.y = minus8((w0 >> 4) & 0x0F0F0F0Fu);
    r.z = minus8(w1 & 0x0F0F0F0Fu);
    r.w = minus8((w1 >> 4) & 0x0F0F0F0Fu);
    return r;
}

// nibbles k0..k7 of a row-major dword -> k0 k4 k1 k5 k2 k6 k3 k7
__device__ __forceinline__ unsigned interleave_nibbles(unsigned w) {
    unsigned lo = w & 0xFFFFu, hi = w >> 16;
    lo = (lo | (lo << 8)) & 0x00FF00FFu;
    lo = (lo | (lo << 4)) & 0x0F0F0F0Fu;
    hi = (hi | (hi << 8)) & 0x00FF00FFu;
    hi = (hi | (hi << 4)) & 0x0F0F0F0Fu;
    return lo | (hi << 4);
}

// One thread per 16-byte chunk of the tiled array.
__global__ __launch_bounds__(256) void tile_weights_kernel(const uint8_t *__restrict__ wp, uint8_t *__restrict__ wt, int N,
                                                           int K, int kb_total, long long chunks) {
    const long long q = (long long)blockIdx.x * 256 + threadIdx.x;
    if (q >= chunks) return;
    const long long block = q >> 7;
    const int c = (int)(q & 127) >> 5, r = (int)(q & 31);
    const long long nb = block / kb_total;
    const int kb = (int)(block - nb * kb_total);
    const long long n = nb * 32 + r;
    const int byte0 = kb * 64 + c * 16;  // within the row of K / 2 bytes
    v4u v = v4u{0u, 0u, 0u, 0u};
    if (n < N && byte0 < (K >> 1)) {
        v = *(const v4u *)(wp + (size_t)n * (size_t)(K >> 1) + byte0);
        v.x = interleave_nibbles(v.x);
        v.y = interleave_nibbles(v.y);
        v.z = interleave_nibbles(v.z);
        v.w = interleave_nibbles(v.w);
    }
    *(v4u *)(wt + (size_t)q * 16) = v;
}

}  // namespace

// WBITS = 4: the W4A8 kernel described above.  WBITS = 8: the W8A8 comparison variant (the paper's Table 4 sets its
// W4A8 against W8A8): int8 weight codes in blocks of 32 channels x 128 k = 4 KB, chunk (c, r), c = 0..7, at
// (c * 32 + r) * 16 holding k = 128 kb + 16 c .. + 15 of channel 32 nb + r; a fragment is an MFMA operand as it is.
// UNS (with WBITS = 4): the "vanilla" unsigned storage the paper measures FastGEMM against (Sec. 5.3, App. A.1,
// Fig. 4(b), "Asym GEMM" of Sec. 7.2): the nibbles hold u = w + 8 and 8 is subtracted from every byte after
// unpacking, 7 VALU operations per 8 weights instead of 3; the sums are then true sums, not sixteen-fold ones.
// FG (with WBITS = 4, signed): the fine-grained recipe the paper argues against (Eq. (5), Fig. 2(b), Sec. 7.2): one
// weight scale per group of 128 k and channel, p.s_w = s_g[K / 128][p.ldg].  A stage of the ring is exactly one
// group, so every stage starts its integer sums from zero and ends by folding them, converted to fp32 and multiplied
// by the group's scales, into a second, floating-point set of accumulators: per MFMA 8 extra VALU operations, twice
// the accumulator registers (which rules out the 256 x 256 tile), and one more 16-byte load per wave and stage (each
// wave brings in the 32 NTW scales it needs itself, next to its share of the operands).
// KS = 2 (signed int4, per-channel scales only): two sets of WM x WN waves share the output tile and split every
// stage's k between them (set ks takes k = 64 ks .. 64 ks + 63 of the stage, i.e. MFMA steps 2 ks and 2 ks + 1); their
// integer sums meet in LDS before the epilogue.  For tiles that a compute unit holds only once (N too small for
// more workgroups) this doubles the waves per SIMD without shrinking the tile.
// SWIGLU (signed int4, per-channel scales, fp16 output): the channels are gate and up projections interleaved
// (channel 2 i = gate_i, 2 i + 1 = up_i) and the epilogue stores h_i = fp16(silu(fp16 gate_i) * fp16 up_i) instead of the
// two values: the glue between the gate+up and the down projection done where its inputs are produced (the fusion
// across operators of Sec. 6.1).  p.out is then h [M][p.ldc], p.ldc = channels / 2; same bits as silu_mul_kernel
// gives on the unfused output.
template <int MTW, int NTW, int WM, int WN, int STAGES, bool ACC_OUT, int WBITS = 4, bool UNS = false, bool FG = false,
          int KS = 1, bool SWIGLU = false>
__global__ __launch_bounds__(64 * WM * WN * KS, 2) void gemm_prefill_tiled_kernel(PrefillArgs p) {
    static_assert(!SWIGLU || (WBITS == 4 && !UNS && !FG && !ACC_OUT), "fused SiLU * up: the plain W4A8 kernel, fp16 output");
    static_assert(KS == 1 || (KS == 2 && WBITS == 4 && !UNS && !FG && STAGES == 3), "k split: the plain W4A8 kernel only");
    static_assert(WBITS == 4 || WBITS == 8, "int4 or int8 weight codes");
    static_assert(!UNS || WBITS == 4, "the unsigned storage is a 4-bit format");
    static_assert(!FG || (WBITS == 4 && !UNS && !ACC_OUT), "group scales: signed int4 codes, fp16 output");
    constexpr bool W8 = WBITS == 8;
    constexpr bool kTrueSums = W8 || UNS;  // else every sum is sixteen times the true one
    constexpr int kBlock = kTiledBlockK * 32 * WBITS / 8;  // bytes of a weight block: 2 KB or 4 KB
    constexpr int kParts = kBlock / 1024;                  // wave loads per block
    constexpr int kOutWaves = WM * WN;     // waves that own a part of the output tile
    constexpr int kWaves = kOutWaves * KS;
    constexpr int BM = 32 * MTW * WM;
    constexpr int BN = 32 * NTW * WN;
    constexpr int A_TOTAL = BM / 8;                 // wave loads (8 rows x 128 B) of an activation stage
    constexpr int B_TOTAL = (BN / 32) * kParts;     // wave loads (1 KB of a weight block) of a weight stage
    static_assert(A_TOTAL % kWaves == 0 && (kWaves & 1) == 0, "activation loads must split evenly over an even wave count");
    constexpr int A_LOADS = A_TOTAL / kWaves;
    constexpr int B_LOADS = (B_TOTAL + kWaves - 1) / kWaves;
    constexpr bool kRagged = B_LOADS * kWaves != B_TOTAL;
    constexpr int kLoads = A_LOADS + B_LOADS + (FG ? 1 : 0);  // per wave and stage, the same for every wave: the waits count on it
    constexpr int A_STAGE = BM * 128;
    constexpr int B_STAGE = (BN / 32) * kBlock;
    constexpr int kBBase = STAGES * A_STAGE;
    constexpr int kSpare = STAGES * (A_STAGE + B_STAGE);  // 1 KB that absorbs the surplus loads of an uneven split
    constexpr int kScaleBase = kSpare + 1024;             // FG: per ring slot and wave, 32 NTW group scales
    constexpr int kScaleWave = NTW * 128;
    // behind everything else: the tile's s_a and s_w for the epilogue (see below); mirrors launch_one's layout
    constexpr int kRingBytes = STAGES * (A_STAGE + B_STAGE) + 1024 + (FG ? STAGES * kOutWaves * NTW * 128 + 1024 : 0);
    constexpr int kMeetBytes = KS == 2 ? kOutWaves * (32 * (64 * NTW + 16) + MTW * NTW * 16 * 256) : 0;
    constexpr int kEpiScales = kRingBytes > kMeetBytes ? kRingBytes : kMeetBytes;
    static_assert(kWaves * 64 >= BM && kWaves * 64 >= BN, "one thread per row and per channel of the tile");
    static_assert(STAGES >= 2 && (STAGES - 1) * kLoads < 64, "outstanding loads must fit the counter");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps LDS addresses in scalar registers
    const int ks = wave / kOutWaves;       // which half of every stage's k this wave multiplies (KS = 2)
    const int wsub = wave % kOutWaves;
    const int wm = wsub / WN;
    const int wn = wsub % WN;
    const int idx = lane & 31;
    const int g = lane >> 5;

    // XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs; consecutive tiles of one XCD share
    // their weight panel, so it is fetched into that XCD's L2 once
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_n = logical / p.tiles_m;
    const int tile_m = logical - tile_n * p.tiles_m;
    const int bm0 = tile_m * BM;
    const int bn0 = tile_n * BN;

    // The epilogue needs s_a of the tile's rows and s_w of its channels.  Fetched there, each of its passes would
    // start with a trip to memory (measured: 5 to 10 us of epilogue per tile).  So they are requested here, ahead of
    // everything, ride in two registers through the main loop and are parked in LDS when the ring has gone idle.
    float sa_mine = 0.f, sw_mine = 0.f;
    if (!ACC_OUT) {
        if (tid < BM && bm0 + tid < p.M) sa_mine = p.s_a[bm0 + tid];
        if (!FG && tid < BN && bn0 + tid < p.N) sw_mine = p.s_w[bn0 + tid];
    }

    // Split of K across workgroups (p.splits > 1, raw sums only): blockIdx.y takes the stages
    // [st_begin, st_begin + st_total) and writes its partial sums to its own M x ldc slab of acc_out.
    const int st_all = (p.K + kStageK - 1) / kStageK;
    const int st_begin = p.splits > 1 ? (int)blockIdx.y * p.stages_per_split : 0;
    const int st_total = p.splits > 1 ? min(st_all - st_begin, p.stages_per_split) : st_all;
    const int k_last = (st_all - 1) * kStageK;
    const int nb_total = (p.N + 31) >> 5;

    constexpr unsigned kNowhere = 0xFFFFFFF0u;  // beyond every buffer: such a lane fetches nothing and delivers zeros
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
    const v4i b_rsrc = make_rsrc(p.wp, (size_t)nb_total * st_all * kBlock);

    // Activation wave load L covers rows 8L .. 8L+7: lane -> row 8L + lane/8, physical slot lane%8, which receives
    // the logical chunk slot ^ fx(row).  With an even wave count fx(row) is the same for all loads of a lane.
    const int a_chunk = (lane & 7) ^ fx(8 * wave + (lane >> 3));
    const bool a_last_ok = k_last + a_chunk * 16 < p.K;
    unsigned a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int m = bm0 + 8 * (i * kWaves + wave) + (lane >> 3);
        a_off[i] = m < p.M ? (unsigned)m * (unsigned)p.K + a_chunk * 16 : kNowhere;
    }
    // Weight wave load L covers the 1 KB part L % kParts of the tile's 32-channel block L / kParts.
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        const int L = i * kWaves + wave;
        const int nb = (bn0 >> 5) + L / kParts;
        b_off[i] = (L < B_TOTAL && nb < nb_total)
                       ? ((unsigned)nb * (unsigned)st_all * kParts + (L % kParts)) * 1024u + lane * 16
                       : kNowhere;
    }
    // FG: lane L < 8 NTW of every wave fetches the scales of channels n_wave + 4 L .. + 3 of the stage's group
    // (p.ldg is a multiple of 4, so a 16-byte run lies wholly inside a row of s_g or wholly outside)
    const v4i g_rsrc = FG ? make_rsrc(p.s_w, (size_t)st_all * (size_t)p.ldg * 4) : v4i{0, 0, 0, 0};
    const int g_n = bn0 + wn * (32 * NTW) + 4 * lane;
    const unsigned g_off = (FG && g_n < p.ldg) ? (unsigned)g_n * 4u : kNowhere;

    // The load is written in assembly on purpose: the compiler orders LDS reads after every LDS-writing load it knows
    // of (it cannot tell the ring slots apart) and would wait for the stage just requested before each fragment read.
    // Here the ordering is explicit instead: wait_vmcnt + barrier before a slot is read, barrier before it is refilled.
    auto dma16 = [](const v4i &rsrc, unsigned lds_addr, unsigned voffset, int soffset) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
                     : "memory", "m0");
    };
    const unsigned lds_base = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)(lds_ptr_t)lds);
    // loads j = part, part + parts, ... of the kLoads loads of stage st (activation loads first), into ring slot `slot`
    auto issue = [&](int st_local, int slot, int part, int parts) {
        const int st = st_begin + st_local;  // position along K
        const bool last = st + 1 >= st_all;
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            if (j % parts != part) continue;
            if (j < A_LOADS) {
                dma16(a_rsrc, lds_base + slot * A_STAGE + (j * kWaves + wave) * 1024,
                      (last && !a_last_ok) ? kNowhere : a_off[j], st * kStageK);
            } else if (j < A_LOADS + B_LOADS) {
                const int i = j - A_LOADS;
                const int L = i * kWaves + wave;
                const unsigned dst = (kRagged && L >= B_TOTAL) ? kSpare : kBBase + slot * B_STAGE + L * 1024;
                dma16(b_rsrc, lds_base + dst, b_off[i], st * kBlock);
            } else if (lane < 8 * NTW) {  // FG: the other lanes are masked off and write nothing
                dma16(g_rsrc, lds_base + kScaleBase + (slot * kWaves + wave) * kScaleWave, g_off, st * p.ldg * 4);
            }
        }
    };

    v16i acc[MTW][NTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int t = 0; t < NTW; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][t][v] = 0;
    // FG: sum over the groups of float(integer sum of the group) * group scale, sixteen-fold like the integer sums
    float facc[FG ? MTW : 1][FG ? NTW : 1][16];
    if (FG) {
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
            for (int t = 0; t < NTW; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) facc[FG ? mt : 0][FG ? t : 0][v] = 0.f;
    }

    // LDS offsets of this lane's fragments inside a stage.  MFMA step j = 0..3 of a stage covers k = 32 j .. 32 j + 31;
    // lane (idx, g) supplies k = 32 j + 16 g .. + 15: activation chunk 2 j + g of its row, and dwords 2 (j % 2), +1
    // of weight chunk ... (the weight chunk c = 32 k holds two steps: c = j / 2 ... see read_w).
    // Steps are numbered so that one weight chunk serves two consecutive steps: step j uses weight chunk
    // 2 (j / 2) + g, dwords 2 (j % 2) and 2 (j % 2) + 1, i.e. k = 64 (j/2) + 32 g + 16 (j%2) .. + 15, and the
    // activation chunk with the same k: 4 (j / 2) + 2 g + (j % 2).
    int xa[4];
    {
        const int row = wm * (32 * MTW) + idx;  // rows of the other m tiles differ by 32: same swizzle
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // int8 weights: step j, lane group g holds k = 32 j + 16 g .. + 15, i.e. activation chunk 2 j + g
            const int chunk = W8 ? 2 * j + g : 4 * (j >> 1) + 2 * g + (j & 1);
            xa[j] = row * 128 + ((chunk ^ fx(row)) << 4);
        }
    }
    const int wa = kBBase + wn * (NTW * kBlock) + (g * 32 + idx) * 16;
    auto read_x_at = [&](v4u(&dst)[MTW], int slot, int offset) {
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) dst[mt] = *(const v4u *)(&lds[slot * A_STAGE + offset + mt * 4096]);
    };
    auto read_x = [&](v4u(&dst)[MTW], int slot, int j) { read_x_at(dst, slot, xa[j]); };
    // weight fragments of the pair of chunks q: int4 -> q = 0, 1 serves MFMA steps 2q and 2q + 1 (halves h = 0, 1 of
    // the fragment); int8 -> q = 0 .. 3 serves MFMA step q
    auto read_w = [&](v4u(&dst)[NTW], int slot, int q) {
#pragma unroll
        for (int t = 0; t < NTW; ++t) dst[t] = *(const v4u *)(&lds[slot * B_STAGE + wa + t * kBlock + q * 1024]);
    };
    // the scales of this wave's channels for the group in ring slot `slot`, in accumulator order:
    // register 4 q + e of block t belongs to channel 32 t + 8 q + 4 g + e
    auto read_sg = [&](float(&dst)[NTW][16], int slot) {
#pragma unroll
        for (int t = 0; t < NTW; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = *(const float4 *)(&lds[kScaleBase + (slot * kWaves + wave) * kScaleWave +
                                                        (32 * t + 8 * q + 4 * g) * 4]);
                dst[t][4 * q] = v.x;
                dst[t][4 * q + 1] = v.y;
                dst[t][4 * q + 2] = v.z;
                dst[t][4 * q + 3] = v.w;
            }
    };
    // fresh = true (FG, first step of a stage): the group's integer sums start from zero
    auto mfma_step = [&](const v4u(&x)[MTW], const v4u(&w)[NTW], int h, bool fresh = false) {
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
            const v4i wop = W8    ? v4i{(int)w[t].x, (int)w[t].y, (int)w[t].z, (int)w[t].w}
                            : UNS ? (h == 0 ? u_operand_tiled(w[t].x, w[t].y) : u_operand_tiled(w[t].z, w[t].w))
                                  : (h == 0 ? w_operand_tiled(w[t].x, w[t].y) : w_operand_tiled(w[t].z, w[t].w));
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
                acc[mt][t] = mfma32(wop, v4i{(int)x[mt].x, (int)x[mt].y, (int)x[mt].z, (int)x[mt].w},
                                    fresh ? v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0} : acc[mt][t]);
        }
    };

    // Two schedules.  Ring of two: stage st + 2 can only be requested once stage st has been read, i.e. in one burst
    // behind the barrier of stage st.  Ring of three or more (kSpread): the slot freed by the barrier of stage st - 1
    // is refilled with stage st + STAGES - 1 in thirds, between the MFMA blocks of stage st; a burst of loads right
    // behind the barrier holds up the issuing wave for as long as the address unit needs to take them (measured: a
    // fifth of the loop time), spread out they cost an issue slot each.
    // Loads return in order, so "at most n outstanding" means all but the youngest n have landed; waiting for fewer
    // than could be allowed is always safe, which is what happens near the end of K.
    // Measured: spreading pays for the 8-wave tiles (3-4 %); the 4-wave tiles with a ring of three lose 5-15 % to
    // the shorter look-ahead it implies, so they keep the burst.
    constexpr bool kSpread = STAGES >= 3 && kWaves >= 8;
    constexpr int kAhead = kSpread ? STAGES - 1 : STAGES;  // stages requested before the loop starts
#pragma unroll
    for (int s = 0; s < kAhead; ++s)
        if (s < st_total) issue(s, s, 0, 1);
    if (st_total >= kAhead)
        wait_vmcnt<(kAhead - 1) * kLoads>();
    else
        wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();

    v4u x0[MTW], x1[MTW], w0[NTW], w1[NTW];
    float sg[FG ? NTW : 1][16];
    int slot = 0;
    if constexpr (KS == 2) {
        // Per stage and wave two MFMA steps (2 ks and 2 ks + 1, one weight fragment) with the barrier between them:
        // by then this wave has every fragment of the stage in registers.  The target stage goes out in halves,
        // one before and one behind the barrier, so behind the barrier's wait only the first half may be in flight.
        static_assert(kSpread, "the k split uses the spread schedule");
        constexpr int kFirstHalf = (kLoads + 1) / 2;
        const int xa_first = ks ? xa[2] : xa[0], xa_second = ks ? xa[3] : xa[1];
        read_x_at(x0, 0, xa_first);
        read_w(w0, 0, ks);
        for (int st = 0; st < st_total; ++st) {
            const int next = slot + 1 == STAGES ? 0 : slot + 1;
            const int prev = slot == 0 ? STAGES - 1 : slot - 1;
            const int target = st + STAGES - 1;
            const bool have_target = target < st_total;
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
            read_x_at(x1, slot, xa_second);
            if (have_target) issue(target, prev, 0, 2);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(x0, w0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (have_target)
                wait_vmcnt<kFirstHalf>();
            else
                wait_vmcnt<0>();
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            if (have_target) issue(target, prev, 1, 2);
            if (st + 1 < st_total) {
                read_x_at(x0, next, xa_first);
                read_w(w1, next, ks);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(x1, w0, 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < NTW; ++t) w0[t] = w1[t];
            slot = next;
        }
    } else {
        read_x(x0, 0, 0);
        read_w(w0, 0, 0);
        for (int st = 0; st < st_total; ++st) {
            const int next = slot + 1 == STAGES ? 0 : slot + 1;
            const int prev = slot == 0 ? STAGES - 1 : slot - 1;
            const int target = st + STAGES - 1;            // kSpread: the stage requested during this one
            const bool have_target = kSpread && target < st_total;
            // The scheduling fences keep each block of LDS reads in front of the MFMA block it overlaps with; left alone
            // the compiler sinks the reads next to their first use and every step then starts with an exposed LDS wait.
            // The fragments of step 0 were requested eight MFMAs ago; waiting for them here, before the next reads go
            // out, costs nothing and spares the wait the compiler would otherwise place behind those reads.
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
            // Weight registers: int4 fragments hold two steps (w0: steps 0, 1; w1: steps 2, 3); int8 fragments one step
            // each, w0 and w1 taking turns (w0: steps 0, 2; w1: steps 1, 3).
            read_x(x1, slot, 1);
            if (W8) read_w(w1, slot, 1);
            if (have_target) issue(target, prev, 0, 3);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(x0, w0, 0, FG);
            __builtin_amdgcn_sched_barrier(0);
            read_x(x0, slot, 2);
            if (W8)
                read_w(w0, slot, 2);
            else
                read_w(w1, slot, 1);
            if (have_target) issue(target, prev, 1, 3);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(x1, *(W8 ? &w1 : &w0), 1);
            __builtin_amdgcn_sched_barrier(0);
            read_x(x1, slot, 3);
            if (W8) read_w(w1, slot, 3);
            if constexpr (FG) read_sg(sg, slot);  // before the barrier that lets the slot be refilled
            if (have_target) issue(target, prev, 2, 3);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(x0, *(W8 ? &w0 : &w1), 0);
            __builtin_amdgcn_sched_barrier(0);
            // Every fragment of this stage is in registers once the reads above have returned, so after the barrier the
            // slot can be refilled; stage st + 1 must be in LDS for every wave.
            if (kSpread ? have_target : st + STAGES <= st_total)
                wait_vmcnt<(STAGES - 2) * kLoads>();  // the stages behind st + 1 may still be in flight
            else
                wait_vmcnt<0>();
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's last fragment reads of the slot have returned
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            if (!kSpread && st + STAGES < st_total) issue(st + STAGES, slot, 0, 1);
            if (st + 1 < st_total) {
                read_x(x0, next, 0);
                read_w(w0, next, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(x1, w1, 1);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (FG) {
                // Dq of Eq. (5) for this group: a group's sums are below 2^24 in magnitude, so the conversion is exact
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                    for (int t = 0; t < NTW; ++t)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            facc[mt][t][v] = __builtin_fmaf((float)acc[mt][t][v], sg[t][v], facc[mt][t][v]);
            }
            slot = next;
        }
    }
    wait_vmcnt<0>();

    // The ring is idle: the last barrier of the loop lies behind every wave's last fragment read and every load has
    // landed.  Park the scales behind it; the barrier that makes them visible is the one of the k halves' meeting
    // where there is one.
    float *const sa_lds = (float *)(lds + kEpiScales);
    float *const sw_lds = sa_lds + BM;
    if (!ACC_OUT) {
        if (tid < BM) sa_lds[tid] = sa_mine;
        if (tid < BN) sw_lds[tid] = sw_mine;
        if constexpr (KS == 1) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        }
    }

    if constexpr (KS == 2) {
        // The two k halves meet: the ring is idle (the last barrier lies behind every wave's last fragment read and
        // every load has landed), the upper set parks its sums behind the area the epilogue's slabs will use and leaves.
        constexpr int kRedBase = kOutWaves * 32 * (64 * NTW + 16);
        int *part = (int *)(lds + kRedBase) + wsub * (MTW * NTW * 16 * 64) + lane;
        if (ks == 1) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int t = 0; t < NTW; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) part[((mt * NTW + t) * 16 + v) * 64] = acc[mt][t][v];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        if (ks == 1) return;
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
            for (int t = 0; t < NTW; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mt][t][v] += part[((mt * NTW + t) * 16 + v) * 64];
    }

    // Epilogue (Eq. (6),(7)).  A lane holds, per (mt, t, quad), four consecutive n of one m, so storing from the
    // accumulator layout writes 16 bytes into each of 32 different rows per instruction.  Instead every wave turns
    // its 32-row slabs around in LDS (the ring is idle now: the last barrier of the loop lies behind every wave's
    // last fragment read and every load has landed) and stores whole 16-byte runs of 8 channels, 8 or more lanes per
    // row, i.e. whole cache lines.
    // int4 sums are sixteen times the true sums (the nibbles sat in the high half of their bytes); int8 sums are true
    auto deq = [](int a, float s_a, float s_w) { return kTrueSums ? (float)a * (s_a * s_w) : dequant(a, s_a, s_w); };
    // FG: the sixteen-fold fp32 sum times s_a / 16 (both scalings by a power of two are exact): one rounding, as in
    // f * s_a on the true sum
    auto value = [&](int mt, int t, int v, float s_a, float s_w) {
        if constexpr (FG)
            return facc[mt][t][v] * (s_a * 0.0625f);
        else
            return deq(acc[mt][t][v], s_a, s_w);
    };
    if (!ACC_OUT && (SWIGLU || (p.ldc & 7) == 0)) {  // the fused form is only launched with a pitch that allows this path
        constexpr int kRowBytes = 64 * NTW;        // fp16 bytes of a slab row (32 NTW channels)
        constexpr int kPitch = kRowBytes + 16;     // padded: rows 16 apart, not 1 apart, share banks
        constexpr int kChunksPerRow = 4 * NTW;     // 16-byte chunks
        constexpr int kReads = (32 * kChunksPerRow + 63) / 64;
        static_assert(kOutWaves * 32 * kPitch <= STAGES * (A_STAGE + B_STAGE), "slabs must fit the ring");
        uint8_t *slab = lds + wsub * (32 * kPitch);
        const int n_wave = bn0 + wn * (32 * NTW);
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            const int m_slab = bm0 + wm * (32 * MTW) + 32 * mt;
            const float sa = sa_lds[wm * (32 * MTW) + 32 * mt + idx];  // 0 for rows past M
#pragma unroll
            for (int t = 0; t < NTW; ++t) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = 32 * t + 8 * q + 4 * g;
                    // channels past N carry scale 0: their values are formed but never stored
                    const float4 sw = FG ? float4{0.f, 0.f, 0.f, 0.f} : *(const float4 *)(sw_lds + wn * (32 * NTW) + nl);
                    v2u o;
                    o.x = pack_f16x2(value(mt, t, 4 * q, sa, sw.x), value(mt, t, 4 * q + 1, sa, sw.y));
                    o.y = pack_f16x2(value(mt, t, 4 * q + 2, sa, sw.z), value(mt, t, 4 * q + 3, sa, sw.w));
                    *(v2u *)(slab + idx * kPitch + nl * 2) = o;
                }
            }
#pragma unroll
            for (int j = 0; j < kReads; ++j) {
                const int c = j * 64 + lane;
                const int row = c / kChunksPerRow, col = c - row * kChunksPerRow;
                if (32 * kChunksPerRow % 64 != 0 && row >= 32) continue;
                const v4u v = *(const v4u *)(slab + row * kPitch + col * 16);
                const int mm = m_slab + row, n = n_wave + col * 8;
                if (mm >= p.M || n >= p.N) continue;
                if constexpr (SWIGLU) {
                    // eight channels = four (gate, up) pairs -> four values of h
                    const v2u hv = silu_mul_pairs4(v);
                    unsigned short *dst = (unsigned short *)p.out + (size_t)mm * p.ldc + (n >> 1);
                    if (n + 8 <= p.N) {
                        *(v2u *)dst = hv;
                    } else {
                        const unsigned w[2] = {hv.x, hv.y};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + 2 * e + 1 < p.N) dst[e] = (unsigned short)(w[e >> 1] >> (16 * (e & 1)));
                    }
                    continue;
                }
                unsigned short *dst = (unsigned short *)p.out + (size_t)mm * p.ldc + n;
                if (n + 8 <= p.N) {
                    *(v4u *)dst = v;
                } else {
                    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (n + e < p.N) dst[e] = (unsigned short)(w[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
        return;
    }

    // general epilogue: raw sums, or an output pitch that rules out 16-byte stores
    const bool vec_ok = (p.ldc & 3) == 0;
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int m = bm0 + wm * (32 * MTW) + 32 * mt + idx;
        if (m >= p.M) continue;
        const float sa = ACC_OUT ? 0.f : sa_lds[wm * (32 * MTW) + 32 * mt + idx];
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = bn0 + wn * (32 * NTW) + 32 * t + 8 * q + 4 * g;
                if (n >= p.N) continue;
                const v4i s = v4i{acc[mt][t][4 * q], acc[mt][t][4 * q + 1], acc[mt][t][4 * q + 2], acc[mt][t][4 * q + 3]};
                if (ACC_OUT) {
                    int *dst = p.acc_out + (size_t)m * p.ldc + n;
                    if (p.splits > 1) dst += (size_t)blockIdx.y * (size_t)p.M * (size_t)p.ldc;
                    constexpr int kShift = kTrueSums ? 0 : 4;  // signed int4: exact, every sum is a multiple of 16
                    const v4i v = v4i{s.x >> kShift, s.y >> kShift, s.z >> kShift, s.w >> kShift};
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
                        const float4 sw = FG ? float4{0.f, 0.f, 0.f, 0.f} : *(const float4 *)(sw_lds + (n - bn0));
                        v2u o;
                        o.x = pack_f16x2(value(mt, t, 4 * q, sa, sw.x), value(mt, t, 4 * q + 1, sa, sw.y));
                        o.y = pack_f16x2(value(mt, t, 4 * q + 2, sa, sw.z), value(mt, t, 4 * q + 3, sa, sw.w));
                        *(v2u *)dst = o;
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (n + j < p.N)
                                dst[j] = f32_to_f16_bits(value(mt, t, 4 * q + j, sa, FG ? 0.f : sw_lds[n + j - bn0]));
                    }
                }
            }
        }
    }
}

namespace {

template <int MTW, int NTW, int WM, int WN, int STAGES, bool ACC_OUT, int WBITS, bool UNS, bool FG, int KS, bool SWIGLU = false>
hipError_t launch_one(const PrefillArgs &p, dim3 grid, hipStream_t stream) {
    constexpr int BM = 32 * MTW * WM, BN = 32 * NTW * WN;
    // ring + spare KB; group scales: 128 NTW bytes per wave and ring slot, and a KB of slack behind them
    constexpr int kRing = STAGES * (BM * 128 + BN * 16 * WBITS) + 1024 + (FG ? STAGES * WM * WN * NTW * 128 + 1024 : 0);
    // k split: the epilogue's slabs and, behind them, the parked sums of the upper wave set
    constexpr int kMeet = KS == 2 ? WM * WN * (32 * (64 * NTW + 16) + MTW * NTW * 16 * 256) : 0;
    constexpr int kLdsBytes = (kRing > kMeet ? kRing : kMeet) + (BM + BN) * 4;  // + the epilogue's s_a and s_w
    static_assert(kLdsBytes <= 160 * 1024, "a workgroup's ring must fit the compute unit's LDS");
    constexpr auto kernel = gemm_prefill_tiled_kernel<MTW, NTW, WM, WN, STAGES, ACC_OUT, WBITS, UNS, FG, KS, SWIGLU>;
    if (const hipError_t e = allow_lds<kernel>(kLdsBytes); e != hipSuccess) return e;
    if (p.prepare_only) return hipSuccess;
    hipLaunchKernelGGL(kernel, grid, dim3(64 * WM * WN * KS), kLdsBytes, stream, p);
    return hipGetLastError();
}

template <int MTW, int NTW, int WM, int WN, int STAGES, int WBITS = 4, bool UNS = false, bool FG = false, int KS = 1>
hipError_t launch_tile(PrefillArgs p, bool acc_out, hipStream_t stream) {
    constexpr int BM = 32 * MTW * WM, BN = 32 * NTW * WN;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    const int total = p.tiles_m * p.tiles_n;
    const dim3 grid(8 * ((total + 7) / 8), p.splits > 1 ? p.splits : 1);
    if (p.splits > 1 && (!acc_out || FG)) return hipErrorInvalidValue;  // a split of K returns raw partial sums
    if constexpr (FG) {
        if (acc_out) return hipErrorInvalidValue;  // there is no single integer sum to return
        return launch_one<MTW, NTW, WM, WN, STAGES, false, WBITS, UNS, true, 1>(p, grid, stream);
    } else {
        return acc_out ? launch_one<MTW, NTW, WM, WN, STAGES, true, WBITS, UNS, false, KS>(p, grid, stream)
                       : launch_one<MTW, NTW, WM, WN, STAGES, false, WBITS, UNS, false, KS>(p, grid, stream);
    }
}

// The fused SiLU * up form of a tile: one launch covers the problem (byte offsets below 2^32 are the caller's check).
template <int MTW, int NTW, int WM, int WN, int STAGES>
hipError_t launch_tile_swiglu(PrefillArgs p, hipStream_t stream) {
    constexpr int BM = 32 * MTW * WM, BN = 32 * NTW * WN;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    const int total = p.tiles_m * p.tiles_n;
    return launch_one<MTW, NTW, WM, WN, STAGES, false, 4, false, false, 1, true>(p, dim3(8 * ((total + 7) / 8)), stream);
}

// One thread per 16-byte chunk of the tiled int8 array (W8A8 variant): a plain gather, no reordering inside a chunk.
__global__ __launch_bounds__(256) void tile_weights8_kernel(const int8_t *__restrict__ w8, uint8_t *__restrict__ wt, int N,
                                                            int K, int kb_total, long long chunks) {
    const long long q = (long long)blockIdx.x * 256 + threadIdx.x;
    if (q >= chunks) return;
    const long long block = q >> 8;
    const int c = (int)(q & 255) >> 5, r = (int)(q & 31);
    const long long nb = block / kb_total;
    const int kb = (int)(block - nb * kb_total);
    const long long n = nb * 32 + r;
    const int k0 = kb * 128 + c * 16;
    v4u v = v4u{0u, 0u, 0u, 0u};
    if (n < N && k0 < K) v = *(const v4u *)(w8 + (size_t)n * (size_t)K + k0);
    *(v4u *)(wt + (size_t)q * 16) = v;
}

}  // namespace

// Second half of a GEMM whose K was split over workgroups: adds the slabs of raw sums and applies Eq. (6),(7).
// Integer addition in any order gives the same sum, so the result has the bits of the unsplit kernel.
__global__ __launch_bounds__(256) void splitk_epilogue_kernel(const int *__restrict__ part, int splits,
                                                              const float *__restrict__ s_a, const float *__restrict__ s_w,
                                                              unsigned short *__restrict__ out, int M, int N, int quads_per_row) {
    const long long q = (long long)blockIdx.x * 256 + threadIdx.x;
    if (q >= (long long)M * quads_per_row) return;
    const int m = (int)(q / quads_per_row);
    const int n = (int)(q - (long long)m * quads_per_row) * 4;
    const size_t slab = (size_t)M * N, at = (size_t)m * N + n;
    const float sa = s_a[m];
    if ((N & 3) == 0) {
        v4i s = *(const v4i *)(part + at);
        for (int i = 1; i < splits; ++i) {
            const v4i t = *(const v4i *)(part + i * slab + at);
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        const float4 sw = *(const float4 *)(s_w + n);
        v2u o;
        o.x = pack_f16x2((float)s.x * (sa * sw.x), (float)s.y * (sa * sw.y));
        o.y = pack_f16x2((float)s.z * (sa * sw.z), (float)s.w * (sa * sw.w));
        *(v2u *)(out + at) = o;
    } else {
        for (int j = 0; j < 4 && n + j < N; ++j) {
            int s = 0;
            for (int i = 0; i < splits; ++i) s += part[i * slab + at + j];
            out[at + j] = f32_to_f16_bits((float)s * (sa * s_w[n + j]));
        }
    }
}

hipError_t launch_splitk_epilogue(const int *part, int splits, const float *s_a, const float *s_w, void *out, int M, int N,
                                  hipStream_t stream) {
    const int quads_per_row = (N + 3) / 4;
    const long long blocks = ((long long)M * quads_per_row + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(splitk_epilogue_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, part, splits, s_a, s_w,
                       (unsigned short *)out, M, N, quads_per_row);
    return hipGetLastError();
}

hipError_t launch_gemm_prefill_tiled(const PrefillArgs &p, bool acc_out, int tile, hipStream_t stream, int wbits) {
    // slices keep every byte offset inside the kernel below 2^32; slices of N start on a 32-channel block
    const long long kMaxBytes = 0xF0000000ll;
    const long long kb_total = (p.K + kTiledBlockK - 1) / kTiledBlockK;
    const long long block_bytes = (long long)kTiledBlockBytes * (wbits == 8 ? 2 : 1);
    if (wbits == kWeightsFineGrained4 && (p.K % kTiledBlockK != 0 || p.ldg < p.N || (p.ldg & 3) != 0 ||
                                          kb_total * (long long)p.ldg * 4 > kMaxBytes))
        return hipErrorInvalidValue;
    long long m_rows = kMaxBytes / p.K, n_rows = kMaxBytes / (kb_total * (block_bytes / 32));
    m_rows -= m_rows % 256;
    n_rows -= n_rows % 3840;  // a multiple of every tile width
    for (long long n0 = 0; n0 < p.N; n0 += n_rows) {
        for (long long m0 = 0; m0 < p.M; m0 += m_rows) {
            PrefillArgs q = p;
            q.M = (int)((p.M - m0) < m_rows ? (p.M - m0) : m_rows);
            q.N = (int)((p.N - n0) < n_rows ? (p.N - n0) : n_rows);
            q.xq = p.xq + (size_t)m0 * p.K;
            q.wp = p.wp + (size_t)(n0 / 32) * (size_t)kb_total * (size_t)block_bytes;
            if (p.s_a) q.s_a = p.s_a + m0;
            if (p.s_w) q.s_w = p.s_w + n0;
            if (p.out) q.out = (unsigned short *)p.out + (size_t)m0 * p.ldc + n0;
            if (p.acc_out) q.acc_out = p.acc_out + (size_t)m0 * p.ldc + n0;
            if (p.splits > 1 && (q.M != p.M || q.N != p.N)) return hipErrorInvalidValue;  // slabs are whole problems
            hipError_t e;
            if (wbits == 4) {
                switch (tile) {
                    case kTiled256x256: e = launch_tile<4, 2, 2, 4, 3>(q, acc_out, stream); break;
                    case kTiled256x256Square: e = launch_tile<2, 4, 4, 2, 3>(q, acc_out, stream); break;
                    case kTiled128x256: e = launch_tile<4, 2, 1, 4, 2>(q, acc_out, stream); break;
                    case kTiled128x160: e = launch_tile<1, 5, 4, 1, 3>(q, acc_out, stream); break;
                    case kTiled128x128: e = launch_tile<2, 2, 2, 2, 3>(q, acc_out, stream); break;
                    case kTiled64x128: e = launch_tile<1, 2, 2, 2, 4>(q, acc_out, stream); break;
                    case kTiled64x64: e = launch_tile<1, 1, 2, 2, 4>(q, acc_out, stream); break;
                    case kTiled32x128: e = launch_tile<1, 1, 1, 4, 4>(q, acc_out, stream); break;
                    case kTiled128x160K2: e = launch_tile<1, 5, 4, 1, 3, 4, false, false, 2>(q, acc_out, stream); break;
                    case kTiled128x128K2: e = launch_tile<2, 2, 2, 2, 3, 4, false, false, 2>(q, acc_out, stream); break;
                    case kTiled256x192: e = launch_tile<2, 3, 4, 2, 3>(q, acc_out, stream); break;
                    case kTiled128x256W8: e = launch_tile<2, 2, 2, 4, 3>(q, acc_out, stream); break;
                    default: e = hipErrorInvalidConfiguration;
                }
            } else if (wbits == 8) {
                // int8 weight stages are twice as large: shallower rings for the same LDS
                switch (tile) {
                    case kTiled256x256: e = launch_tile<4, 2, 2, 4, 2, 8>(q, acc_out, stream); break;
                    case kTiled256x256Square: e = launch_tile<2, 4, 4, 2, 2, 8>(q, acc_out, stream); break;
                    case kTiled128x256: e = launch_tile<4, 2, 1, 4, 2, 8>(q, acc_out, stream); break;
                    case kTiled128x160: e = launch_tile<1, 5, 4, 1, 2, 8>(q, acc_out, stream); break;
                    case kTiled128x128: e = launch_tile<2, 2, 2, 2, 2, 8>(q, acc_out, stream); break;
                    case kTiled64x128: e = launch_tile<1, 2, 2, 2, 3, 8>(q, acc_out, stream); break;
                    case kTiled64x64: e = launch_tile<1, 1, 2, 2, 4, 8>(q, acc_out, stream); break;
                    case kTiled32x128: e = launch_tile<1, 1, 1, 4, 3, 8>(q, acc_out, stream); break;
                    default: e = hipErrorInvalidConfiguration;
                }
            } else if (wbits == kWeightsUnsigned4) {
                switch (tile) {
                    case kTiled256x256: e = launch_tile<4, 2, 2, 4, 3, 4, true>(q, acc_out, stream); break;
                    case kTiled256x256Square: e = launch_tile<2, 4, 4, 2, 3, 4, true>(q, acc_out, stream); break;
                    case kTiled128x256: e = launch_tile<4, 2, 1, 4, 2, 4, true>(q, acc_out, stream); break;
                    case kTiled128x160: e = launch_tile<1, 5, 4, 1, 3, 4, true>(q, acc_out, stream); break;
                    case kTiled128x128: e = launch_tile<2, 2, 2, 2, 3, 4, true>(q, acc_out, stream); break;
                    case kTiled64x128: e = launch_tile<1, 2, 2, 2, 4, 4, true>(q, acc_out, stream); break;
                    case kTiled64x64: e = launch_tile<1, 1, 2, 2, 4, 4, true>(q, acc_out, stream); break;
                    case kTiled32x128: e = launch_tile<1, 1, 1, 4, 4, 4, true>(q, acc_out, stream); break;
                    default: e = hipErrorInvalidConfiguration;
                }
            } else if (wbits == kWeightsFineGrained4) {
                // one problem, one launch: the group scales are addressed with the whole problem's pitch
                if (q.M != p.M || q.N != p.N) return hipErrorInvalidValue;
                switch (tile) {
                    case kFine128x256: e = launch_tile<2, 2, 2, 4, 3, 4, false, true>(q, acc_out, stream); break;
                    case kFine256x128: e = launch_tile<2, 2, 4, 2, 3, 4, false, true>(q, acc_out, stream); break;
                    case kFine128x128: e = launch_tile<2, 2, 2, 2, 3, 4, false, true>(q, acc_out, stream); break;
                    case kFine64x128: e = launch_tile<1, 2, 2, 2, 4, 4, false, true>(q, acc_out, stream); break;
                    case kFine64x64: e = launch_tile<1, 1, 2, 2, 4, 4, false, true>(q, acc_out, stream); break;
                    case kFine32x128: e = launch_tile<1, 1, 1, 4, 4, 4, false, true>(q, acc_out, stream); break;
                    default: e = hipErrorInvalidConfiguration;
                }
            } else {
                e = hipErrorInvalidConfiguration;
            }
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_gemm_prefill_tiled_swiglu(const PrefillArgs &p, int tile, hipStream_t stream) {
    // p.N interleaved channels (even), p.out = h with pitch p.ldc (a multiple of 4 elements: the 8-byte stores of four
    // values are aligned)
    const long long kMaxBytes = 0xF0000000ll;
    const long long kb_total = (p.K + kTiledBlockK - 1) / kTiledBlockK;
    if ((p.N & 1) || (p.ldc & 3) || (long long)p.M * p.K > kMaxBytes ||
        (long long)((p.N + 31) / 32) * kb_total * kTiledBlockBytes > kMaxBytes)
        return hipErrorInvalidValue;
    switch (tile) {
        case kTiled256x256: return launch_tile_swiglu<4, 2, 2, 4, 3>(p, stream);
        case kTiled256x192: return launch_tile_swiglu<2, 3, 4, 2, 3>(p, stream);
        case kTiled128x256: return launch_tile_swiglu<4, 2, 1, 4, 2>(p, stream);
        case kTiled128x256W8: return launch_tile_swiglu<2, 2, 2, 4, 3>(p, stream);
        case kTiled128x128: return launch_tile_swiglu<2, 2, 2, 2, 3>(p, stream);
        default: return hipErrorInvalidConfiguration;
    }
}

hipError_t prepare_tiled_kernels() {
    PrefillArgs a{};
    a.M = 32; a.N = 32; a.K = kTiledBlockK; a.ldc = 32; a.ldg = 32;
    a.prepare_only = true;
    for (int tile : {kTiled256x256, kTiled256x192, kTiled128x256, kTiled128x256W8, kTiled128x128})
        if (const hipError_t e = launch_gemm_prefill_tiled_swiglu(a, tile, nullptr); e != hipSuccess) return e;
    struct Format { int wbits, tiles; bool acc; };
    const Format formats[] = {{4, kTiledTileMax4, true}, {8, kTiledTileMax, true}, {kWeightsUnsigned4, kTiledTileMax, true},
                              {kWeightsFineGrained4, kFineTileMax, false}};
    for (const Format &f : formats)
        for (int tile = 1; tile <= f.tiles; ++tile)
            for (int acc = 0; acc <= (f.acc ? 1 : 0); ++acc) {
                const hipError_t e = launch_gemm_prefill_tiled(a, acc != 0, tile, nullptr, f.wbits);
                if (e != hipSuccess) return e;
            }
    return hipSuccess;
}

size_t tiled_weight_bytes(int N, int K, int wbits) {
    return (size_t)((N + 31) / 32) * (size_t)((K + kTiledBlockK - 1) / kTiledBlockK) * (size_t)(kTiledBlockBytes * wbits / 4);
}

hipError_t launch_tile_weights(const uint8_t *wp, uint8_t *wt, int N, int K, hipStream_t stream) {
    const int kb_total = (K + kTiledBlockK - 1) / kTiledBlockK;
    const long long chunks = (long long)(tiled_weight_bytes(N, K, 4) / 16);
    const long long blocks = (chunks + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tile_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, wp, wt, N, K, kb_total, chunks);
    return hipGetLastError();
}

hipError_t launch_tile_weights8(const int8_t *w8, uint8_t *wt, int N, int K, hipStream_t stream) {
    const int kb_total = (K + kTiledBlockK - 1) / kTiledBlockK;
    const long long chunks = (long long)(tiled_weight_bytes(N, K, 8) / 16);
    const long long blocks = (chunks + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tile_weights8_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w8, wt, N, K, kb_total, chunks);
    return hipGetLastError();
}

}  // namespace w4a8
