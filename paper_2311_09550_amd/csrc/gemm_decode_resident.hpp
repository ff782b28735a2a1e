// The persistent weight-streaming kernel with register-resident activations, its resource estimates and its launch:
// shared by the translation units that instantiate it (gemm_decode.hip: up to 32 tokens with the activations staged
// whole; gemm_decode_wide.hip: up to 64 tokens with every wave staging its own k steps).
#pragma once

#include "common.hpp"
#include "kernels.hpp"

namespace w4a8 {

namespace {

// Store four consecutive raw sums (n .. n+3 of row m) held by one lane.
__device__ __forceinline__ void store4_acc(const DecodeArgs &p, int m, int n, int n_end, v4i s) {
    int *dst = p.acc_out + (size_t)m * p.N + n;
    const v4i v = v4i{s.x >> 4, s.y >> 4, s.z >> 4, s.w >> 4};  // exact: every sum is a multiple of 16
    if ((p.N & 3) == 0 && n + 3 < n_end) {
        *(v4i *)dst = v;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (n + j < n_end) dst[j] = v[j];
    }
}

// Dequantise (Eq. (6),(7)) and store four consecutive fp16 outputs; sw holds s_w[n .. n+3].
__device__ __forceinline__ void store4_f16(const DecodeArgs &p, int m, int n, int n_end, v4i s, float sa, float4 sw) {
    unsigned short *dst = (unsigned short *)p.out + (size_t)m * p.N + n;
    if ((p.N & 3) == 0 && n + 3 < n_end) {
        v2u o;
        o.x = pack_f16x2(dequant(s.x, sa, sw.x), dequant(s.y, sa, sw.y));
        o.y = pack_f16x2(dequant(s.z, sa, sw.z), dequant(s.w, sa, sw.w));
        *(v2u *)dst = o;
    } else {
        const float w[4] = {sw.x, sw.y, sw.z, sw.w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (n + j < n_end) dst[j] = f32_to_f16_bits(dequant(s[j], sa, w[j]));
    }
}

// The four channels are two (gate, up) pairs of interleaved gate / up weights: dequantise and round to fp16 as
// store4_f16 would, then store h = fp16(silu(gate) * up) of both pairs (row m of h, N / 2 values long).  Same bits as
// the fp16 GEMM output run through the row-wise SiLU * up kernel.
__device__ __forceinline__ void store4_h(const DecodeArgs &p, int m, int n, v4i s, float sa, float4 sw) {
    const unsigned gu0 = pack_f16x2(dequant(s.x, sa, sw.x), dequant(s.y, sa, sw.y));
    const unsigned gu1 = pack_f16x2(dequant(s.z, sa, sw.z), dequant(s.w, sa, sw.w));
    unsigned short *dst = (unsigned short *)p.out + (size_t)m * (size_t)(p.N >> 1) + (n >> 1);
    *(unsigned *)dst = pack_f16x2(silu_mul_f32(lo_half(gu0), hi_half(gu0)), silu_mul_f32(lo_half(gu1), hi_half(gu1)));
}

template <bool ACC_OUT>
__device__ __forceinline__ void store4(const DecodeArgs &p, int m, int n, v4i s) {
    if (ACC_OUT) {
        store4_acc(p, m, n, p.N, s);
    } else {
        float4 sw;
        sw.x = p.s_w[n];
        sw.y = p.s_w[min(n + 1, p.N - 1)];
        sw.z = p.s_w[min(n + 2, p.N - 1)];
        sw.w = p.s_w[min(n + 3, p.N - 1)];
        store4_f16(p, m, n, p.N, s, p.s_a[m], sw);
    }
}

}  // namespace

__device__ __forceinline__ void lds_release() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local"); }
__device__ __forceinline__ void lds_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local"); }
// Barrier that orders LDS accesses only: an ordinary __syncthreads() would also wait for the wave's outstanding
// global loads, i.e. drain the weight prefetch.
__device__ __forceinline__ void lds_barrier() {
    lds_release();
    __builtin_amdgcn_s_barrier();
    lds_acquire();
}

// ---------------------------------------------------------------------------------------------
// Persistent kernel with register-resident activations.  MT = ceil(M/16) column tiles, XS = k steps per wave
// (ceil(ceil(K/128) / WAVES) <= XS), P = chunks of weight loads a wave keeps in flight.
//
//   * Workgroup b owns the contiguous output channels [b * rows_per_wg, (b + 1) * rows_per_wg) and walks them in
//     chunks of p.chunk_rows <= 16 channels (the launcher splits a range evenly, so that 24 channels are two chunks
//     of 12, not 16 and 8); P chunks form an epoch.  The last chunk of a range may be partial: its missing rows are
//     simply not loaded.
//   * A wave's k steps are the same for every chunk, so its activation operands are fetched ONCE and stay in
//     registers; per chunk only weights are loaded, and the loads of chunk c + P are issued as soon as a register of
//     chunk c has been converted, into that very register, so a wave always has P * XS loads of 16 bytes per lane in
//     flight.  When a range has no more than P chunks, every weight byte of the workgroup is requested before the
//     first one is used.
//   * Weights are read with bounds-checked buffer loads: an offset past the end of the buffer returns zeros and
//     touches no memory.  That is how a dead K group (K % 128 != 0), a wave without a step, a row outside the
//     workgroup's range and a finished walk are handled, with neither a branch nor a select nor a wasted access.
//   * Per epoch every wave writes its partial sums (plain LDS stores into its own slots), the workgroup meets at
//     one LDS-only barrier, and all threads share the epilogue of the epoch's P chunks (sum over the waves,
//     Eq. (6),(7), store).  Two sets of slots take turns, so one barrier per epoch is enough: a wave can only be
//     writing epoch e + 2 after every wave has passed the barrier of epoch e + 1, i.e. finished reading epoch e.
//     The epilogue reads nothing from global memory (s_a sits in a register, the s_w of the range in LDS): a load
//     there would queue behind the whole weight prefetch.
//
// TILED: p.wp is the tiled weight array of the large-M kernel (2 KB blocks of 32 channels x 128 k, see
// gemm_prefill_tiled.hip) instead of the row-major one, so that one copy of the weights serves every M.  A lane's
// 16 bytes are the chunk (c = its K group, r = its channel within the block); a wave load then covers four runs of
// 256 contiguous bytes.  The nibble order inside the tiled dwords yields the natural k order, so the activations are
// used as they are.
// AUX: cache-policy bits of the weight loads (0 = default, 2 = non-temporal: weights are read once per launch and
// should not displace anything; measured 5 to 10 % faster, and a plain read probe gains 30 % from it).
constexpr int kCuLdsBytes = 160 * 1024;
constexpr int kEpochScaleBytes = 4 * kResidentMaxRows;
constexpr int kEpochAmaxBytes = 1024;  // 16 waves x 16 rows of fp32

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt_at_most() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// FQ: the kernel is handed fp16 activations (p.x16, rows p.ldx apart) and quantises them per token itself, exactly as
// quantize_act_kernel would (Sec. 3 "per token"; Eq. (2), z = 0): the workgroup copies the fp16 rows into LDS, finds
// the row maxima (one barrier), and then every wave quantises the k steps it multiplies into a second LDS area and
// picks its operands from there: the waves' parts are disjoint, so nothing but the maxima crosses waves.  One launch instead of two for a linear at token-generation sizes (the
// kind of fusion across operators the paper's engine relies on, Sec. 6.1).  M <= 4: every workgroup repeats the
// quantisation, which costs about ten vector instructions per value, so beyond a few rows a launch of its own is
// cheaper.
//
// XW (tiled weights only): every wave stages its own k steps.  Beyond some thirty tokens the rows no longer fit in LDS
// whole, and in operand order a load from memory touches sixteen cache lines.  But a wave only ever multiplies its own
// k steps, and a k step of a row is exactly one 128-byte line: so each wave copies, window by window, the 16 MT rows of
// a few of its k steps into a private piece of LDS (LDS-direct loads of whole lines, eight rows per load, the 16-byte
// slots of a row swizzled as in the large-M kernel so that the sixteen rows of an operand read fall into different
// banks) and picks its operands from there.  No barrier is involved until the operands are in registers; the windows
// lie where the partial sums will go later, so one barrier separates the two uses.
//
// K slices (p.ks_per_slice < ceil(K / 128), raw sums only): workgroup (x, y) multiplies the k steps
// [y * ks_per_slice, (y + 1) * ks_per_slice) of its channels and writes slab y of p.acc_out ([slices][M][N]); a second
// kernel adds the slabs and dequantises.  That is how a K too long for a wave's registers is served, and it divides the
// activations a workgroup has to bring in by the number of slices.
//
// SWIGLU (fp16 output only): the weights are those of the gate and up projections with their channels interleaved
// (channel 2 i = gate_i, 2 i + 1 = up_i, N = 2 I), and the epilogue stores h = silu(gate) * up, I values per token,
// instead of the 2 I outputs (Sec. 6.1: glue operators folded into their neighbours).  The four channels an epilogue
// item holds are two such pairs; ranges and chunks are multiples of 4 channels, so no pair is ever split.
//
// NORM (with FQ): the rows handed over are the residual stream's; the workgroup first forms r = fp16(res + x) and
// y = fp16(r * rsqrt(mean r^2 + eps) * gamma) in place in its LDS copy (two passes in which every thread works on the
// same chunks, one barrier for the sum of squares between them, the row maxima falling out of the second), and the
// quantiser goes on from y.  The first workgroup writes r (the residual stream that goes on) and, on request, y.
template <int MT, int XS, int P, int WAVES, bool ACC_OUT, bool TILED, int AUX, bool FQ = false, bool XW = false,
          bool SWIGLU = false, bool NORM = false>
__global__ __launch_bounds__(WAVES * 64) void gemm_decode_resident_kernel(DecodeArgs p) {
    static_assert(!NORM || FQ, "the norm sits in front of the fused quantiser");
    static_assert(!FQ || (MT == 1 && !ACC_OUT), "the fused quantiser serves up to four tokens and the fp16 output");
    static_assert(!SWIGLU || (TILED && !ACC_OUT), "SiLU * up in the epilogue: tiled weights, fp16 output");
    static_assert(!XW || (TILED && !FQ), "per-wave staging: tiled weights, quantised activations");
    extern __shared__ __attribute__((aligned(16))) uint8_t epoch_lds[];
    float *sw_lds = (float *)epoch_lds;
    float *amax_lds = (float *)(epoch_lds + kEpochScaleBytes);  // FQ: [wave][16] row maxima of the waves' k steps
    v4i *part = (v4i *)(epoch_lds + kEpochScaleBytes + kEpochAmaxBytes);  // [set][q][mt][wave][lane]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // Uniform over the wave, and said so where the activations are staged whole: what derives from it (k steps, their
    // liveness) becomes scalar arithmetic, and a wave's first load goes out some hundred nanoseconds earlier (measured
    // 2 to 4 % on a 5 to 13 us GEMM at one to four tokens).  With per-wave windows the same change measured 1 to 2 %
    // slower, so there the compiler keeps its own view.
    const int wave = XW ? tid >> 6 : __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15;  // row of the 16-row operand tile
    const int g = lane >> 4;  // K group of the lane
    const int R = p.chunk_rows;
    const int row0 = blockIdx.x * p.rows_per_wg;
    const int row_end = min(p.N, row0 + p.rows_per_wg);
    const int chunks = max(0, (row_end - row0 + R - 1) / R);

    constexpr unsigned kNowhere = 0xFFFFFFF0u;  // beyond the buffer: such a load returns zeros and touches no memory
    const int ks_total = (p.K + 127) >> 7;
    const int ks_first = (int)blockIdx.y * p.ks_per_slice;       // this workgroup's slice of K, in k steps
    const int ks_limit = min(ks_total, ks_first + p.ks_per_slice);
    if (ACC_OUT) p.acc_out += (size_t)blockIdx.y * (size_t)p.M * (size_t)p.N;  // its slab of raw sums
    auto k_step = [&](int i) {
        constexpr int kPaired = 2 * (XS / 2);
        return ks_first + (i < kPaired ? ((i >> 1) * WAVES + wave) * 2 + (i & 1) : kPaired * WAVES + wave);
    };
    // whether this lane's K group of the wave's k step i exists; evaluated where it is used, so that the steps' address
    // arithmetic does not stand between the start of the wave and its first loads
    auto live_step = [&](int i) {
        const int ks = k_step(i);
        return ks < ks_limit && (ks * 128 + 32 * g) < p.K;
    };

    // Issue order: activations, scales, weights.  A compute unit accepts only some 40 to 50 outstanding wave-wide
    // loads; whatever is issued behind that many waits for the first returns, a memory latency later.  The weight
    // prefetch is that many, so the small loads the first multiplication depends on must be ahead of it, not behind.
    //
    // Activations.  Every wave needs its own k steps of all M rows as MFMA operands.  Fetched straight from memory
    // in operand order a wave-wide load touches 16 cache lines and uses half of each, and at M = 1 all sixteen token
    // lanes fetch the same row.  So, when they fit, the workgroup copies the M rows into LDS once with LDS-direct
    // loads of whole 1 KB pieces (p.x_lds_pitch > 0) and every wave picks its operands from there.
    v4u xraw[XS][MT][2];
    const int pitch = p.x_lds_pitch;  // FQ: always staged (the launcher sees to it that the rows fit)
    // XW: a wave's window holds kWindow k steps of 16 MT rows x 128 bytes and starts where the partial sums go later
    constexpr int kStepBytes = MT * 2048;
    constexpr int kWindowRoom = (kCuLdsBytes - kEpochScaleBytes - kEpochAmaxBytes) / (WAVES * kStepBytes);
    constexpr int kWindow = kWindowRoom < 1 ? 1 : (kWindowRoom > XS ? XS : kWindowRoom);
    constexpr int kWindows = (XS + kWindow - 1) / kWindow;
    static_assert(!XW || kWindowRoom >= 1, "a wave's window must hold at least one k step");
    const uint8_t *const window = epoch_lds + kEpochScaleBytes + kEpochAmaxBytes + wave * (kWindow * kStepBytes);
    const unsigned window_lds = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)(lds_ptr_t)window);
    const v4i xw_rsrc = [&] {
        const unsigned long long b = (unsigned long long)p.xq;
        v4i rs;
        rs.x = __builtin_amdgcn_readfirstlane((int)(unsigned)b);
        rs.y = __builtin_amdgcn_readfirstlane((int)(unsigned)((b >> 32) & 0xFFFFu));
        rs.z = __builtin_amdgcn_readfirstlane((int)((unsigned)p.M * (unsigned)p.K));
        rs.w = 0x00020000;
        return rs;
    }();
    // k step i of this wave into slot j of its window.  Load L brings in rows 8 L .. 8 L + 7: lane -> row 8 L + lane / 8,
    // 16-byte slot lane % 8 of that row, which receives the row's piece slot ^ fx(row), fx(row) = (row & 7) ^ ((row >> 3) & 1).
    // Rows past M, k steps past the slice and k past K are not fetched and read as zeros.
    auto stage = [&](int i, int j) {
        const int ks = k_step(i);
#pragma unroll
        for (int L = 0; L < 2 * MT; ++L) {
            const int row = 8 * L + (lane >> 3);
            const int piece = (lane & 7) ^ (lane >> 3) ^ (L & 1);
            const int k0 = ks * 128 + piece * 16;
            const unsigned src = (ks < ks_limit && row < p.M && k0 < p.K) ? (unsigned)row * (unsigned)p.K + (unsigned)k0 : kNowhere;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :
                         : "s"(window_lds + (unsigned)(j * kStepBytes + L * 1024)), "v"(src), "s"(xw_rsrc)
                         : "memory", "m0");
        }
    };
    // operands of k step i from slot j: lane (r, g) multiplies k = 32 g + 16 h .. + 15 of row 16 mt + r, i.e. piece 2 g + h
    auto pick = [&](int i, int j) {
        const int fxr = (r & 7) ^ (r >> 3);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                xraw[i][mt][h] = *(const v4u *)(window + j * kStepBytes + (16 * mt + r) * 128 + (((2 * g + h) ^ fxr) << 4));
    };
    if constexpr (FQ) {
        // the fp16 rows go to LDS in 1 KB pieces, as the int8 rows do in the other form
        const unsigned long long x_bytes = ((unsigned long long)(p.M - 1) * (unsigned long long)p.ldx + (unsigned long long)p.K) * 2ull;
        const v4i x_rsrc = [&] {
            const unsigned long long b = (unsigned long long)p.x16;
            v4i r;
            r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)b);
            r.y = __builtin_amdgcn_readfirstlane((int)(unsigned)((b >> 32) & 0xFFFFu));
            r.z = __builtin_amdgcn_readfirstlane((int)(unsigned)x_bytes);
            r.w = 0x00020000;
            return r;
        }();
        const int per_row = (2 * p.K + 1023) >> 10;
        const int pieces = p.M * per_row;
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        auto copy_rows = [&](v4i rsrc, long long ld, int lds_offset) {
            const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)(lds_ptr_t)(epoch_lds + lds_offset));
            int m = 0, c = wave_u;  // piece j = wave, wave + WAVES, ... is piece c of row m, kept without a division
            for (int j = wave_u; j < pieces; j += WAVES, c += WAVES) {
                while (c >= per_row) c -= per_row, ++m;
                const unsigned in_row = (unsigned)(c * 1024 + lane * 16);
                const unsigned src = in_row < 2u * (unsigned)p.K ? (unsigned)((unsigned long long)m * (unsigned long long)ld * 2ull) + in_row : kNowhere;
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                             :
                             : "s"(base + (unsigned)(m * p.x16_lds_pitch + c * 1024)), "v"(src), "s"(rsrc)
                             : "memory", "m0");
            }
        };
        copy_rows(x_rsrc, p.ldx, p.x16_lds_offset);
        if constexpr (NORM) {
            if (p.res16 != nullptr) {  // uniform
                const unsigned long long res_bytes = ((unsigned long long)(p.M - 1) * (unsigned long long)p.ldres + (unsigned long long)p.K) * 2ull;
                const unsigned long long b = (unsigned long long)p.res16;
                v4i rr;
                rr.x = __builtin_amdgcn_readfirstlane((int)(unsigned)b);
                rr.y = __builtin_amdgcn_readfirstlane((int)(unsigned)((b >> 32) & 0xFFFFu));
                rr.z = __builtin_amdgcn_readfirstlane((int)(unsigned)res_bytes);
                rr.w = 0x00020000;
                copy_rows(rr, p.ldres, p.res_lds_offset);
            }
        }
    } else if constexpr (XW) {
        // every window but the last: copy, wait, pick.  Nothing else is outstanding yet, so the wait is for the copy.
#pragma unroll
        for (int wdw = 0; wdw + 1 < kWindows; ++wdw) {
#pragma unroll
            for (int j = 0; j < kWindow; ++j) stage(wdw * kWindow + j, j);
            wait_vmcnt_at_most<0>();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < kWindow; ++j) pick(wdw * kWindow + j, j);
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the operands are in registers before the window is refilled
            __builtin_amdgcn_sched_barrier(0);
        }
        // the last window is only requested here; it is picked up below, with the weight prefetch already behind it
#pragma unroll
        for (int j = 0; j < kWindow; ++j)
            if ((kWindows - 1) * kWindow + j < XS) stage((kWindows - 1) * kWindow + j, j);
    } else if (pitch > 0) {
        const v4i x_rsrc = [&] {
            const unsigned long long b = (unsigned long long)p.xq;
            v4i r;
            r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)b);
            r.y = __builtin_amdgcn_readfirstlane((int)(unsigned)((b >> 32) & 0xFFFFu));
            r.z = __builtin_amdgcn_readfirstlane((int)((unsigned)p.M * (unsigned)p.K));
            r.w = 0x00020000;
            return r;
        }();
        const unsigned x_base = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)(lds_ptr_t)(epoch_lds + p.x_lds_offset));
        const int per_row = (p.K + 1023) >> 10;
        const int pieces = p.M * per_row;
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        int m = 0, c = wave_u;  // piece j = 1 KB of row j / per_row = piece c of row m, kept without a division
        for (int j = wave_u; j < pieces; j += WAVES, c += WAVES) {
            while (c >= per_row) c -= per_row, ++m;
            const unsigned in_row = (unsigned)(c * 1024 + lane * 16);
            const unsigned src = in_row < (unsigned)p.K ? (unsigned)m * (unsigned)p.K + in_row : kNowhere;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :
                         : "s"(x_base + (unsigned)(m * pitch + c * 1024)), "v"(src), "s"(x_rsrc)
                         : "memory", "m0");
        }
    } else {
#pragma unroll
        for (int i = 0; i < XS; ++i) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                // rows past M read row M-1: what they produce lands in output columns that are never stored;
                // a dead K group reads the start of the row: it meets zero weights
                const int m = min(16 * mt + r, p.M - 1);
                const v4u *px = (const v4u *)(p.xq + (size_t)m * p.K + (live_step(i) ? k_step(i) * 128 + 32 * g : 0));
                xraw[i][mt][0] = px[0];
                xraw[i][mt][1] = px[1];
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    const int n_sw = ACC_OUT ? 0 : max(0, row_end - row0);
    float sw_first = 0.f;
    float sa[MT];
    if (!ACC_OUT) {
        if (tid < n_sw) sw_first = p.s_w[row0 + tid];
        if constexpr (!FQ) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) sa[mt] = p.s_a[min(16 * mt + r, p.M - 1)];
        }
    }
    v4u gam[2] = {v4u{0, 0, 0, 0}, v4u{0, 0, 0, 0}};  // NORM: the gains of the chunks this thread normalises (K <= 16 threads)
    if constexpr (NORM) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = tid + i * WAVES * 64;
            if (c < (p.K >> 3)) gam[i] = ((const v4u *)p.gamma)[c];
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    const unsigned w_bytes = TILED ? (unsigned)((size_t)((p.N + 31) >> 5) * ks_total * kTiledBlockBytes)
                                   : (unsigned)((size_t)p.N * (p.K >> 1));
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, w_bytes, 0x00020000);
    unsigned w_off[XS];
    const unsigned w_stride = (unsigned)(p.K >> 1);
    auto w_row = [&](int c) {
        const int n = row0 + R * c + r;
        if (!(c < chunks && r < R && n < row_end)) return kNowhere;
        return TILED ? (unsigned)(n >> 5) * (unsigned)(ks_total * kTiledBlockBytes) + (unsigned)(n & 31) * 16u
                     : (unsigned)n * w_stride;
    };
    auto w_load = [&](unsigned row, unsigned off) {
        const unsigned o = (row >= kNowhere || off >= kNowhere) ? kNowhere : row + off;
        return __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, o, 0, AUX);
    };
    v4u wreg[P][XS];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const unsigned row = w_row(q);
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            if (q == 0) {
                // a step's offset is worked out right before its first load and the compiler is held to that: with
                // all offsets first, a wave with 14 steps would spend half a microsecond before its first weight load
                const int ks = k_step(i);
                w_off[i] = !live_step(i) ? kNowhere : TILED ? (unsigned)(ks * kTiledBlockBytes + 512 * g) : (unsigned)(ks * 64 + 16 * g);
            }
            wreg[q][i] = w_load(row, w_off[i]);
            if (q == 0) __builtin_amdgcn_sched_barrier(0);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (FQ) {
        // The row maxima are found by the workgroup together; then every wave quantises the k steps it multiplies,
        // its lanes sharing the work (were every lane to quantise the operands it multiplies itself, a wave would
        // spend some 1600 vector instructions on it whatever M is: measured slower than a quantiser launch of its own).
        constexpr int T = WAVES * 64;
        wait_vmcnt_at_most<P * XS>();  // the copy and the scales are in: only the weight loads issued behind them remain
        __builtin_amdgcn_sched_barrier(0);
        if (tid < n_sw) sw_lds[tid] = sw_first;
        lds_barrier();
        uint8_t *x16 = epoch_lds + p.x16_lds_offset;
        uint8_t *xq_lds = epoch_lds + p.x_lds_offset;
        const int chunks_row = p.K >> 3;  // 8 fp16 = 16 bytes
        sa[0] = 0.f;
        if constexpr (NORM) {
            // r = res + x in place, and the rows' sums of squares; a thread's chunks are tid and tid + T in both passes
            float *sum_lds = amax_lds + 64;
            const uint8_t *res_l = epoch_lds + p.res_lds_offset;
            const bool writer = blockIdx.x == 0;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                if (m < p.M) {  // uniform
                    float ss = 0.f;
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const int c = tid + i * T;
                        if (c < chunks_row) {
                            v4u *slot = (v4u *)(x16 + m * p.x16_lds_pitch + c * 16);
                            v4u rv = *slot;
                            if (p.res16 != nullptr) {
                                rv = add_halves8(*(const v4u *)(res_l + m * p.x16_lds_pitch + c * 16), rv);
                                *slot = rv;
                            }
                            if (writer && p.r_out != nullptr) ((v4u *)(p.r_out + (size_t)m * p.K))[c] = rv;
                            ss = add_squares8(rv, ss);
                        }
                    }
                    ss = wave_sum(ss);
                    if (lane == 0) sum_lds[wave * 4 + m] = ss;
                }
            }
            lds_barrier();
            // y = r * rsqrt(mean r^2 + eps) * gamma in place, and the maxima of |y| on the way
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                if (m < p.M) {
                    float total = 0.f;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w) total += sum_lds[w * 4 + m];
                    const float inv = rms_inverse(total, p.K, p.eps);
                    unsigned pm2 = 0u;
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const int c = tid + i * T;
                        if (c < chunks_row) {
                            v4u *slot = (v4u *)(x16 + m * p.x16_lds_pitch + c * 16);
                            const v4u y = norm_scale8(*slot, inv, gam[i]);
                            *slot = y;
                            if (writer && p.y_out != nullptr) ((v4u *)(p.y_out + (size_t)m * p.K))[c] = y;
                            pm2 = absmax8_packed(y, pm2);
                        }
                    }
                    const float pm = wave_max_nonneg(absmax_packed_value(pm2));
                    if (lane == 0) amax_lds[wave * 4 + m] = pm;
                }
            }
        } else {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                if (m < p.M) {  // uniform
                    unsigned pm2 = 0u;
                    for (int c = tid; c < chunks_row; c += T) pm2 = absmax8_packed(*(const v4u *)(x16 + m * p.x16_lds_pitch + c * 16), pm2);
                    const float pm = wave_max_nonneg(absmax_packed_value(pm2));
                    if (lane == 0) amax_lds[wave * 4 + m] = pm;
                }
            }
        }
        lds_barrier();
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            if (m < p.M) {
                float amax = 0.f;
#pragma unroll
                for (int w = 0; w < WAVES; ++w) amax = fmaxf(amax, amax_lds[w * 4 + m]);
                const RowQuantizer rq(amax, 127.0f, -127.f, 127.f);  // amax == 0 gives scale 0
                if (tid == 0 && p.s_a_out != nullptr && blockIdx.x == 0) p.s_a_out[m] = rq.scale;
                if (min(r, p.M - 1) == m) sa[0] = rq.scale;
                // Every wave quantises the k steps it multiplies, all lanes sharing the work (16 chunks of 8 values
                // per step; units of 4 values, which spread more evenly, measured 2 % slower), into the int8 copy of
                // the row: the waves' parts are disjoint and a wave reads back only its own, so no barrier follows --
                // LDS serves a wave's accesses in program order.
                const bool zero_row = amax == 0.f;
                for (int u = lane; u < XS * 16; u += 64) {
                    const int ks = k_step(u >> 4), k0 = ks * 128 + (u & 15) * 8;
                    if (ks < ks_limit && k0 < p.K) {
                        v2u codes = v2u{0u, 0u};
                        if (!zero_row) {
                            float xf[8];
                            halves8(*(const v4u *)(x16 + m * p.x16_lds_pitch + k0 * 2), xf);
                            codes = rq.packed8_own_max(xf);
                        }
                        *(v2u *)(xq_lds + m * pitch + k0) = codes;
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            const int m = min(r, p.M - 1);
            const v4u *px = (const v4u *)(xq_lds + m * pitch + (live_step(i) ? k_step(i) * 128 + 32 * g : 0));
            xraw[i][0][0] = px[0];
            xraw[i][0][1] = px[1];
        }
    } else if constexpr (XW) {
        // the last window and the scales behind it are in once at most the P XS weight loads issued after them remain
        wait_vmcnt_at_most<P * XS>();
        __builtin_amdgcn_sched_barrier(0);
        if (!ACC_OUT) {
            if (tid < n_sw) sw_lds[tid] = sw_first;
        }
#pragma unroll
        for (int j = 0; j < kWindow; ++j)
            if ((kWindows - 1) * kWindow + j < XS) pick((kWindows - 1) * kWindow + j, j);
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        lds_barrier();  // every wave has its operands: from here on the windows' memory takes the partial sums
    } else if (pitch > 0) {
        // The copy, and the scales behind it, are in once at most the P XS weight loads issued after them are
        // outstanding (loads return in order).  The compiler does not know of the copy, so the wait is spelled out;
        // the scales are parked in LDS behind it, where the compiler's own wait for them is already satisfied.
        wait_vmcnt_at_most<P * XS>();
        __builtin_amdgcn_sched_barrier(0);
        if (!ACC_OUT) {
            if (tid < n_sw) sw_lds[tid] = sw_first;
        }
        lds_barrier();
        const uint8_t *xs = epoch_lds + p.x_lds_offset;
#pragma unroll
        for (int i = 0; i < XS; ++i) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = min(16 * mt + r, p.M - 1);
                const v4u *px = (const v4u *)(xs + m * pitch + (live_step(i) ? k_step(i) * 128 + 32 * g : 0));
                xraw[i][mt][0] = px[0];
                xraw[i][mt][1] = px[1];
            }
        }
    } else if (!ACC_OUT) {
        if (tid < n_sw) sw_lds[tid] = sw_first;
    }
    v4i xop[XS][MT][2];
#pragma unroll
    for (int i = 0; i < XS; ++i) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const v4u x = xraw[i][mt][h];
                xop[i][mt][h] = TILED ? v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w} : x_operand(x);
            }
        }
    }

    int set = 0;
    for (int c0 = 0; c0 < chunks; c0 += P) {
        v4i *mine = part + ((size_t)set * (P * MT * WAVES) + wave) * 64 + lane;
        // Every epoch walks all P chunk slots: a slot past the end of the range holds zeros (its loads went nowhere)
        // and costs a few idle MFMAs, while a branch here would make the compiler merge loaded and unloaded
        // registers behind it, i.e. wait for the whole prefetch at every turn.
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const unsigned next = w_row(c0 + q + P);
            // two chains of sums per column tile while there are few tiles, so that no MFMA waits for the one before
            // it; from three tiles on the tiles themselves are chains enough
            constexpr int kChains = MT >= 3 ? 1 : 2;
            v4i acc[MT][kChains];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int ch = 0; ch < kChains; ++ch) acc[mt][ch] = v4i{0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < XS; ++i) {
                // convert first, refill second: the old register is dead when the new load is issued, so the load can
                // go into the very register it replaces and stay in flight until that register's next turn
                const v4i w0 = TILED ? w_operand_tiled(wreg[q][i].x, wreg[q][i].y) : w_operand(wreg[q][i].x, wreg[q][i].y);
                const v4i w1 = TILED ? w_operand_tiled(wreg[q][i].z, wreg[q][i].w) : w_operand(wreg[q][i].z, wreg[q][i].w);
                __builtin_amdgcn_sched_barrier(0);
                wreg[q][i] = w_load(next, w_off[i]);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (kChains == 2) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        acc[mt][0] = mfma_i8_16x16x64(w0, xop[i][mt][0], acc[mt][0]);
                        acc[mt][1] = mfma_i8_16x16x64(w1, xop[i][mt][1], acc[mt][1]);
                    }
                } else {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt][0] = mfma_i8_16x16x64(w0, xop[i][mt][0], acc[mt][0]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt][0] = mfma_i8_16x16x64(w1, xop[i][mt][1], acc[mt][0]);
                }
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                mine[(size_t)((q * MT + mt) * WAVES) * 64] = kChains == 2 ? acc[mt][0] + acc[mt][kChains - 1] : acc[mt][0];
        }
        lds_barrier();  // LDS only: the weight prefetch stays in flight
        // one item = the four consecutive channels 4 g .. 4 g + 3 of chunk c0 + q for token 16 mt + r
        for (int it = tid; it < P * MT * 64; it += WAVES * 64) {
            const int mt = (it >> 6) % MT, q = (it >> 6) / MT;
            const int m = 16 * mt + r;
            const int local = R * (c0 + q) + 4 * g;  // relative to row0
            const int n = row0 + local;
            if (m >= p.M || 4 * g >= R || n >= row_end) continue;
            const v4i *src = part + ((size_t)set * (P * MT * WAVES) + (size_t)(q * MT + mt) * WAVES) * 64 + lane;
            v4i s = src[0];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) s += src[w * 64];
            if (ACC_OUT) {
                store4_acc(p, m, n, row_end, s);
            } else {
                float4 sw;  // the range is a multiple of 4 channels long, so the four scales are inside the staged part
                sw.x = sw_lds[local];
                sw.y = sw_lds[local + 1];
                sw.z = sw_lds[local + 2];
                sw.w = sw_lds[local + 3];
                float sa_m = sa[0];
#pragma unroll
                for (int t = 1; t < MT; ++t) sa_m = mt == t ? sa[t] : sa_m;
                if constexpr (SWIGLU)
                    store4_h(p, m, n, s, sa_m, sw);
                else
                    store4_f16(p, m, n, row_end, s, sa_m, sw);
            }
        }
        set ^= 1;
    }
}

// Registers a wave needs, roughly: the weight prefetch, the resident activations, and some forty-five for the rest.
// 8 waves have 256 registers each (one workgroup per compute unit), 16 waves 128.  A prefetch of one chunk always
// exists (at the longest K it spills a few registers), deeper ones only where they fit.
constexpr bool epoch_fits(int mt, int xs, int prefetch, int waves) {
    const bool regs = prefetch == 1 || 4 * prefetch * xs + 8 * xs * mt + 45 <= (waves == 8 ? 240 : 128);
    return regs && prefetch * mt * waves <= 64;
}

constexpr int epoch_lds_bytes(int mt, int prefetch, int waves, int sets) {
    return kEpochScaleBytes + kEpochAmaxBytes + sets * prefetch * mt * waves * 1024;
}

// (column tiles, k steps per wave, waves) for which the form with per-wave staging is instantiated
constexpr bool wide_shape_exists(int mt, int xs, int waves) {
    if (mt == 1) return (waves == 8 && ((xs >= 1 && xs <= 8) || xs == 11 || xs == 14)) || (waves == 16 && xs >= 5 && xs <= 8);
    if (mt == 2) return (waves == 16 && xs >= 1 && xs <= 4) || (waves == 8 && xs >= 1 && xs <= 7);
    if (mt == 3 || mt == 4) return waves == 8 && xs >= 1 && xs <= 5;
    return false;
}
// ... and those of one column tile for which the form with the fused quantiser is
constexpr bool fused_shape_exists(int xs, int waves) {
    return (xs >= 1 && xs <= 8 && (waves == 8 || waves == 16)) || (waves == 8 && (xs == 11 || xs == 14));
}

template <int MT, int XS, int P, int WAVES, bool ACC_OUT, bool TILED, int AUX, bool FQ = false, bool XW = false,
          bool SWIGLU = false, bool NORM = false>
static hipError_t launch_epoch_one(const DecodeArgs &p, int grid, int sets, bool prepare_only, hipStream_t stream) {
    constexpr auto kernel = gemm_decode_resident_kernel<MT, XS, P, WAVES, ACC_OUT, TILED, AUX, FQ, XW, SWIGLU, NORM>;
    static_assert(epoch_lds_bytes(MT, P, WAVES, 2) <= kCuLdsBytes, "both sets of slots must fit the compute unit's LDS");
    if (const hipError_t e = allow_lds<kernel>(kCuLdsBytes); e != hipSuccess) return e;
    if (prepare_only) return hipSuccess;
    // The activations are staged in LDS behind the slots of the partial sums when they fit: rows padded to whole
    // 1 KB pieces (the unit of the copy) plus 16 bytes, so that the sixteen token rows of an operand read fall into
    // different banks.  p.x_lds_pitch < 0 on entry = the caller wants them read straight from memory.
    DecodeArgs a = p;
    int lds = epoch_lds_bytes(MT, P, WAVES, sets);
    const long long pitch = ((p.K + 1023) / 1024) * 1024 + 16;
    a.x_lds_pitch = 0;
    a.x_lds_offset = 0;
    const int ks_total = (p.K + 127) / 128;
    if (a.ks_per_slice <= 0 || a.ks_per_slice > ks_total) a.ks_per_slice = ks_total;
    const int slices = (ks_total + a.ks_per_slice - 1) / a.ks_per_slice;
    if (slices > 1 && !ACC_OUT) return hipErrorInvalidConfiguration;  // slices of K hand back raw sums
    if (XW) {
        // the waves' windows overlay the slots of the partial sums
        constexpr int kStepBytes = MT * 2048;
        constexpr int kRoom = (kCuLdsBytes - kEpochScaleBytes - kEpochAmaxBytes) / (WAVES * kStepBytes);
        constexpr int kWindow = kRoom < 1 ? 1 : (kRoom > XS ? XS : kRoom);
        const int windows = kEpochScaleBytes + kEpochAmaxBytes + WAVES * kWindow * kStepBytes;
        if (windows > lds) lds = windows;
    } else if (FQ) {
        // fused quantiser: the int8 rows and, behind them, the fp16 rows (whole 1 KB pieces) must both fit
        const long long pitch16 = ((2ll * p.K + 1023) / 1024) * 1024;
        const long long copies16 = NORM ? 2 : 1;  // with the norm in front the residual rows are staged too
        if (p.M > 4 || lds + (pitch + copies16 * pitch16) * p.M > kCuLdsBytes) return hipErrorInvalidConfiguration;
        if (NORM && (p.K >> 3) > 2 * WAVES * 64) return hipErrorInvalidConfiguration;  // two chunks a thread
        a.x_lds_pitch = (int)pitch;
        a.x_lds_offset = lds;
        a.x16_lds_pitch = (int)pitch16;
        a.x16_lds_offset = lds + (int)(pitch * p.M);
        a.res_lds_offset = a.x16_lds_offset + (int)(pitch16 * p.M);
        lds += (int)((pitch + copies16 * pitch16) * p.M);
    } else if (p.x_lds_pitch >= 0 && lds + pitch * p.M <= kCuLdsBytes) {
        a.x_lds_pitch = (int)pitch;
        a.x_lds_offset = lds;
        lds += (int)(pitch * p.M);
    }
    hipLaunchKernelGGL(kernel, dim3(grid, slices), dim3(WAVES * 64), lds, stream, a);
    return hipGetLastError();
}

}  // namespace w4a8
