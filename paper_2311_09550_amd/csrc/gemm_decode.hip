// Weight-streaming W4A8 GEMM for small M (the self-decoding stage, which the
// paper calls memory-intensive: Sec. 4.1).  Time goes to reading the packed
// weights once from HBM, so both kernels here are built around that stream:
//
//   * a lane loads 16 packed bytes (32 weights) straight from global memory
//     into registers, converts them with the sign-bit placement of Sec. 5.3
//     and feeds two 16x16x64 int8 MFMAs; the activations are byte-permuted to
//     the same k order;
//   * the waves of a workgroup take interleaved 128-wide k steps of the same
//     16 output channels, so that together they read a contiguous run of
//     every weight row; their partial sums meet in LDS (integer sums: any
//     order gives the same bits);
//   * the dequantisation of Eq. (6),(7) is applied once, to the complete sum.
//
// gemm_decode_resident_kernel (M <= 16 and friends): a persistent workgroup
// walks over many 16-channel row blocks.  A wave's k steps are the same for
// every row block, so its activation operands are loaded and permuted ONCE
// and stay in registers; per row block only weights are loaded, and the loads
// of the next block are issued as soon as a register is consumed, so a wave
// always has its full set of 16-byte loads in flight.
//
// gemm_decode_stream_kernel: the general form (any M <= 64, any K), one row
// block per workgroup, activations re-read from cache for every block.
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

// ---------------------------------------------------------------------------------------------
// Persistent kernel with register-resident activations.  MT = ceil(M/16) column tiles, XS = k steps
// per wave (ceil(ceil(K/128) / WAVES) <= XS), P = row chunks of weight loads a wave keeps in flight.
//
// Workgroup b owns the contiguous output channels [b * rows_per_wg, (b + 1) * rows_per_wg) and walks
// them in chunks of 16 (one MFMA tile); rows_per_wg is a multiple of 4 chosen by the launcher so that
// every workgroup streams the same number of weight bytes -- with whole 16-row blocks as the unit, a
// 5120-channel layer on 256 compute units would leave a quarter of them with twice the work.  The
// last chunk of a range may be partial: its missing rows are simply not loaded.
//
// The waves of a workgroup are not tied together by a barrier per chunk: each wave adds its partial
// sums into an LDS tile with LDS atomics and then bumps the tile's arrival counter; the wave that
// arrives last owns the complete sums, clears the tile and writes the outputs.  Tiles form a ring of
// 2*kEpoch slots and the workgroup meets at a barrier every kEpoch chunks, so a slot is always
// cleared before its next use (its previous user finished two barriers earlier).
//
// All of that synchronisation concerns LDS only, so it is written with LDS-only fences: an ordinary
// workgroup fence or __syncthreads() would also wait for the wave's outstanding global loads, i.e.
// drain the weight prefetch at every chunk.  For the same reason the epilogue reads nothing from
// global memory: s_a sits in a register and the s_w of the workgroup's channels in LDS.
constexpr int kEpoch = 8;

__device__ __forceinline__ void lds_release() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local"); }
__device__ __forceinline__ void lds_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local"); }
__device__ __forceinline__ void lds_barrier() {
    lds_release();
    __builtin_amdgcn_s_barrier();
    lds_acquire();
}

//
// TILED: p.wp is the tiled weight array of the large-M kernel (2 KB blocks of 32 channels x 128 k, see
// gemm_prefill_tiled.hip) instead of the row-major one, so that one copy of the weights serves every M.  A lane's
// 16 bytes are the chunk (c = its K group, r = its channel within the block); a wave load then covers four runs of
// 256 contiguous bytes.  The nibble order inside the tiled dwords yields the natural k order, so the activations are
// used as they are.
template <int MT, int XS, int P, int WAVES, bool ACC_OUT, bool TILED>
__global__ __launch_bounds__(WAVES * 64) void gemm_decode_resident_kernel(DecodeArgs p) {
    __shared__ int tile[2 * kEpoch][MT][256];  // sixteen-fold sums of one chunk each
    __shared__ int arrived[2 * kEpoch];
    __shared__ float sw_lds[ACC_OUT ? 1 : kResidentMaxRows];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 15;  // row of the 16-row operand tile
    const int g = lane >> 4;  // K group of the lane
    const int row0 = blockIdx.x * p.rows_per_wg;
    const int row_end = min(p.N, row0 + p.rows_per_wg);
    const int chunks = (row_end - row0 + 15) >> 4;

    for (int i = tid; i < 2 * kEpoch * MT * 256; i += WAVES * 64) (&tile[0][0][0])[i] = 0;
    if (tid < 2 * kEpoch) arrived[tid] = 0;
    // The weight scales of this workgroup's channels go to LDS.  Their loads are issued first and stored
    // last, so that nothing waits for them before the weight prefetch is out.
    const int n_sw = ACC_OUT ? 0 : row_end - row0;
    float sw_first = 0.f;
    float sa[MT];
    if (!ACC_OUT) {
        if (tid < n_sw) sw_first = p.s_w[row0 + tid];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) sa[mt] = p.s_a[min(16 * mt + r, p.M - 1)];
    }

    const int ks_total = (p.K + 127) >> 7;
    // K % 32 == 0, so a lane's 32-wide K group is entirely inside or outside K; only the last step can be partial.
    // Weights are read with buffer loads: an offset past the end of the buffer returns zeros and touches no memory.
    // That is how a dead K group (K % 128 != 0), a wave without a step, a row outside the workgroup's range and a
    // finished walk are handled, with neither a branch nor a select nor a wasted access.
    constexpr unsigned kNowhere = 0xFFFFFFF0u;
    const unsigned w_bytes = TILED ? (unsigned)((size_t)((p.N + 31) >> 5) * ks_total * kTiledBlockBytes)
                                   : (unsigned)((size_t)p.N * (p.K >> 1));
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, w_bytes, 0x00020000);
    // k steps of this wave.  Where possible a wave takes two adjacent steps (128 contiguous bytes of every row,
    // i.e. whole 128-byte lines) -- steps i = 0 .. 2*(XS/2)-1 -- and, if XS is odd, one single step at the end.
    auto k_step = [&](int i) {
        constexpr int kPaired = 2 * (XS / 2);
        return i < kPaired ? ((i >> 1) * WAVES + wave) * 2 + (i & 1) : kPaired * WAVES + wave;
    };
    unsigned w_off[XS];
    bool live[XS];
#pragma unroll
    for (int i = 0; i < XS; ++i) {
        const int ks = k_step(i);
        live[i] = ks < ks_total && (ks * 128 + 32 * g) < p.K;
        w_off[i] = !live[i] ? kNowhere : TILED ? (unsigned)(ks * kTiledBlockBytes + 512 * g) : (unsigned)(ks * 64 + 16 * g);
    }

    const unsigned w_stride = (unsigned)(p.K >> 1);
    // byte offset of this lane's row in chunk c of the workgroup's range, or nowhere
    auto w_row = [&](int c) {
        const int n = row0 + 16 * c + r;
        if (!(c < chunks && n < row_end)) return kNowhere;
        return TILED ? (unsigned)(n >> 5) * (unsigned)(ks_total * kTiledBlockBytes) + (unsigned)(n & 31) * 16u
                     : (unsigned)n * w_stride;
    };
    auto w_load = [&](unsigned row, unsigned off) {
        const unsigned o = (row >= kNowhere || off >= kNowhere) ? kNowhere : row + off;
        return __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, o, 0, 0);
    };

    // The weight prefetch goes out before the activation loads: both are then in flight together, and waiting for
    // the (younger) activations cannot be scheduled ahead of issuing the weights.
    v4u wreg[P][XS];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const unsigned row = w_row(q);
#pragma unroll
        for (int i = 0; i < XS; ++i) wreg[q][i] = w_load(row, w_off[i]);
    }
    v4i xop[XS][MT][2];
#pragma unroll
    for (int i = 0; i < XS; ++i) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            // rows past M read row M-1: what they produce lands in output columns that are never stored;
            // a dead K group reads the start of the row: it meets zero weights
            const int m = min(16 * mt + r, p.M - 1);
            const v4u *px = (const v4u *)(p.xq + (size_t)m * p.K + (live[i] ? k_step(i) * 128 + 32 * g : 0));
            xop[i][mt][0] = TILED ? v4i{(int)px[0].x, (int)px[0].y, (int)px[0].z, (int)px[0].w} : x_operand(px[0]);
            xop[i][mt][1] = TILED ? v4i{(int)px[1].x, (int)px[1].y, (int)px[1].z, (int)px[1].w} : x_operand(px[1]);
        }
    }
    if (!ACC_OUT) {
        if (tid < n_sw) sw_lds[tid] = sw_first;
        for (int i = tid + WAVES * 64; i < n_sw; i += WAVES * 64) sw_lds[i] = p.s_w[row0 + i];
    }
    lds_barrier();  // tiles, counters and scales are in LDS; the weight prefetch stays in flight

    for (int c0 = 0; c0 < chunks; c0 += P) {
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const int c = c0 + q;
            if (c < chunks) {  // workgroup-uniform
                const unsigned next = w_row(c + P);
                v4i acc[MT][2];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[mt][0] = acc[mt][1] = v4i{0, 0, 0, 0};
                // No branch and no conditional assignment in here, so that a refill is a plain load into the register it
                // replaces and stays in flight until that register is used again.
#pragma unroll
                for (int i = 0; i < XS; ++i) {
                    const v4u w = wreg[q][i];
                    wreg[q][i] = w_load(next, w_off[i]);
                    const v4i w0 = TILED ? w_operand_tiled(w.x, w.y) : w_operand(w.x, w.y);
                    const v4i w1 = TILED ? w_operand_tiled(w.z, w.w) : w_operand(w.z, w.w);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        acc[mt][0] = mfma_i8_16x16x64(w0, xop[i][mt][0], acc[mt][0]);
                        acc[mt][1] = mfma_i8_16x16x64(w1, xop[i][mt][1], acc[mt][1]);
                    }
                }
                const int slot = c & (2 * kEpoch - 1);
                {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const v4i s = acc[mt][0] + acc[mt][1];
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            __hip_atomic_fetch_add(&tile[slot][mt][j * 64 + lane], s[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    }
                }
                lds_release();
                int seen = 0;
                if (lane == 0) seen = __hip_atomic_fetch_add(&arrived[slot], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                seen = __builtin_amdgcn_readfirstlane(seen);
                if (seen == WAVES - 1) {  // this wave arrived last: the sums are complete
                    lds_acquire();
                    if (lane == 0) arrived[slot] = 0;
                    const int local = 16 * c + 4 * g;  // first of this lane's four channels, relative to row0
                    const int n = row0 + local;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        v4i s;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            s[j] = tile[slot][mt][j * 64 + lane];
                            tile[slot][mt][j * 64 + lane] = 0;
                        }
                        const int m = 16 * mt + r;
                        if (m >= p.M || n >= row_end) continue;
                        if (ACC_OUT) {
                            store4_acc(p, m, n, row_end, s);
                        } else {
                            float4 sw;  // rows_per_wg is a multiple of 4, so the four scales are inside the staged range
                            sw.x = sw_lds[local];
                            sw.y = sw_lds[local + 1];
                            sw.z = sw_lds[local + 2];
                            sw.w = sw_lds[local + 3];
                            store4_f16(p, m, n, row_end, s, sa[mt], sw);
                        }
                    }
                }
                if (((c + 1) & (kEpoch - 1)) == 0) lds_barrier();
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// General kernel: one workgroup per 16*T output channels, U k steps of loads in flight per wave.
template <int MT, int T, int WAVES, int U, bool ACC_OUT, bool TILED>
__global__ __launch_bounds__(WAVES * 64) void gemm_decode_stream_kernel(DecodeArgs p) {
    constexpr int kThreads = WAVES * 64;
    __shared__ v4i red[WAVES * MT * T * 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 15;
    const int g = lane >> 4;
    const int n0 = blockIdx.x * (16 * T);
    const int ks_total = (p.K + 127) >> 7;

    const size_t w_stride = (size_t)(p.K >> 1);
    const uint8_t *wrow[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int n = min(n0 + 16 * t + r, p.N - 1);
        wrow[t] = TILED ? p.wp + ((size_t)(n >> 5) * ks_total) * kTiledBlockBytes + (n & 31) * 16 + 512 * g
                        : p.wp + (size_t)n * w_stride + 16 * g;
    }
    const int8_t *xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xrow[mt] = p.xq + (size_t)min(16 * mt + r, p.M - 1) * p.K + 32 * g;

    v4i acc[MT][T];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t) acc[mt][t] = v4i{0, 0, 0, 0};

    for (int ks0 = wave; ks0 < ks_total; ks0 += WAVES * U) {
        v4u wreg[U][T];
        v4u xreg[U][MT][2];
        // issue every load of the U steps before the first use; dead lanes read valid memory and are zeroed
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ks = ks0 + u * WAVES;
            const bool live = ks < ks_total && (ks * 128 + 32 * g) < p.K;
            const size_t ksafe = live ? (size_t)ks : 0;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const v4u v = TILED ? *(const v4u *)(wrow[t] + ksafe * kTiledBlockBytes - (live ? 0 : 512 * g))
                                    : *(const v4u *)(wrow[t] + ksafe * 64 - (live ? 0 : 16 * g));
                wreg[u][t] = live ? v : v4u{0, 0, 0, 0};
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const v4u *px = (const v4u *)(xrow[mt] + ksafe * 128 - (live ? 0 : 32 * g));
                xreg[u][mt][0] = px[0];
                xreg[u][mt][1] = px[1];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i xop[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const v4u x = xreg[u][mt][h];
                    xop[mt] = TILED ? v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w} : x_operand(x);
                }
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const v4u wf = wreg[u][t];
                    const v4i wop = TILED ? (h == 0 ? w_operand_tiled(wf.x, wf.y) : w_operand_tiled(wf.z, wf.w))
                                          : (h == 0 ? w_operand(wf.x, wf.y) : w_operand(wf.z, wf.w));
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
    for (int it = tid; it < kItems; it += kThreads) {
        const int l = it & 63, t = (it >> 6) % T, mt = (it >> 6) / T;
        const int m = 16 * mt + (l & 15);
        const int n = n0 + 16 * t + 4 * (l >> 4);
        if (m >= p.M || n >= p.N) continue;
        v4i s = red[it];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) s += red[w * kItems + it];
        store4<ACC_OUT>(p, m, n, s);
    }
}

// ---------------------------------------------------------------------------------------------

template <int MT, int XS, int P, int WAVES, bool ACC_OUT>
static hipError_t launch_resident_as(const DecodeArgs &p, bool tiled, int grid, hipStream_t stream) {
    if (tiled)
        hipLaunchKernelGGL((gemm_decode_resident_kernel<MT, XS, P, WAVES, ACC_OUT, true>), dim3(grid), dim3(WAVES * 64), 0,
                           stream, p);
    else
        hipLaunchKernelGGL((gemm_decode_resident_kernel<MT, XS, P, WAVES, ACC_OUT, false>), dim3(grid), dim3(WAVES * 64), 0,
                           stream, p);
    return hipGetLastError();
}

template <int MT, int XS, int P, int WAVES>
static hipError_t launch_resident(const DecodeArgs &p, bool acc_out, bool tiled, int grid, hipStream_t stream) {
    return acc_out ? launch_resident_as<MT, XS, P, WAVES, true>(p, tiled, grid, stream)
                   : launch_resident_as<MT, XS, P, WAVES, false>(p, tiled, grid, stream);
}

template <int MT, int T, int WAVES, int U, bool ACC_OUT>
static hipError_t launch_stream_as(const DecodeArgs &p, bool tiled, hipStream_t stream) {
    dim3 grid((p.N + 16 * T - 1) / (16 * T));
    if (tiled)
        hipLaunchKernelGGL((gemm_decode_stream_kernel<MT, T, WAVES, U, ACC_OUT, true>), grid, dim3(WAVES * 64), 0, stream, p);
    else
        hipLaunchKernelGGL((gemm_decode_stream_kernel<MT, T, WAVES, U, ACC_OUT, false>), grid, dim3(WAVES * 64), 0, stream, p);
    return hipGetLastError();
}

template <int MT, int T, int WAVES, int U>
static hipError_t launch_stream(const DecodeArgs &p, bool acc_out, bool tiled, hipStream_t stream) {
    return acc_out ? launch_stream_as<MT, T, WAVES, U, true>(p, tiled, stream)
                   : launch_stream_as<MT, T, WAVES, U, false>(p, tiled, stream);
}

bool decode_resident_supported(int M, int N, int K, const DecodeShape &s) {
    const int mt = (M + 15) / 16;
    const int steps = (((K + 127) / 128) + s.waves - 1) / s.waves;
    if (steps != s.x_steps || (s.waves != 8 && s.waves != 16)) return false;
    // 32-bit buffer offsets (the tiled array rounds N up to 32 and K up to 128)
    const unsigned long long w_bytes = s.tiled ? (unsigned long long)tiled_weight_bytes(N, K)
                                               : (unsigned long long)N * (unsigned long long)(K >> 1);
    if (w_bytes > 0xFFFF0000ull) return false;
    if (s.rows_per_wg < 4 || (s.rows_per_wg & 3) || s.rows_per_wg > kResidentMaxRows) return false;
    if (s.waves == 8) return mt == 1 && s.x_steps >= 1 && s.x_steps <= 5;
    if (mt == 1) return s.x_steps >= 1 && s.x_steps <= 8;
    if (mt == 2) return s.x_steps >= 1 && s.x_steps <= 4;
    return false;
}

hipError_t launch_gemm_decode(const DecodeArgs &p, bool acc_out, const DecodeShape &s, hipStream_t stream) {
    const int mt = (p.M + 15) / 16;
    if (s.resident) {
        if (!decode_resident_supported(p.M, p.N, p.K, s)) return hipErrorInvalidConfiguration;
#define W4A8_RES(MT_, XS_, P_, WV_) \
    if (mt == MT_ && s.x_steps == XS_ && s.waves == WV_) return launch_resident<MT_, XS_, P_, WV_>(p, acc_out, s.tiled, (p.N + s.rows_per_wg - 1) / s.rows_per_wg, stream);
        W4A8_RES(1, 1, 4, 8) W4A8_RES(1, 2, 4, 8) W4A8_RES(1, 3, 2, 8) W4A8_RES(1, 4, 2, 8) W4A8_RES(1, 5, 1, 8)
        W4A8_RES(1, 1, 4, 16) W4A8_RES(1, 2, 4, 16) W4A8_RES(1, 3, 3, 16) W4A8_RES(1, 4, 2, 16)
        W4A8_RES(1, 5, 1, 16) W4A8_RES(1, 6, 1, 16) W4A8_RES(1, 7, 1, 16) W4A8_RES(1, 8, 1, 16)
        W4A8_RES(2, 1, 4, 16) W4A8_RES(2, 2, 2, 16) W4A8_RES(2, 3, 1, 16) W4A8_RES(2, 4, 1, 16)
#undef W4A8_RES
        return hipErrorInvalidConfiguration;
    }
#define W4A8_STR(MT_, T_, WV_, U_) \
    if (mt == MT_ && s.row_tiles == T_ && s.waves == WV_) return launch_stream<MT_, T_, WV_, U_>(p, acc_out, s.tiled, stream);
    W4A8_STR(1, 1, 8, 4) W4A8_STR(1, 2, 8, 4) W4A8_STR(1, 1, 4, 4) W4A8_STR(1, 2, 4, 4)
    W4A8_STR(2, 1, 8, 4) W4A8_STR(2, 2, 8, 2) W4A8_STR(2, 1, 4, 4) W4A8_STR(2, 2, 4, 2)
    W4A8_STR(3, 1, 8, 2) W4A8_STR(3, 2, 8, 2) W4A8_STR(3, 1, 4, 2) W4A8_STR(3, 2, 4, 2)
    W4A8_STR(4, 1, 8, 2) W4A8_STR(4, 1, 4, 2) W4A8_STR(4, 2, 4, 2)
#undef W4A8_STR
    return hipErrorInvalidConfiguration;
}

}  // namespace w4a8
