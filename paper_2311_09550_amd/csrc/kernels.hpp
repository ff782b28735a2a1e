// Host-visible argument blocks and launchers of the W4A8 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

namespace w4a8 {

constexpr int kMaxDevices = 64;  // device ordinals the per-device tables of the host code cover

// A kernel that uses more than 64 KB of LDS per workgroup has to ask the runtime for it, once per device.  One
// set of flags per kernel (the kernel is the template argument); the flags are atomic and the request itself is
// serialised, so first launches from several threads are safe.  w4a8_init makes all requests up front, so that no
// launch, in particular none under stream capture, has to.
template <auto Kernel>
inline hipError_t allow_lds(int bytes) {
    static std::atomic<bool> raised[kMaxDevices];
    static std::mutex raise_lock;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!raised[dev].load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> hold(raise_lock);
        if (!raised[dev].load(std::memory_order_relaxed)) {
            const hipError_t e = hipFuncSetAttribute((const void *)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
            if (e != hipSuccess) return e;
            raised[dev].store(true, std::memory_order_release);
        }
    }
    return hipSuccess;
}

struct DecodeArgs {
    const uint16_t *x16; // fused-quantiser form only: fp16 activations, rows ldx elements apart (xq, s_a unused)
    long long ldx;
    float *s_a_out;      // fused-quantiser form only: where the per-token scales are also written, or NULL
    // fused-quantiser form with the norm in front (DecodeShape::norm): y = rmsnorm(res + x) * gamma is what gets quantised
    const uint16_t *res16;  // residual rows, ldres elements apart, or NULL (then r = x)
    long long ldres;
    const uint16_t *gamma;  // [K] fp16
    float eps;
    uint16_t *r_out;        // [M][K] dense: res + x, written by the first workgroup, or NULL
    uint16_t *y_out;        // [M][K] dense: the normalised rows, written by the first workgroup, or NULL
    int res_lds_offset;     // where the residual rows are staged in LDS (rows x16_lds_pitch apart)
    const int8_t *xq;    // [M][K]
    const float *s_a;    // [M]     (unused when the raw sums are requested)
    const uint8_t *wp;   // [N][K/2]
    const float *s_w;    // [N]
    void *out;           // fp16 [M][N]
    int *acc_out;        // int32 [M][N]
    int M, N, K;
    int rows_per_wg;     // persistent kernels: output channels per workgroup (multiple of 4)
    int chunk_rows;      // persistent kernel: channels per chunk, 4, 8, 12 or 16
    int x_lds_pitch;     // persistent kernel: > 0 = the activations are staged in LDS, rows this many bytes apart
    int x_lds_offset;    //   ... starting at this byte of the kernel's dynamic LDS
    int x16_lds_pitch;   // fused-quantiser form: the fp16 rows are staged too, rows this many bytes apart
    int x16_lds_offset;  //   ... starting here
    int ks_per_slice;    // persistent kernel: k steps (of 128) per K slice; <= 0 = all of K in one slice.  With more than
                         // one slice acc_out holds one [M][N] slab of raw sums per slice
};

constexpr int kResidentMaxRows = 512;  // channels per workgroup of the persistent kernel (their scales are staged in LDS,
                                       // one load per thread of the smaller workgroup shape)


struct DecodeShape {
    bool resident;  // persistent kernel with register-resident activations, else the general streaming kernel
    int prefetch;   // resident: chunks of weight loads a wave keeps in flight (1, 2, 3, 4 or 8)
    int chunk_rows; // resident: channels per chunk (4, 8, 12 or 16)
    int aux;        // resident: cache-policy bits of the weight loads (0 or 2 = non-temporal)
    bool x_direct;  // resident: never stage the activations in LDS (they are staged when they fit, otherwise)
    bool fused_quant;  // resident: the kernel quantises fp16 activations itself (M <= 4, tiled weights, rows must fit LDS)
    int waves;      // waves per workgroup: resident 8 or 16, streaming 4 or 8
    int x_steps;    // resident: k steps per wave = ceil(ceil(K/128) / waves)
    int rows_per_wg;  // resident: output channels per persistent workgroup, a multiple of 4, at most kResidentMaxRows
    int row_tiles;  // streaming: 16-row weight tiles per wave, 1 or 2
    bool tiled;     // DecodeArgs::wp is the tiled weight array (2 KB blocks) instead of the row-major one
    bool x_window;  // resident: every wave stages its own k steps through a window of LDS (tiled weights; the only
                    // form beyond 32 tokens)
    int k_slices;   // resident: workgroups along K (0 or 1 = none); more than one only with raw sums, one slab each
    bool norm;      // resident, with fused_quant: residual addition + RMSNorm in front of the quantiser (K <= 8192, 8 waves)
    bool swiglu;    // resident: interleaved gate / up channels, the epilogue stores h = silu(gate) * up (tiled weights,
                    // fp16 output, with the fused quantiser or with per-wave staging)
};

// Token counts the persistent kernel serves: 32 with the activations staged whole or read directly, 64 with per-wave
// staging.
constexpr int kResidentMaxM = 64;

bool decode_resident_supported(int M, int N, int K, const DecodeShape &s);
// Per-device preparations (LDS allowance) of every instantiation of the persistent kernel, for the current device.
hipError_t prepare_decode_kernels();
hipError_t launch_gemm_decode(const DecodeArgs &p, bool acc_out, const DecodeShape &s, hipStream_t stream);
// The instantiations with per-wave staging (mt = column tiles of 16 tokens, 2 to 4): whether one exists for the shape,
// and its launch (prepare_only: the per-device preparations of all of them).
bool decode_wide_supported(int mt, const DecodeShape &s);
hipError_t launch_gemm_decode_wide(const DecodeArgs &p, bool acc_out, const DecodeShape &s, int mt, bool prepare_only,
                                   hipStream_t stream);
// The instantiations with the norm in front of the fused quantiser (DecodeShape::norm, with or without swiglu): the same pair.
bool decode_norm_supported(int mt, const DecodeShape &s);
hipError_t launch_gemm_decode_norm(const DecodeArgs &p, const DecodeShape &s, bool prepare_only, hipStream_t stream);
// The instantiations whose epilogue applies SiLU * up (DecodeShape::swiglu): the same pair.
bool decode_swiglu_supported(int mt, const DecodeShape &s);
hipError_t launch_gemm_decode_swiglu(const DecodeArgs &p, const DecodeShape &s, int mt, bool prepare_only, hipStream_t stream);

struct PrefillArgs {
    const int8_t *xq;
    const float *s_a;
    const uint8_t *wp;
    const float *s_w;
    void *out;
    int *acc_out;
    int M, N, K;       // extent of this launch (a slice of the whole problem when that exceeds 32-bit byte offsets)
    int ldc;           // row stride of out / acc_out in elements (the full N)
    int splits;            // tiled kernel, raw sums only: > 1 = K is split over this many workgroups per tile, each
    int stages_per_split;  // taking this many 128-k stages and writing its own M x ldc slab of acc_out
    int ldg;           // fine-grained variant only: s_w then holds group scales [K / 128][ldg], ldg >= N, ldg % 4 == 0
    int tiles_m, tiles_n;
    bool prepare_only;  // host side only: make the per-device preparations of the chosen kernel and launch nothing
};

constexpr int kPrefillBK = 128;
// output tile shapes (rows of X x output channels) of the LDS-staged kernel
constexpr int kPrefillTile128x256 = 1;
constexpr int kPrefillTile128x128 = 2;
constexpr int kPrefillTile128x160 = 3;
constexpr int kPrefillTile128x256Square = 4;  // 128 x 256 with 2 x 2 waves of 64 x 128 (1 uses 1 x 4 waves of 128 x 64)

// the same tile shapes with operands brought into LDS by LDS-direct buffer loads (four-stage ring)
constexpr int kPrefillDma128x256 = 5;
constexpr int kPrefillDma128x256Square = 6;
constexpr int kPrefillDma128x160 = 7;
constexpr int kPrefillDma128x128 = 8;
constexpr int kPrefillTileMax = 8;

// Tiled weight layout (see gemm_prefill_tiled.hip): 2 KB blocks of 32 output channels x 128 k
constexpr int kTiledBlockK = 128;
constexpr int kTiledBlockBytes = 2048;
// output tiles of the kernel that reads the tiled layout (PrefillArgs::wp then points to the tiled array)
constexpr int kTiled256x256 = 1;        // 8 waves of 128 x 64, one workgroup per compute unit
constexpr int kTiled256x256Square = 2;  // 8 waves of 64 x 128
constexpr int kTiled128x256 = 3;        // 4 waves of 128 x 64, two-stage ring, two workgroups per compute unit
constexpr int kTiled128x160 = 4;        // 4 waves of 32 x 160
constexpr int kTiled128x128 = 5;        // 4 waves of 64 x 64
constexpr int kTiled64x128 = 6;         // 4 waves of 32 x 64: medium M, where 128-row tiles leave most of the chip idle
constexpr int kTiled64x64 = 7;          // 4 waves of 32 x 32
constexpr int kTiled32x128 = 8;         // 4 waves of 32 x 32 side by side
constexpr int kTiled128x160K2 = 9;      // 128 x 160 with two wave sets of 4 splitting each stage's k (int4 weights only)
constexpr int kTiled128x128K2 = 10;     // 128 x 128 likewise
constexpr int kTiled256x192 = 11;       // 8 waves of 64 x 96 (int4 weights only): the narrower partner of 1 for the columns
                                        // that whole rounds of 256 x 256 tiles leave over
constexpr int kTiledTileMax = 8;        // tiles every weight format has
constexpr int kTiled128x256W8 = 12;     // 128 x 256 as 8 waves of 64 x 64, three-stage ring, one workgroup per compute unit
                                        // (int4 weights only): where 128 x 256 tiles number no more than the compute units
constexpr int kTiledTileMax4 = 12;      // tiles of the signed int4 format

// wbits = 4: packed int4 codes (blocks of 2 KB); wbits = 8: int8 codes of the W8A8 comparison variant (blocks of 4 KB);
// wbits = kWeightsUnsigned4: the 2 KB blocks with unsigned nibbles u = w + 8 (the paper's vanilla storage, GEMM only)
constexpr int kWeightsUnsigned4 = 104;
// wbits = kWeightsFineGrained4: signed int4 blocks with one scale per group of 128 k and channel (the fine-grained
// recipe of Eq. (5)); its accumulators take twice the registers, hence its own, smaller set of tiles
constexpr int kWeightsFineGrained4 = 204;
constexpr int kFine128x256 = 1;  // 8 waves of 64 x 64
constexpr int kFine256x128 = 2;  // 8 waves of 64 x 64, four down and two across
constexpr int kFine128x128 = 3;  // 4 waves of 64 x 64
constexpr int kFine64x128 = 4;   // 4 waves of 32 x 64
constexpr int kFine64x64 = 5;    // 4 waves of 32 x 32
constexpr int kFine32x128 = 6;   // 4 waves of 32 x 32 side by side
constexpr int kFineTileMax = 6;
size_t tiled_weight_bytes(int N, int K, int wbits = 4);
hipError_t launch_tile_weights(const uint8_t *wp, uint8_t *wt, int N, int K, hipStream_t stream);
hipError_t launch_tile_weights8(const int8_t *w8, uint8_t *wt, int N, int K, hipStream_t stream);
hipError_t launch_gemm_prefill_tiled(const PrefillArgs &p, bool acc_out, int tile, hipStream_t stream, int wbits = 4);
// The same over gate and up channels interleaved, storing h = fp16(silu(gate) * up) (p.out = h, p.ldc = its pitch);
// tiles 256 x 256, 256 x 192, 128 x 256 (both forms) and 128 x 128.
hipError_t launch_gemm_prefill_tiled_swiglu(const PrefillArgs &p, int tile, hipStream_t stream);
// Per-device preparations (LDS allowance) of every instantiation of the tiled kernel, for the current device.
hipError_t prepare_tiled_kernels();
// fp16 output from `splits` slabs [M][N] of raw int32 sums (what the tiled kernel writes when PrefillArgs::splits > 1)
hipError_t launch_splitk_epilogue(const int *part, int splits, const float *s_a, const float *s_w, void *out, int M, int N,
                                  hipStream_t stream);

hipError_t launch_gemm_prefill(const PrefillArgs &p, bool acc_out, int tile, hipStream_t stream);
hipError_t launch_prefill_dma_slice(const PrefillArgs &p, bool acc_out, int tile, hipStream_t stream);

hipError_t launch_quantize_act(const void *x, long long ldx, int8_t *xq, float *s_a, int M, int K, hipStream_t stream);
hipError_t launch_quantize_weights(const void *w, uint8_t *wp, float *s_w, int N, int K, hipStream_t stream);
hipError_t launch_quantize_weights_clip(const void *w, const float *gamma, const float *beta, uint8_t *wp, float *s_w, int N,
                                        int K, hipStream_t stream);
hipError_t launch_silu_mul(const void *gate_up, void *h, int M, int I, hipStream_t stream);
hipError_t launch_probe_stream_read(const void *src, size_t bytes, unsigned *sink, int workgroups, hipStream_t stream);
hipError_t launch_probe_mixed_read(const void *cold, unsigned cold_chunks_per_wg, const void *hot, unsigned hot_chunks,
                                   unsigned *sink, int mode, int workgroups, hipStream_t stream);
hipError_t launch_probe_read_pattern(const void *src, size_t bytes, unsigned *sink, int pattern, int loads, int workgroups,
                                     hipStream_t stream);
hipError_t launch_probe_mfma_i8(int *sink, int workgroups, int iters, int pattern, hipStream_t stream);
hipError_t launch_silu_mul_quantize(const void *gate_up, int8_t *xq, float *s_a, int M, int I, hipStream_t stream);
hipError_t launch_add_rmsnorm_quantize(const void *x, const void *res, const void *gamma, float eps, void *r_out, void *y_out,
                                       int8_t *xq, float *s_a, int M, int K, hipStream_t stream);

}  // namespace w4a8
