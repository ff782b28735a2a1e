// Host-visible argument blocks and launchers of the W4A8 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace w4a8 {

struct DecodeArgs {
    const int8_t *xq;    // [M][K]
    const float *s_a;    // [M]     (unused when the raw sums are requested)
    const uint8_t *wp;   // [N][K/2]
    const float *s_w;    // [N]
    void *out;           // fp16 [M][N]
    int *acc_out;        // int32 [M][N]
    int *counters;       // one arrival counter per row block (split-K only)
    int *partials;       // [splits][M][N] sixteen-fold partial sums (split-K only)
    int M, N, K;
    int splits;
};

struct DecodeShape {
    int row_tiles;  // 16-row weight tiles per wave: 1, 2 or 4
    int waves;      // waves per workgroup: 4 or 8
};

hipError_t launch_gemm_decode(const DecodeArgs &p, bool acc_out, const DecodeShape &s, hipStream_t stream);

struct PrefillArgs {
    const int8_t *xq;
    const float *s_a;
    const uint8_t *wp;
    const float *s_w;
    void *out;
    int *acc_out;
    int *counters;   // one arrival counter per output tile (split-K only)
    int *partials;   // [splits][tiles][128*256] sixteen-fold partial sums (split-K only)
    int M, N, K;
    int splits;
    int tiles_m, tiles_n;
};

constexpr int kPrefillBM = 128;
constexpr int kPrefillBN = 256;
constexpr int kPrefillBK = 128;

hipError_t launch_gemm_prefill(const PrefillArgs &p, bool acc_out, hipStream_t stream);

hipError_t launch_quantize_act(const void *x, int8_t *xq, float *s_a, int M, int K, hipStream_t stream);
hipError_t launch_quantize_weights(const void *w, uint8_t *wp, float *s_w, int N, int K, hipStream_t stream);
hipError_t launch_silu_mul(const void *gate_up, void *h, int M, int I, hipStream_t stream);

}  // namespace w4a8
