// C ABI of the W4A8 library: argument validation, tiling choice, launches.
// Nothing here touches the data; every step of the path runs in the kernels.
#include "../../include/w4a8.h"

#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace {

using namespace w4a8;

constexpr int kMaxSplits = 8;
constexpr int kDecodeMaxM = 64;
// Arrival counters live in a region of fixed size at the start of the workspace, so that the partial sums
// of one shape can never land on the counters of another shape sharing the same buffer.
constexpr size_t kCounterRegion = 65536;
constexpr int kMaxCounters = (int)(kCounterRegion / sizeof(int));

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline int check_gemm_shape(int M, int N, int K) {
    if (M < 1 || N < 1 || K < 32 || (K % 32) != 0 || K > W4A8_MAX_K) return W4A8_ERR_SHAPE;
    return W4A8_OK;
}

struct Plan {
    int tiling;
    int splits;
    DecodeShape decode;
};

// Tiling choice.  Small M streams the weights once (HBM bound): pick the row
// tile count and K split so that the launch has a few workgroups per compute
// unit, each with enough bytes to keep loads in flight.  Large M goes to the
// LDS-staged tiling (matrix-core bound).
Plan choose_plan(int M, int N, int K, int tiling, int split_k) {
    Plan pl{};
    pl.tiling = tiling;
    if (tiling == W4A8_TILING_AUTO) pl.tiling = M <= kDecodeMaxM ? W4A8_TILING_DECODE : W4A8_TILING_PREFILL;
    pl.splits = 1;
    if (pl.tiling == W4A8_TILING_DECODE) {
        const int mt = (M + 15) / 16;
        pl.decode.row_tiles = M <= 8 ? 1 : 2;
        pl.decode.waves = (mt >= 4 && pl.decode.row_tiles == 2) ? 4 : 8;
        const int row_blocks = (N + 16 * pl.decode.row_tiles - 1) / (16 * pl.decode.row_tiles);
        const int ks_total = (K + 127) / 128;
        int s = 1;
        if (split_k > 0) {
            s = split_k;
        } else {
            const int target = 768;  // about three workgroups per compute unit
            s = (target + row_blocks - 1) / row_blocks;
            // keep at least two k steps per wave in a slice
            const int max_by_k = ks_total / (2 * pl.decode.waves);
            if (s > max_by_k) s = max_by_k;
        }
        if (s > kMaxSplits) s = kMaxSplits;
        if (s > ks_total) s = ks_total;
        if (row_blocks > kMaxCounters) s = 1;  // more row blocks than counters: such a launch needs no split
        if (s < 1) s = 1;
        pl.splits = s;
    }
    return pl;
}

int run_gemm(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w, void *out_fp16, int32_t *acc_i32,
             int M, int N, int K, int tiling, int split_k, void *workspace, size_t workspace_bytes, void *stream) {
    const bool want_acc = acc_i32 != nullptr;
    if ((out_fp16 != nullptr) == want_acc) return W4A8_ERR_NULL;  // exactly one output
    if (!xq || !wp) return W4A8_ERR_NULL;
    if (!want_acc && (!s_a || !s_w)) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, N, K)) return e;
    if (tiling < W4A8_TILING_AUTO || tiling > W4A8_TILING_PREFILL) return W4A8_ERR_ARG;
    if (split_k < 0 || split_k > kMaxSplits) return W4A8_ERR_ARG;
    if (tiling == W4A8_TILING_DECODE && M > kDecodeMaxM) return W4A8_ERR_ARG;
    if (misaligned(xq) || misaligned(wp) || misaligned(out_fp16) || misaligned(acc_i32) || misaligned(workspace) ||
        (s_w && misaligned(s_w)))
        return W4A8_ERR_ALIGN;

    const Plan pl = choose_plan(M, N, K, tiling, split_k);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t err;
    if (pl.tiling == W4A8_TILING_DECODE) {
        DecodeArgs a{};
        a.xq = xq; a.s_a = s_a; a.wp = wp; a.s_w = s_w;
        a.out = out_fp16; a.acc_out = acc_i32;
        a.M = M; a.N = N; a.K = K; a.splits = pl.splits;
        if (pl.splits > 1) {
            const size_t need = kCounterRegion + (size_t)pl.splits * M * N * sizeof(int);
            if (!workspace || workspace_bytes < need) return W4A8_ERR_WORKSPACE;
            a.counters = static_cast<int *>(workspace);
            a.partials = reinterpret_cast<int *>(static_cast<char *>(workspace) + kCounterRegion);
        }
        err = launch_gemm_decode(a, want_acc, pl.decode, st);
    } else {
        PrefillArgs a{};
        a.xq = xq; a.s_a = s_a; a.wp = wp; a.s_w = s_w;
        a.out = out_fp16; a.acc_out = acc_i32;
        a.M = M; a.N = N; a.K = K; a.splits = 1;
        a.tiles_m = (M + kPrefillBM - 1) / kPrefillBM;
        a.tiles_n = (N + kPrefillBN - 1) / kPrefillBN;
        err = launch_gemm_prefill(a, want_acc, st);
    }
    return err == hipSuccess ? W4A8_OK : W4A8_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int w4a8_version(void) { return 100; }

const char *w4a8_strerror(int err) {
    switch (err) {
        case W4A8_OK: return "ok";
        case W4A8_ERR_NULL: return "a required pointer is NULL (or both / neither output given)";
        case W4A8_ERR_SHAPE: return "shape outside the contract: M,N >= 1, 32 <= K <= 65536, K % 32 == 0";
        case W4A8_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case W4A8_ERR_WORKSPACE: return "workspace missing or too small (see w4a8_gemm_workspace_bytes)";
        case W4A8_ERR_LAUNCH: return "HIP rejected the kernel launch";
        case W4A8_ERR_VALUE: return "weight code outside [-8, 7]";
        case W4A8_ERR_ARG: return "tiling id or split count out of range for this shape";
        default: return "unknown w4a8 error code";
    }
}

int w4a8_quantize_act(const void *x_fp16, int8_t *xq, float *s_a, int M, int K, void *stream) {
    if (!x_fp16 || !xq || !s_a) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(M, 1, K)) return e;
    if (misaligned(x_fp16) || misaligned(xq)) return W4A8_ERR_ALIGN;
    return launch_quantize_act(x_fp16, xq, s_a, M, K, static_cast<hipStream_t>(stream)) == hipSuccess ? W4A8_OK
                                                                                                         : W4A8_ERR_LAUNCH;
}

size_t w4a8_gemm_workspace_bytes(int M, int N, int K) {
    if (check_gemm_shape(M, N, K) != W4A8_OK) return 0;
    if (M > kDecodeMaxM) return 0;
    return kCounterRegion + (size_t)kMaxSplits * M * N * sizeof(int);
}

int w4a8_gemm(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w, void *out_fp16, int M, int N, int K,
              void *workspace, size_t workspace_bytes, void *stream) {
    if (!out_fp16) return W4A8_ERR_NULL;
    return run_gemm(xq, s_a, wp, s_w, out_fp16, nullptr, M, N, K, W4A8_TILING_AUTO, 0, workspace, workspace_bytes, stream);
}

int w4a8_gemm_acc_i32(const int8_t *xq, const uint8_t *wp, int32_t *acc, int M, int N, int K, void *workspace,
                      size_t workspace_bytes, void *stream) {
    if (!acc) return W4A8_ERR_NULL;
    return run_gemm(xq, nullptr, wp, nullptr, nullptr, acc, M, N, K, W4A8_TILING_AUTO, 0, workspace, workspace_bytes, stream);
}

int w4a8_gemm_tuned(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w, void *out_fp16,
                    int32_t *acc_i32, int M, int N, int K, int tiling, int split_k, void *workspace, size_t workspace_bytes,
                    void *stream) {
    return run_gemm(xq, s_a, wp, s_w, out_fp16, acc_i32, M, N, K, tiling, split_k, workspace, workspace_bytes, stream);
}

int w4a8_quantize_weights(const void *w_fp16, uint8_t *wp, float *s_w, int N, int K, void *stream) {
    if (!w_fp16 || !wp || !s_w) return W4A8_ERR_NULL;
    if (int e = check_gemm_shape(1, N, K)) return e;
    if (misaligned(w_fp16) || misaligned(wp)) return W4A8_ERR_ALIGN;
    return launch_quantize_weights(w_fp16, wp, s_w, N, K, static_cast<hipStream_t>(stream)) == hipSuccess ? W4A8_OK
                                                                                                             : W4A8_ERR_LAUNCH;
}

int w4a8_silu_mul(const void *gate_up_fp16, void *h_fp16, int M, int I, void *stream) {
    if (!gate_up_fp16 || !h_fp16) return W4A8_ERR_NULL;
    if (M < 1 || I < 8 || (I % 8) != 0 || M > 65535) return W4A8_ERR_SHAPE;
    if (misaligned(gate_up_fp16) || misaligned(h_fp16)) return W4A8_ERR_ALIGN;
    return launch_silu_mul(gate_up_fp16, h_fp16, M, I, static_cast<hipStream_t>(stream)) == hipSuccess ? W4A8_OK
                                                                                                          : W4A8_ERR_LAUNCH;
}

int w4a8_pack_weights_host(const int8_t *wq_host, uint8_t *wp_host, int N, int K) {
    if (!wq_host || !wp_host) return W4A8_ERR_NULL;
    if (N < 1 || K < 2 || (K & 1)) return W4A8_ERR_SHAPE;
    const size_t total = (size_t)N * (size_t)(K / 2);
    for (size_t i = 0; i < total; ++i) {
        const int even = wq_host[2 * i], odd = wq_host[2 * i + 1];
        if (even < -8 || even > 7 || odd < -8 || odd > 7) return W4A8_ERR_VALUE;
    }
    for (size_t i = 0; i < total; ++i) {
        const unsigned even = (unsigned)wq_host[2 * i] & 15u, odd = (unsigned)wq_host[2 * i + 1] & 15u;
        wp_host[i] = (uint8_t)(even | (odd << 4));
    }
    return W4A8_OK;
}

}  // extern "C"
