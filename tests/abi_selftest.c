/*
 * Sanitizer driver for the host side of the C ABI (no GPU needed, none used).
 *
 * Linked against a build of the library whose HOST code is instrumented with AddressSanitizer and
 * UndefinedBehaviorSanitizer (python -m paper_2311_09550_amd.build --host-sanitize), it drives what the host side does
 * with caller memory and caller numbers: the one function that reads and writes host arrays
 * (w4a8_pack_weights_host, on heap blocks of exactly the documented size), the size and planning functions over a grid
 * of shapes including the extremes of the contract (integer overflow in a size computation would trip UBSan), and
 * the argument checks of every launching entry point with pointers that must never be dereferenced.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/w4a8.h"
#include "../include/w4a8_tuning.h"

static int failures;
#define EXPECT(call, want)                                                                              \
    do {                                                                                                \
        const long long got_ = (long long)(call);                                                       \
        if (got_ != (long long)(want)) {                                                                \
            ++failures;                                                                                 \
            fprintf(stderr, "abi selftest: %s = %lld, expected %lld (line %d)\n", #call, got_, (long long)(want), __LINE__); \
        }                                                                                               \
    } while (0)

int main(void)
{
    void *p = (void *)0x1000, *odd = (void *)0x1008;
    const size_t big = (size_t)1 << 40;

    /* host packing on exact-size blocks */
    {
        const int N = 37, K = 130;
        int8_t *wq = (int8_t *)malloc((size_t)N * K);
        uint8_t *wp = (uint8_t *)malloc((size_t)N * (K / 2));
        for (int i = 0; i < N * K; ++i) wq[i] = (int8_t)(i * 7 % 16 - 8);
        EXPECT(w4a8_pack_weights_host(wq, wp, N, K), W4A8_OK);
        for (int n = 0; n < N; ++n)
            for (int j = 0; j < K / 2; ++j) {
                const int lo = wq[n * K + 2 * j], hi = wq[n * K + 2 * j + 1];
                if (wp[n * (K / 2) + j] != (uint8_t)((lo & 15) | ((hi & 15) << 4))) { ++failures; n = N; break; }
            }
        wq[5] = 8;
        EXPECT(w4a8_pack_weights_host(wq, wp, N, K), W4A8_ERR_VALUE);
        EXPECT(w4a8_pack_weights_host(wq, wp, N, K + 1), W4A8_ERR_SHAPE);
        EXPECT(w4a8_pack_weights_host(NULL, wp, N, K), W4A8_ERR_NULL);
        free(wq);
        free(wp);
    }

    /* sizes and plans over the contract's range: pure functions of the shape */
    {
        static const int Ms[] = {1, 4, 5, 16, 17, 32, 33, 64, 65, 128, 512, 1024, 4096, 1 << 20};
        static const int Ns[] = {1, 16, 33, 5120, 57344, 1 << 20};
        static const int Ks[] = {32, 160, 4096, 5120, 13824, 28672, 65536};
        for (size_t a = 0; a < sizeof Ms / sizeof *Ms; ++a)
            for (size_t b = 0; b < sizeof Ns / sizeof *Ns; ++b)
                for (size_t c = 0; c < sizeof Ks / sizeof *Ks; ++c) {
                    const int M = Ms[a], N = Ns[b], K = Ks[c];
                    const size_t blocks = (size_t)((N + 31) / 32) * (size_t)((K + 127) / 128);
                    EXPECT(w4a8_tiled_weight_bytes(N, K), blocks * 2048);
                    EXPECT(w8a8_tiled_weight_bytes(N, K), blocks * 4096);
                    EXPECT(w4a8_gemm_workspace_bytes(M, N, K), 0);
                    const size_t ws = w4a8_gemm_tiled_workspace_bytes(M, N, K);
                    const size_t slab = (size_t)M * (size_t)N * 4;
                    if (ws % slab != 0 || ws / slab == 1 || ws / slab > 8) {
                        ++failures;
                        fprintf(stderr, "abi selftest: workspace of (%d, %d, %d) is %zu bytes\n", M, N, K, ws);
                    }
                }
        EXPECT(w4a8_tiled_weight_bytes(16, 48), 0);
        EXPECT(w4a8_gemm_tiled_workspace_bytes(0, 16, 32), 0);
    }

    /* argument checks happen before anything is launched or dereferenced */
    EXPECT(w4a8_gemm(NULL, p, p, p, p, 1, 16, 32, p, big, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_gemm(p, p, p, p, p, 0, 16, 32, p, big, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_gemm(p, p, p, p, p, 1, 16, 65536 + 32, p, big, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_gemm(odd, p, p, p, p, 1, 16, 32, p, big, NULL), W4A8_ERR_ALIGN);
    EXPECT(w4a8_gemm_acc_i32(p, p, NULL, 1, 16, 32, p, big, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_gemm_tuned(p, p, p, p, p, NULL, 1, 16, 1024, 10, 0, p, big, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_gemm_tuned(p, p, p, p, p, NULL, 65, 16, 1024, 1, 0, p, big, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_gemm_tuned(p, p, p, p, p, NULL, 1, 16, 1024, 4, 13, p, big, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_gemm_tuned(p, p, p, p, p, NULL, 1, 16, 1024, 1, 2147483647, p, big, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_quantize_act(NULL, p, p, 1, 32, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_quantize_act(p, p, p, 1, 40, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_quantize_act_strided(p, 24, p, p, 1, 32, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_quantize_weights(p, p, NULL, 4, 32, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_quantize_weights_clipped(odd, NULL, NULL, p, p, 4, 32, NULL), W4A8_ERR_ALIGN);
    EXPECT(w4a8_silu_mul(p, p, 1, 12, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_silu_mul_quantize(p, NULL, p, 1, 32, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_tile_weights(p, odd, 32, 128, NULL), W4A8_ERR_ALIGN);
    EXPECT(w4a8_gemm_tiled(p, p, p, p, NULL, 1, 16, 32, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_gemm_tiled_splitk(p, p, p, p, p, 1, 16, 256, 0, 65, p, big, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_gemm_tiled_splitk(p, p, p, p, p, 1, 16, 256, 0, 2, p, 127, NULL), W4A8_ERR_WORKSPACE);
    EXPECT(w4a8_gemm_tiled_splitk(p, p, p, p, p, 64, 512, 13824, 0, 0, NULL, 0, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_gemm_tiled_splitk_static(p, p, p, p, p, 512, 4096, 1024, 6, 8, NULL), W4A8_ERR_WORKSPACE);
    EXPECT(w4a8_gemm_tiled_swiglu(p, p, p, p, p, 4, 40, 64, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_gemm_tiled_swiglu(p, p, p, p, odd, 4, 64, 64, NULL), W4A8_ERR_ALIGN);
    EXPECT(w4a8_linear_tiled_fp16(p, 1000, p, p, p, NULL, 1, 16, 1024, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_linear_tiled_fp16(p, 1024, p, p, p, NULL, 17, 16, 1024, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_linear_tiled_norm_fp16(p, 1024, NULL, 0, NULL, 1e-5f, NULL, NULL, p, p, p, NULL, 1, 64, 1024, 0, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_linear_tiled_norm_fp16(p, 1024, NULL, 0, p, 1e-5f, NULL, NULL, p, p, p, NULL, 5, 64, 1024, 0, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_linear_tiled_norm_fp16(p, 1024, NULL, 0, p, 1e-5f, NULL, NULL, p, p, p, NULL, 1, 96, 1024, 1, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_add_rmsnorm_quantize(p, NULL, NULL, 1e-5f, NULL, NULL, p, p, 1, 64, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_add_rmsnorm_quantize(p, NULL, p, 1e-5f, NULL, NULL, p, p, 1, 40, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_add_rmsnorm_quantize(p, NULL, p, -1.0f, NULL, NULL, p, p, 1, 64, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_linear_tiled_swiglu_fp16(p, 1024, p, p, NULL, NULL, 1, 32, 1024, NULL), W4A8_ERR_NULL);
    EXPECT(w4a8_linear_tiled_swiglu_fp16(p, 1024, p, p, p, NULL, 1, 40, 1024, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_linear_tiled_swiglu_fp16(p, 1024, p, p, p, NULL, 5, 32, 1024, NULL), W4A8_ERR_ARG);
    EXPECT(w4a8_gemm_fine_grained(p, p, p, p, 12, p, 1, 16, 128, 0, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_gemm_tiled_unsigned(p, p, p, p, p, NULL, 1, 16, 32, 9, NULL), W4A8_ERR_ARG);
    EXPECT(w8a8_gemm_tiled(p, p, p, p, p, NULL, 1, 16, 48, 0, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_probe_stream_read(p, 8, p, NULL), W4A8_ERR_SHAPE);
    EXPECT(w4a8_probe_mfma_int8(p, 0, 0, NULL), W4A8_ERR_ARG);
    for (int code = 1; code >= -9; --code)
        if (w4a8_strerror(code) == NULL || w4a8_strerror(code)[0] == 0) ++failures;
    if (strcmp(w4a8_last_hip_error(), "hipSuccess") != 0) {
        ++failures;
        fprintf(stderr, "abi selftest: a validation error reached HIP: %s\n", w4a8_last_hip_error());
    }
    if (w4a8_version() < 100) ++failures;

    if (failures) {
        fprintf(stderr, "abi selftest: %d check(s) failed\n", failures);
        return 1;
    }
    puts("abi selftest ok");
    return 0;
}
