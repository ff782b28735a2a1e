/*
 * w4a8_tuning.h -- the tuning surface of the MI355X (gfx950) W4A8 library: forced tilings and variants for sweeps
 * and for tests that must cover every kernel at every shape, and probes of what the chip sustains.  Nothing here is
 * needed to use the library (w4a8.h is the interface of the path); the encodings below may change with the kernels.
 * Conventions (pointers, stream, return codes) as in w4a8.h.
 */
#ifndef W4A8_TUNING_H
#define W4A8_TUNING_H

#include "w4a8.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * w4a8_gemm and w4a8_gemm_acc_i32 (see w4a8.h), with the tiling forced instead of chosen from the
 * shape.  For tuning sweeps and for tests that must cover every tiling at
 * every shape.  `tiling` is one of W4A8_TILING_*.  `variant` refines it
 * (0 = library default, W4A8_ERR_ARG if not available for the shape):
 *   DECODE_RESIDENT: workgroups (size of the persistent grid, 0 = library's choice)
 *                    + 100000 * waves (8 or 16, 0 = library's choice: 8 wherever a wave's k steps fit its registers)
 *                    + 10000000 * chunks of weight loads a wave keeps in flight (1, 2, 3, 4 or 8; 0 = library's choice)
 *                    + 100000000 * flags (1 = chunks of 16 channels even where a workgroup's range does not divide
 *                      evenly, 2 = non-temporal weight loads, 8 = default cache policy (neither = library's choice),
 *                      4 = activations read straight from memory instead of staged in LDS, 16 = every wave stages
 *                      its own k steps through a window of LDS: tiled weights only, 17 to 64 tokens, 8 waves (or 16
 *                      for up to 32 tokens and K <= 8192), one or two chunks in flight);
 *   DECODE_STREAM:   row_tiles * 100 + waves, row_tiles in {1, 2}, waves in {4, 8};
 *   PREFILL:         output tile (rows of X x channels): 1 = 128 x 256 as 1 x 4 waves, 2 = 128 x 128,
 *                    3 = 128 x 160, 4 = 128 x 256 as 2 x 2 waves (operands staged through registers);
 *                    5..8 = the shapes of 1, 4, 3, 2 with LDS-direct loads and a four-stage ring;
 *   PREFILL_TILED:   `wp` is the TILED weight array of w4a8_tile_weights; output tile 1 = 256 x 256 as
 *                    2 x 4 waves, 2 = 256 x 256 as 4 x 2 waves, 3 = 128 x 256, 4 = 128 x 160, 5 = 128 x 128,
 *                    6 = 64 x 128, 7 = 64 x 64, 8 = 32 x 128 (the small tiles are for medium M);
 *                    9, 10 = the tiles of 4, 5 run by two sets of waves that split every 128-k stage between
 *                    them and add their integer sums before the epilogue (same bits; never the library's choice);
 *                    11 = 256 x 192 as 4 x 2 waves (the library pairs it with 1 where whole rounds of 256 x 256 tiles
 *                    leave columns over); 12 = 128 x 256 as 2 x 4 waves with a three-stage ring, one workgroup per
 *                    compute unit (the library's choice where such tiles number no more than the compute units).
 * Exactly one of out_fp16 / acc_i32 must be non-NULL (s_a and s_w may be NULL
 * when acc_i32 is requested).
 */
#define W4A8_TILING_AUTO 0
#define W4A8_TILING_DECODE_RESIDENT 1 /* persistent weight-streaming kernel, activations kept in registers:
                                         M <= 16 with K <= 16384, or M <= 32 with K <= 8192 (flag 16: M <= 32
                                         with K <= 8192, M <= 64 with K <= 5120); at most 512 channels per
                                         workgroup                                                         */
#define W4A8_TILING_DECODE_STREAM 2   /* general weight-streaming kernel, M <= 64                         */
#define W4A8_TILING_PREFILL 3         /* LDS-staged output tiles on 32x32x32 int8 MFMA, for large M       */
#define W4A8_TILING_PREFILL_TILED 4   /* the same over the tiled weight layout (any M; meant for large M)  */
#define W4A8_TILING_DECODE_RESIDENT_TILED 5 /* tilings 1 and 2 reading the TILED weight array (`wp` = wt);        */
#define W4A8_TILING_DECODE_STREAM_TILED 6   /* same limits and variants as 1 and 2                                 */
#define W4A8_TILING_AUTO_TILED 7      /* library's choice over the TILED array: 5 or 6 up to M = 16, 5 with flag 16
                                         up to M = 64 where K allows, 4 otherwise                            */
int w4a8_gemm_tuned(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w,
                    void *out_fp16, int32_t *acc_i32, int M, int N, int K,
                    int tiling, int variant,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * Two probes of what the chip sustains, for a benchmark to set its figures against (they are no part of the path and
 * compute nothing of use):
 * w4a8_probe_stream_read: a read-only streaming reduction over buf (device, `bytes` long, 16-byte aligned) by 8
 *   workgroups per compute unit; bytes / run time is the read rate a plain kernel reaches on this buffer.
 * w4a8_probe_mfma_int8: a register-resident loop of `iters` x 8 int8 32x32x32 MFMAs per wave, 8 waves per compute
 *   unit; operations = compute units * 8 waves * iters * 8 * 65536.  pattern 0 = constant operands, 1 = random int8
 *   activations and random multiples of 16 as weights (what the W4A8 kernel feeds the matrix cores): the rate depends
 *   on the operand values through the chip's power management.
 * sink: 4 bytes of device memory that are practically never written.
 */
int w4a8_probe_stream_read(const void *buf, size_t bytes, void *sink, void *stream);

/*
 * w4a8_probe_stream_read with the access pattern as arguments, to find the read rate the chip sustains and the
 * pattern that reaches it (bytes below 4 GiB):
 *   pattern : 0 = all workgroups sweep the buffer together (grid-wide stride), 1 = every workgroup reads one contiguous
 *             run; 2, 3 = the same with bounds-checked buffer loads (the instruction of the weight-streaming kernels)
 *             instead of global loads; 4, 5 = 2, 3 with the non-temporal cache policy;
 *   loads   : 16-byte loads a thread issues before it uses the first, 4, 8 or 16;
 *   workgroups_per_cu : workgroups of 256 threads per compute unit, 1 .. 64.
 */
int w4a8_probe_read_pattern(const void *buf, size_t bytes, void *sink, int pattern, int loads, int workgroups_per_cu,
                            void *stream);
/*
 * What one compute unit can pull in when part of what it reads sits in L2 and part comes from memory -- the situation of
 * a GEMM at a hundred or so tokens, whose workgroups re-read the activations from cache while they stream the weights:
 * one workgroup of 4 waves per compute unit, 16 loads of 16 bytes per thread in flight; `cold` (cold_bytes, read once,
 * every workgroup its own contiguous run of cold_bytes / compute units, rounded down to whole iterations) and `hot`
 * (hot_bytes, shared by all workgroups, read over and over).
 *   mode 0: every wave alternates cold and hot loads, as many bytes of each; 1: two waves read cold, two hot, same
 *   bytes; 2: cold only, twice the cold bytes (the same total); 3: hot only, the same total.
 * cold_bytes at least 32 KiB (64 KiB in mode 2) per compute unit, hot_bytes 16 .. 4 GiB, both 16-byte aligned.
 */
int w4a8_probe_mixed_read(const void *cold, size_t cold_bytes, const void *hot, size_t hot_bytes, void *sink, int mode,
                          void *stream);
int w4a8_probe_mfma_int8(void *sink, int iters, int pattern, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* W4A8_TUNING_H */
