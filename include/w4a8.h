/*
 * w4a8.h -- C ABI of the MI355X (gfx950) W4A8 linear-layer library.
 *
 * The library implements the inference hot path of a W4A8 quantised linear
 * layer as described in arXiv 2311.09550 ("A Speed Odyssey for Deployable
 * Quantization of LLMs"): activations quantised per token to signed 8 bit,
 * weights quantised per output channel to signed 4 bit with no group scales,
 * integer GEMM with int32 accumulation, one dequantisation after the GEMM
 * (Sec. 4.2, Eq. (6),(7); Sec. 5.3 "Fast Mixed-Precision GEMM").
 *
 * Conventions that hold for every entry point
 *   - Pointers are DEVICE pointers unless the name ends in _host.
 *   - Matrices are dense row-major with no padding between rows.
 *       X   : M x K        (Fig. 2 caption: the activation is M x K)
 *       Wp  : N x K/2      packed weights, N = output dimension (Table 5 caption)
 *       O   : M x N
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls are asynchronous on that stream; the library never synchronises,
 *     allocates or frees device memory.  The caller owns every buffer.
 *   - Inputs and outputs must not alias.  Device buffers must be 16-byte
 *     aligned (any hipMalloc / torch allocation is).
 *   - Return value: W4A8_OK (0) or a negative W4A8_ERR_* code.  When an error
 *     is returned nothing has been launched and no output was touched.
 *   - Shape contract: M, N >= 1; K >= 32, K % 32 == 0 (a packed row is a
 *     multiple of 16 bytes) and K <= 65536.  The upper bound keeps the
 *     sixteen-fold accumulator of the sign-bit trick (Sec. 5.3) inside int32
 *     even for activations equal to -128 and weights equal to -8.
 */
#ifndef W4A8_H
#define W4A8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define W4A8_OK 0
#define W4A8_ERR_NULL (-1)      /* a required pointer is NULL                          */
#define W4A8_ERR_SHAPE (-2)     /* M, N, K outside the shape contract above            */
#define W4A8_ERR_ALIGN (-3)     /* a device pointer is not 16-byte aligned             */
#define W4A8_ERR_WORKSPACE (-4) /* workspace smaller than w4a8_gemm_workspace_bytes()  */
#define W4A8_ERR_LAUNCH (-5)    /* the HIP runtime rejected the launch                 */
#define W4A8_ERR_VALUE (-6)     /* host helper: a weight code outside [-8, 7]          */
#define W4A8_ERR_ARG (-7)       /* tiling id or variant not available for the shape    */

#define W4A8_MAX_K 65536

/* Library version: major*10000 + minor*100 + patch. */
int w4a8_version(void);

/* Static, never-NULL description of an error code. */
const char *w4a8_strerror(int err);

/* Name of the HIP error behind the last W4A8_ERR_LAUNCH that an entry point returned on the calling thread
 * ("hipSuccess" if none did): static, never NULL. */
const char *w4a8_last_hip_error(void);

/*
 * Per-token activation quantisation (Sec. 3 "Per tensor vs. Per token";
 * Eq. (2) with zero point 0; Table 1 row RTN_pt).
 * For every row m:  amax = max_k |X[m][k]|,  s_a[m] = amax / 127 (fp32 division),
 * Xq[m][k] = clamp(round_half_even(X[m][k] / s_a[m]), -127, 127).
 * A row of zeros yields s_a[m] = 0 and zero codes.  Non-finite inputs are
 * outside the contract.
 *   x_fp16 [M][K] IEEE binary16      in
 *   xq     [M][K] int8               out
 *   s_a    [M]    fp32               out
 */
int w4a8_quantize_act(const void *x_fp16, int8_t *xq, float *s_a, int M, int K, void *stream);

/*
 * The same for an input whose rows are ldx elements apart (ldx >= K, ldx % 8 == 0): a block of K consecutive
 * columns of a wider fp16 matrix, e.g. one projection's slice of a fused QKV output, quantised in place of a copy.
 * xq and s_a are dense as above.
 */
int w4a8_quantize_act_strided(const void *x_fp16, long long ldx, int8_t *xq, float *s_a, int M, int K, void *stream);

/*
 * Bytes of scratch memory w4a8_gemm / w4a8_gemm_acc_i32 / w4a8_gemm_tuned need
 * for this shape: a pure function of the shape.  The present tilings combine
 * their partial sums in LDS and need none, so this returns 0 and the
 * `workspace` argument of the calls below may be NULL; callers that size and
 * pass a buffer from this function stay correct if a later tiling needs one.
 * A workspace, when one is required, must not be shared by calls that may
 * overlap in time (different streams).
 */
size_t w4a8_gemm_workspace_bytes(int M, int N, int K);

/*
 * The W4A8 GEMM with fused dequantisation (Sec. 5.3; Eq. (6),(7)):
 *   O[m][n] = fp16( float( sum_k Xq[m][k] * Wq[n][k] ) * (s_a[m] * s_w[n]) )
 * where Wq[n][k] in [-8,7] is the signed value of the nibble stored in
 * wp[n][k/2] (low nibble for even k, high nibble for odd k; App. A.1: the low
 * four bits of the two's complement are what is packed).  The sum is exact
 * (int32); the scale product is rounded to fp32, multiplied by the fp32 value
 * of the sum and rounded once to fp16 (round to nearest even, overflow to inf).
 *   xq  [M][K]   int8 (any value in [-128,127])  in
 *   s_a [M]      fp32                            in
 *   wp  [N][K/2] uint8                           in, immutable during the call
 *   s_w [N]      fp32 (the paper's s)            in
 *   out_fp16 [M][N] IEEE binary16                out
 */
int w4a8_gemm(const int8_t *xq, const float *s_a, const uint8_t *wp, const float *s_w,
              void *out_fp16, int M, int N, int K,
              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Same contraction, raw result: acc[m][n] = sum_k Xq[m][k] * Wq[n][k] as int32
 * (the division by 16 that undoes the high-nibble placement is already applied).
 * For tests and debugging.
 */
int w4a8_gemm_acc_i32(const int8_t *xq, const uint8_t *wp, int32_t *acc, int M, int N, int K,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Tiled weight layout for large M.  The weights are static, so, like the paper's offline weight format (Sec. 5.3),
 * they may be reordered once after packing into the order in which the large-M kernel consumes them; every wave
 * load then moves whole cache lines.  Same codes, same arithmetic, same results as the row-major array.
 *   Layout of wt: 2048-byte blocks; block (nb, kb), nb = n / 32, kb = k / 128, starts at ((nb * KB) + kb) * 2048
 *   with KB = ceil(K / 128).  Inside a block the 16-byte chunk (c, r), c = 0..3, r = 0..31, at (c * 32 + r) * 16
 *   holds the 32 codes k = 128 kb + 32 c .. + 31 of channel 32 nb + r; a dword holds 8 consecutive codes k0..k7
 *   as nibbles k0 k4 k1 k5 k2 k6 k3 k7 from the lowest to the highest.  Channels >= N and k >= K hold zero codes.
 * w4a8_tiled_weight_bytes: size of wt in bytes (0 for a shape outside the contract).
 * w4a8_tile_weights: wp [N][K/2] (device) in -> wt (device, 16-byte aligned, w4a8_tiled_weight_bytes(N, K)) out.
 * w4a8_gemm_tiled: w4a8_gemm over wt instead of wp (all other arguments as there).  Every M is accepted, and one
 *   copy of the weights, the tiled one, serves them all: up to 16 tokens (token generation) the weight-streaming kernels
 *   read wt directly; so they do from 17 to 64 tokens where all of K fits the registers of a workgroup (K <= 5120 for
 *   49 to 64 tokens, K <= 7168 or 8192 for 17 to 32); above that, and for a longer K, the large-M kernel runs
 *   (w4a8_gemm_tiled_splitk, which has a workspace, serves 17 to 64 tokens with the weight-streaming kernel at any K
 *   and fills the chip with the large-M kernel at a few hundred rows).  w4a8_gemm serves every M from the row-major
 *   array, at up to twice the tiled time for M between 17 and 512.
 */
size_t w4a8_tiled_weight_bytes(int N, int K);
int w4a8_tile_weights(const uint8_t *wp, uint8_t *wt, int N, int K, void *stream);
int w4a8_gemm_tiled(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w,
                    void *out_fp16, int M, int N, int K, void *stream);

/*
 * Offline weight preparation on the device (Sec. 5.1 Eq. (8),(9) with 4 bits
 * and clipping strengths gamma = beta = 1, followed by the packing of App. A.1):
 *   s_w[n] = max_k |W[n][k]| / 7,  Wq = clamp(round_half_even(W / s_w), -8, 7),
 *   wp[n][j] = (Wq[n][2j] & 15) | ((Wq[n][2j+1] & 15) << 4).
 *   w_fp16 [N][K] in, wp [N][K/2] out, s_w [N] out.
 */
int w4a8_quantize_weights(const void *w_fp16, uint8_t *wp, float *s_w, int N, int K, void *stream);

/*
 * The same with the clipping strengths of the symmetric weight clipping (Sec. 5.1, Eq. (8),(9)) given per output
 * channel, e.g. as found by a calibration that is not part of this library:
 *   s_w[n] = max(|gamma[n] * max_k W[n][k]|, |beta[n] * min_k W[n][k]|) / 7   (fp32: products, max, division)
 *   Wq     = clamp(round_half_even(W / s_w), -8, 7)     -- values outside the clipped range saturate, -8 occurs.
 * gamma, beta: fp32 [N] on the device, finite and such that s_w[n] is a normal fp32 or zero; NULL stands for all ones
 * (with both NULL the result equals w4a8_quantize_weights).
 */
int w4a8_quantize_weights_clipped(const void *w_fp16, const float *gamma, const float *beta,
                                  uint8_t *wp, float *s_w, int N, int K, void *stream);

/*
 * The gate and up projections of a gated MLP and the glue behind them in one launch (fusion across operators,
 * Sec. 6.1): w4a8_gemm_tiled over the 2 I channels of both projections, stored INTERLEAVED (channel 2 i = gate_i,
 * channel 2 i + 1 = up_i: the caller interleaves the rows of the two weight matrices before w4a8_quantize_weights and
 * w4a8_tile_weights; s_w_gu follows the same order), with w4a8_silu_mul applied in the epilogue:
 *   h[m][i] = fp16( silu(fp16 gate[m][i]) * fp16 up[m][i] ),  gate / up = the W4A8 linear of Eq. (6),(7)
 * i.e. exactly what w4a8_gemm_tiled followed by w4a8_silu_mul gives on the same weights in the usual order, bit for
 * bit, without the M x 2 I intermediate going to memory.
 *   xq [M][K], s_a [M], wt_gu (tiled array of 2 I channels x K), s_w_gu [2 I]   in;   h_fp16 [M][I]   out.
 *   I follows the K contract (I % 32 == 0, I <= 65536).  Up to 64 tokens the weight-streaming kernel runs (where all
 *   of K fits its waves' registers, as for w4a8_gemm_tiled), otherwise the large-M kernel, which has the fused form
 *   for its 256- and 128-row tiles: from 65 to some hundred tokens w4a8_gemm_tiled and w4a8_silu_mul_quantize are
 *   faster.
 *   M * K and the tiled weight bytes must each be below 0xF0000000 (W4A8_ERR_SHAPE).
 */
int w4a8_gemm_tiled_swiglu(const int8_t *xq, const float *s_a, const uint8_t *wt_gu, const float *s_w_gu, void *h_fp16,
                           int M, int I, int K, void *stream);

/*
 * w4a8_gemm_tiled for shapes whose output tiles alone would leave most of the chip idle (medium M, small N: e.g.
 * 40 tiles for M = 32, N = 5120): K is cut into slices, every (tile, slice) pair is a workgroup of the same kernel that
 * writes its raw int32 sums to a slab of the workspace, and a second kernel adds the slabs and applies Eq. (6),(7).
 * Integer sums do not depend on the order of addition: the output has the bits w4a8_gemm_tiled gives.
 * With 17 to 64 tokens and no tile forced the slices are slices of the weight-streaming kernel instead (each workgroup
 * streams its channels' share of one K slice, with its slice of the activations in registers): as few slices as let a
 * slice of K fit the registers, often one, and then no slab at all.
 *   variant : output tile as for W4A8_TILING_PREFILL_TILED, 0 = library's choice;
 *   splits  : number of K slices, 0 = library's choice (1 when the tiles fill the chip: then this is w4a8_gemm_tiled
 *             and the workspace is not touched), at most 64 and at most K / 128 rounded up;
 *   workspace (device, 16-byte aligned), workspace_bytes: at least splits * M * N * 4 bytes when more than one slice is
 *             used, else W4A8_ERR_WORKSPACE; w4a8_gemm_tiled_workspace_bytes(M, N, K) is the size the library's own
 *             choice (splits = 0) needs, 0 if it does not split.  Contents on return: unspecified.
 *   With more than one slice M * K and the tiled weight bytes must each be below 0xF0000000 (W4A8_ERR_SHAPE).
 */
size_t w4a8_gemm_tiled_workspace_bytes(int M, int N, int K);
int w4a8_gemm_tiled_splitk(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16,
                           int M, int N, int K, int variant, int splits, void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * A whole W4A8 linear at token-generation sizes in one launch: the per-token quantiser of w4a8_quantize_act folded
 * into the weight-streaming GEMM (fusion across operators, Sec. 6.1; the per-token overhead of Sec. 3).  The result is,
 * bit for bit,
 *   w4a8_quantize_act_strided(x_fp16, ldx, xq, s_a, M, K);  w4a8_gemm_tiled(xq, s_a, wt, s_w, out_fp16, M, N, K)
 * without xq ever going to memory: every persistent workgroup copies the fp16 rows into LDS and finds the row maxima,
 * and each of its waves quantises there the part of the rows it multiplies (Eq. (2), z = 0, same rounding rule).
 *   x_fp16 [M] rows of K fp16 values, ldx elements apart (ldx >= K, ldx % 8 == 0)      in
 *   wt     tiled weights of w4a8_tile_weights                                          in
 *   s_w    [N] fp32                                                                    in
 *   out_fp16 [M][N]                                                                    out
 *   s_a_out  [M] fp32 or NULL: where the per-token scales are written as well          out
 * M <= 4 and the rows must fit in LDS twice over (fp16 and int8: about M * K <= 40000); W4A8_ERR_ARG otherwise, and
 * the caller falls back to the two calls above.  Every workgroup repeats the quantisation (about ten vector
 * instructions per value), so the fusion pays for a few tokens only (measured on a LLaMA-13B layer whose four linears
 * all run this way, the gate / up one through w4a8_linear_tiled_swiglu_fp16: 35.3 against 43.5 us at M = 1, 39.9
 * against 44.8 at M = 2, 44.6 against 45.4 at M = 3).
 */
int w4a8_linear_tiled_fp16(const void *x_fp16, long long ldx, const uint8_t *wt, const float *s_w, void *out_fp16,
                           float *s_a_out, int M, int N, int K, void *stream);

/*
 * w4a8_linear_tiled_fp16 over the interleaved gate / up weights of w4a8_gemm_tiled_swiglu, with SiLU * up in the
 * epilogue: from the fp16 input of a gated MLP to h = silu(gate) * up in one launch (Sec. 6.1), bit for bit
 *   w4a8_quantize_act_strided(x_fp16, ldx, xq, s_a, M, K);  w4a8_gemm_tiled_swiglu(xq, s_a, wt_gu, s_w_gu, h_fp16, M, I, K).
 *   x_fp16, ldx, s_a_out as above;  wt_gu, s_w_gu: 2 I interleaved channels;  h_fp16 [M][I] out;  I % 32 == 0.
 * Same limits as w4a8_linear_tiled_fp16 (M <= 4, rows must fit in LDS twice over; W4A8_ERR_ARG otherwise).
 */
int w4a8_linear_tiled_swiglu_fp16(const void *x_fp16, long long ldx, const uint8_t *wt_gu, const float *s_w_gu, void *h_fp16,
                                  float *s_a_out, int M, int I, int K, void *stream);

/*
 * The two entries above with the residual addition and the RMSNorm of w4a8_add_rmsnorm_quantize in front of the
 * quantiser: from the residual stream of a pre-norm decoder layer to the output of the linear behind the norm (QKV, or
 * gate / up with SiLU * up) in one launch at token-generation sizes (Sec. 6.1 taken one operator further).
 *   r = fp16(res + x) (r = x when res_fp16 is NULL),  y = fp16(r * rsqrt(mean r^2 + eps) * gamma),
 *   out = w4a8_linear_tiled_fp16(y, ...)          (swiglu = 0; out_fp16 [M][N])
 *   out = w4a8_linear_tiled_swiglu_fp16(y, ...)   (swiglu = 1; wt, s_w hold N = 2 I interleaved channels, out_fp16 = h [M][N / 2])
 * Every element of r and y is computed with the arithmetic of w4a8_add_rmsnorm_quantize (y may differ from that
 * entry's by an fp16 rounding, since the fp32 sum of squares is taken in another order); the output is, bit for bit,
 * what the entry named above gives on this call's y, which y_out_fp16 hands out for checking.
 *   x_fp16 [M] rows ldx apart, res_fp16 [M] rows ldres apart or NULL (ld >= K, ld % 8 == 0), gamma_fp16 [K], eps >= 0   in
 *   r_out_fp16 [M][K] dense or NULL, y_out_fp16 [M][K] dense or NULL (both written by one workgroup)                   out
 *   r_out_fp16 and y_out_fp16 must not overlap any input: other workgroups are still reading those.
 *   M <= 4, K <= 8192, and the rows must fit in LDS three times over (about M * K <= 28000); W4A8_ERR_ARG otherwise.
 */
int w4a8_linear_tiled_norm_fp16(const void *x_fp16, long long ldx, const void *res_fp16, long long ldres,
                                const void *gamma_fp16, float eps, void *r_out_fp16, void *y_out_fp16, const uint8_t *wt,
                                const float *s_w, void *out_fp16, float *s_a_out, int M, int N, int K, int swiglu,
                                void *stream);

/*
 * w4a8_gemm_tiled_splitk for callers that cannot allocate device memory and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same kernels, same output bits.  The slabs of the K slices live in a scratch array inside the library instead:
 * W4A8_STATIC_SCRATCH_BYTES of device memory per GPU, present from the moment the library is loaded until the process
 * ends.  The call allocates and frees nothing (the first call on a device looks up the array's address, as
 * w4a8_init does).  A shape whose slabs (splits * M * N * 4 bytes, splits being the library's choice or the forced
 * count) exceed the array is refused with W4A8_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share the
 * one array: calls that may overlap in time on the same GPU (different streams, different threads) race on it and
 * must be serialised by the caller; calls on one stream are ordered and safe.  The array's contents carry over from
 * call to call and are never read before they are rewritten.
 */
#define W4A8_STATIC_SCRATCH_BYTES (16u << 20)
int w4a8_gemm_tiled_splitk_static(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w, void *out_fp16,
                                  int M, int N, int K, int variant, int splits, void *stream);

/*
 * Optional set-up for the current device, once per device and process: asks the runtime for the LDS allowance of
 * every kernel that needs more than the default and looks up the address of the static scratch array, so that no
 * later call has to (a first launch made under stream capture or from several threads at once is then as plain as
 * any other).  Calls without it do the same on first use, serialised.  Launches nothing, allocates nothing.
 */
int w4a8_init(void);

/*
 * W8A8 comparison variant (the paper sets its W4A8 against its own W8A8, Table 4): the same contraction and the
 * same epilogue (Eq. (6),(7)) with int8 weight codes,
 *   O[m][n] = fp16( float( sum_k Xq[m][k] * W8[n][k] ) * (s_a[m] * s_w[n]) ),   W8 in [-128, 127],
 * run by the large-M kernel without the int4 conversion.  Per-channel 8-bit weights (Eq. (8),(9) with 8 bits,
 * gamma = beta = 1: s_w = absmax / 127) are what w4a8_quantize_act computes when given the weight matrix as its
 * rows, so there is no separate weight quantiser.
 *   Layout of wt: 4096-byte blocks; block (nb, kb), nb = n / 32, kb = k / 128, starts at ((nb * KB) + kb) * 4096,
 *   KB = ceil(K / 128); inside a block the 16-byte chunk (c, r), c = 0..7, r = 0..31, at (c * 32 + r) * 16 holds
 *   the codes k = 128 kb + 16 c .. + 15 of channel 32 nb + r.  Channels >= N and k >= K hold zeros.
 * w8a8_tiled_weight_bytes: size of wt in bytes (0 for a shape outside the contract).
 * w8a8_tile_weights: w8 [N][K] int8 (device) in -> wt (device, 16-byte aligned) out.
 * w8a8_gemm_tiled: exactly one of out_fp16 / acc_i32 non-NULL (raw int32 sums for tests; s_a, s_w may then be NULL);
 *   variant = output tile as for W4A8_TILING_PREFILL_TILED, 0 = library's choice.  Any M.
 */
size_t w8a8_tiled_weight_bytes(int N, int K);
int w8a8_tile_weights(const int8_t *w8, uint8_t *wt, int N, int K, void *stream);
int w8a8_gemm_tiled(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_w,
                    void *out_fp16, int32_t *acc_i32, int M, int N, int K, int variant, void *stream);

/*
 * Ablation of the weight storage (the paper's "Asym GEMM", Sec. 5.3 / App. A.1 / Sec. 7.2): the vanilla unsigned
 * format stores u = Wq + 8 in [0, 15] in each nibble and subtracts 8 again in registers before the multiplication,
 *   O[m][n] = fp16( float( sum_k Xq[m][k] * (u[n][k] - 8) ) * (s_a[m] * s_w[n]) ),
 * i.e. the result of w4a8_gemm_tiled for Wq = u - 8, at a higher conversion cost (7 instead of 3 vector operations per
 * 8 weights).  ut is the TILED array made by w4a8_tile_weights from the packed unsigned codes
 * (up[n][j] = u[n][2j] | u[n][2j+1] << 4); exactly one of out_fp16 / acc_i32 non-NULL; variant as for
 * W4A8_TILING_PREFILL_TILED.  For measurements and tests; a deployment uses the signed format.
 */
int w4a8_gemm_tiled_unsigned(const int8_t *xq, const float *s_a, const uint8_t *ut, const float *s_w,
                             void *out_fp16, int32_t *acc_i32, int M, int N, int K, int variant, void *stream);

/*
 * Ablation of the scale granularity (the paper's "fine-grained" GEMM: Eq. (5), Fig. 2(b), Sec. 4.2 and 7.2): the
 * weights carry one scale per group of 128 consecutive k and output channel instead of one per channel, so each
 * group's integer sum has to be made floating point and scaled before it can be added to the others:
 *   f[m][n]  = sum over groups g = 0 .. K/128 - 1, in ascending order, in fp32 with one fused multiply-add per group, of
 *              float( sum_{k in group g} Xq[m][k] * Wq[n][k] ) * s_g[g][n],
 *   O[m][n]  = fp16( f[m][n] * s_a[m] ).
 * The per-token factor is common to all groups and is applied once, after the sum.  A group's integer sum is below
 * 2^24 in magnitude, so its conversion to fp32 is exact.
 *   wt   : signed int4 codes in the TILED layout (w4a8_tile_weights), device.
 *   s_g  : group scales, fp32 [K / 128][ldg] (group-major: the scales of one group for all channels are consecutive),
 *          device, 16-byte aligned; ldg >= N, ldg % 4 == 0; columns N .. ldg - 1 are read but never used.
 *   K % 128 == 0; M * K, the tiled weight bytes and (K / 128) * ldg * 4 each below 0xF0000000 (one launch covers the
 *   problem), otherwise W4A8_ERR_SHAPE.
 *   variant: output tile, 0 = library's choice, 1 = 128 x 256 (rows of X x channels), 2 = 256 x 128, 3 = 128 x 128,
 *            4 = 64 x 128, 5 = 64 x 64, 6 = 32 x 128; the 256 x 256 tile of the per-channel kernel does not exist here
 *            because the second, floating-point set of accumulators does not fit the register file beside the first.
 * For measurements and tests: this is the cost the per-channel recipe avoids.
 */
int w4a8_gemm_fine_grained(const int8_t *xq, const float *s_a, const uint8_t *wt, const float *s_g, int ldg,
                           void *out_fp16, int M, int N, int K, int variant, void *stream);

/*
 * Glue between the gate/up GEMM and the down GEMM of a LLaMA MLP:
 *   h[m][i] = fp16( silu(gate_up[m][i]) * gate_up[m][I + i] ),  fp32 arithmetic.
 *   gate_up_fp16 [M][2I] in, h_fp16 [M][I] out.  I % 8 == 0.
 */
int w4a8_silu_mul(const void *gate_up_fp16, void *h_fp16, int M, int I, void *stream);

/*
 * The glue above fused with the per-token quantiser that follows it in a LLaMA MLP (the kind of fusion across
 * operators the paper's engine relies on, Sec. 6.1): h is formed as in w4a8_silu_mul, kept on chip, and quantised
 * exactly as w4a8_quantize_act would quantise it.  The result equals
 *   w4a8_silu_mul(gate_up, h); w4a8_quantize_act(h, xq, s_a)
 * bit for bit, without h going to memory.
 *   gate_up_fp16 [M][2I] in, xq [M][I] int8 out, s_a [M] out.  I follows the K contract (I % 32 == 0, I <= 65536).
 */
int w4a8_silu_mul_quantize(const void *gate_up_fp16, int8_t *xq, float *s_a, int M, int I, void *stream);

/*
 * The per-token quantiser fused behind the residual addition and the RMSNorm of a pre-norm decoder layer (Sec. 6.1:
 * the engine folds the quantiser into the operator in front of each linear; the norm is LLaMA's, not the paper's):
 *   r[m][k] = fp16( fp32(res[m][k]) + fp32(x[m][k]) )                     r = x when res_fp16 is NULL
 *   y[m][k] = fp16( fp32(r[m][k]) * rsqrt( mean_k r[m][k]^2 + eps ) * fp32(gamma[k]) )
 *   (xq, s_a) = w4a8_quantize_act(y)                                      Eq. (2), z = 0, per token
 * in one pass over the row: the mean of squares is an fp32 sum, the reciprocal square root a correctly rounded square
 * root and division, the products are taken in the order written.  xq and s_a are, bit for bit, what
 * w4a8_quantize_act gives on the y this call computes; r is exactly defined; y is within an fp16 rounding of the
 * real-number formula.
 *   x_fp16 [M][K] in;  res_fp16 [M][K] in or NULL;  gamma_fp16 [K] in;  eps >= 0 (W4A8_ERR_ARG otherwise; an all-zero
 *   row needs eps > 0);  r_out_fp16 [M][K] out or NULL (the residual stream that goes on);  y_out_fp16 [M][K] out or
 *   NULL (for inspection: no later step of the path reads it);  xq [M][K] int8 out;  s_a [M] out.
 *   K follows the K contract.  r_out_fp16 may be the same buffer as res_fp16 or x_fp16 (the residual stream updated in
 *   place: every element is read before it is written, by the same thread); no other buffers may overlap.
 */
int w4a8_add_rmsnorm_quantize(const void *x_fp16, const void *res_fp16, const void *gamma_fp16, float eps,
                              void *r_out_fp16, void *y_out_fp16, int8_t *xq, float *s_a, int M, int K, void *stream);

/*
 * Host-side packing of already quantised weights (App. A.1; no GPU needed).
 *   wq_host [N][K] int8 codes in [-8,7]  ->  wp_host [N][K/2].
 * Returns W4A8_ERR_VALUE if a code is out of range, W4A8_ERR_SHAPE if K is odd.
 */
int w4a8_pack_weights_host(const int8_t *wq_host, uint8_t *wp_host, int N, int K);

#ifdef __cplusplus
}
#endif
#endif /* W4A8_H */
