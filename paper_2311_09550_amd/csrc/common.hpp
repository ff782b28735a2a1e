// Internal device helpers shared by the gfx950 kernels of the W4A8 library.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace w4a8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// D(16x16,int32) += A(16x64,int8) * B(64x16,int8).
// Operand layout on a 64-lane wave: lane l supplies row (l & 15) of A and column
// (l & 15) of B, 16 consecutive-in-register bytes of K group (l >> 4).  Lane l
// receives D[4*(l >> 4) + r][l & 15] in register r.  Which 16 values of k a K
// group stands for is the same for A and B, so any assignment of k to
// (group, byte) may be used as long as both operands follow it.
__device__ __forceinline__ v4i mfma_i8_16x16x64(v4i a, v4i b, v4i c) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

// Signed int4 -> signed int8 without a subtraction (Sec. 5.3 "Reusing the sign
// bit", App. A.1): each stored nibble is moved into the high half of a byte, so
// the byte reads as 16 times the weight.  One packed word holds k = 0..7
// (low nibble of byte j is k = 2j, high nibble is k = 2j+1):
//   even = bytes {16 w0, 16 w2, 16 w4, 16 w6},  odd = bytes {16 w1, 16 w3, 16 w5, 16 w7}.
__device__ __forceinline__ void sint4_to_s8x16(unsigned w, int &even, int &odd) {
    even = (int)((w << 4) & 0xF0F0F0F0u);
    odd = (int)(w & 0xF0F0F0F0u);
}

// Two packed words (k = 0..15 of a lane's K group) -> one MFMA operand whose
// registers hold k = {0,2,4,6}, {1,3,5,7}, {8,10,12,14}, {9,11,13,15}.
__device__ __forceinline__ v4i w_operand(unsigned w0, unsigned w1) {
    v4i r;
    int e, o;
    sint4_to_s8x16(w0, e, o);
    r.x = e;
    r.y = o;
    sint4_to_s8x16(w1, e, o);
    r.z = e;
    r.w = o;
    return r;
}

// Two dwords of the TILED weight layout (16 codes; nibbles of a dword hold k0 k4 k1 k5 k2 k6 k3 k7 from the lowest
// up) -> one MFMA operand: int8 values 16 * w in the natural k order, so the activations need no reordering.
__device__ __forceinline__ v4i w_operand_tiled(unsigned w0, unsigned w1) {
    v4i r;
    r.x = (int)((w0 << 4) & 0xF0F0F0F0u);
    r.y = (int)(w0 & 0xF0F0F0F0u);
    r.z = (int)((w1 << 4) & 0xF0F0F0F0u);
    r.w = (int)(w1 & 0xF0F0F0F0u);
    return r;
}

// 16 consecutive int8 activations (k = 0..15) reordered to the k order of
// w_operand: bytes {0,2,4,6}, {1,3,5,7} of the first eight, then of the second eight.
__device__ __forceinline__ v4i x_operand(v4u x) {
    v4i r;
    r.x = (int)__builtin_amdgcn_perm(x.y, x.x, 0x06040200u);
    r.y = (int)__builtin_amdgcn_perm(x.y, x.x, 0x07050301u);
    r.z = (int)__builtin_amdgcn_perm(x.w, x.z, 0x06040200u);
    r.w = (int)__builtin_amdgcn_perm(x.w, x.z, 0x07050301u);
    return r;
}

// Dequantisation after the GEMM (Eq. (6),(7)): acc16 is sixteen times the true
// sum; the arithmetic shift restores it exactly (its low four bits are zero).
// Both products are rounded to fp32 (S_ij = s_a * s_w first, Eq. (7)); the rounding to fp16 follows in
// f32_to_f16_bits.
__device__ __forceinline__ float dequant(int acc16, float s_a, float s_w) {
    const float s_ij = s_a * s_w;
    return (float)(acc16 >> 4) * s_ij;
}

// fp32 -> fp16, round to nearest even, of a FINISHED fp32 value.  The empty asm makes v opaque at this point:
// otherwise the compiler may merge the multiplication that produced v with the conversion into one mixed-precision
// FMA (v_fma_mixlo_f16), which rounds the exact product once and lands on the other fp16 neighbour in some tie
// cases.  Whether it merges depends on the surrounding code, so two kernels with the same source arithmetic could
// differ in the last bit; the definition is "fp32 value, then one rounding to fp16" (Eq. (6),(7) give an fp32 O).
__device__ __forceinline__ unsigned short f32_to_f16_bits(float v) {
    asm("" : "+v"(v));
    return __half_as_ushort(__float2half_rn(v));
}

__device__ __forceinline__ unsigned pack_f16x2(float lo, float hi) {
    return (unsigned)f32_to_f16_bits(lo) | ((unsigned)f32_to_f16_bits(hi) << 16);
}

// ---- per-token / per-channel symmetric quantisation, shared by the row-wise quantisers and by the
// token-generation GEMM that quantises its own activations

__device__ __forceinline__ float half_bits_to_float(unsigned short h) { return __half2float(__ushort_as_half(h)); }
__device__ __forceinline__ float lo_half(unsigned w) { return half_bits_to_float((unsigned short)(w & 0xFFFFu)); }
__device__ __forceinline__ float hi_half(unsigned w) { return half_bits_to_float((unsigned short)(w >> 16)); }

// Running absolute maximum of fp16 values, two at a time: with the sign bits cleared, finite fp16 values order like
// their bit patterns, so the maximum is a packed 16-bit integer maximum (one AND and one v_pk_max_u16 per two values)
// and nothing is converted until the end.  m2 holds the two running maxima (start from 0).
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned absmax8_packed(v4u c, unsigned m2) {
    u16x2 m = __builtin_bit_cast(u16x2, m2);
#pragma unroll
    for (int j = 0; j < 4; ++j) m = __builtin_elementwise_max(m, __builtin_bit_cast(u16x2, c[j] & 0x7FFF7FFFu));
    return __builtin_bit_cast(unsigned, m);
}
__device__ __forceinline__ float absmax_packed_value(unsigned m2) {
    return half_bits_to_float((unsigned short)max(m2 & 0xFFFFu, m2 >> 16));
}

// Pieces of the residual addition + RMSNorm in front of a quantiser, shared by the row-wise kernel and the linear that
// takes them in, so that both apply the same arithmetic to an element: eight sums fp16(fp32(a) + fp32(b)); the fp32
// sum of eight squares added to a running sum; eight values fp16(fp32(r) * inv * fp32(g)).
__device__ __forceinline__ v4u add_halves8(v4u a, v4u b) {
    v4u o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = pack_f16x2(lo_half(a[j]) + lo_half(b[j]), hi_half(a[j]) + hi_half(b[j]));
    return o;
}
__device__ __forceinline__ float add_squares8(v4u r, float ss) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float a = lo_half(r[j]), b = hi_half(r[j]);
        ss += a * a;
        ss += b * b;
    }
    return ss;
}
__device__ __forceinline__ v4u norm_scale8(v4u r, float inv, v4u g) {
    v4u o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = pack_f16x2(lo_half(r[j]) * inv * lo_half(g[j]), hi_half(r[j]) * inv * hi_half(g[j]));
    return o;
}
// 1 / sqrt(sum / count + eps): correctly rounded division, square root and division
__device__ __forceinline__ float rms_inverse(float sum, int count, float eps) {
    return __fdiv_rn(1.0f, __fsqrt_rn(__fdiv_rn(sum, (float)count) + eps));
}

// Maximum over the wave of a non-negative value (as such it orders like its bit pattern), in every lane.  Six DPP steps
// in the vector ALU: shifts within rows of 16 lanes (lanes shifted in from outside a row contribute 0), then lane 15 of
// a row broadcast into the next row and lane 31 into the upper half; lane 63 ends up with the maximum.  A butterfly of
// shuffles, which goes through the LDS crossbar, costs six dependent LDS round trips instead.
__device__ __forceinline__ float wave_max_nonneg(float v) {
    int x = __float_as_int(v);
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true));   // row_shr:1
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true));   // row_shr:2
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true));   // row_shr:4
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true));   // row_shr:8
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false));  // row_bcast:15 into rows 1 and 3
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false));  // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(x, 63));
}

// Sum over the wave, in every lane, by the same six DPP steps with additions: a prefix sum inside each row of 16 lanes
// (lanes shifted in from outside a row contribute 0), then the rows' totals passed on; lane 63 ends up with the sum.
// The order of the additions is fixed, so the result is the same on every run.
__device__ __forceinline__ float wave_sum(float v) {
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x111, 0xF, 0xF, true));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x112, 0xF, 0xF, true));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xF, 0xF, true));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xF, 0xF, true));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x142, 0xA, 0xF, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x143, 0xC, 0xF, false));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Symmetric quantisation of one row (Eq. (2) with zero point 0): code = clamp(rne(fl32(x / scale)), lo, hi).
//
// The definition divides.  A correctly rounded fp32 division costs about ten instructions, so the common case
// takes a shortcut that provably gives the same integer: with r = fl32(1/scale) and q' = fl32(x * r),
// |q' - x/scale| <= |x/scale| * (2^-23 + 2^-48) < 1.6e-5 for |x/scale| <= 128, and the definition's quotient
// fl32(x/scale) lies within 3.9e-6 of x/scale.  So when q' is at least 1e-4 away from the nearest half-integer,
// both quotients round to the same integer; otherwise (about 2 in 10^4 elements, or rows whose quotients are
// exact halves) the eight values of the chunk are redone with the division.
struct RowQuantizer {
    float scale, recip, lo, hi;
    __device__ __forceinline__ RowQuantizer(float amax, float qmax, float lo_, float hi_) : lo(lo_), hi(hi_) {
        scale = __fdiv_rn(amax, qmax);
        recip = __fdiv_rn(1.0f, scale);  // unused when amax == 0
    }
    __device__ __forceinline__ void codes8(const float (&x)[8], int (&q)[8]) const {
        bool near_tie = false;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float qp = x[j] * recip;
            const float n = rintf(qp);
            near_tie |= fabsf(qp - n) > 0.5f - 1e-4f;
            q[j] = (int)fminf(fmaxf(n, lo), hi);
        }
        if (near_tie) {
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = (int)fminf(fmaxf(rintf(__fdiv_rn(x[j], scale)), lo), hi);
        }
    }
    // The same eight codes as bytes of two words, for rows quantised to [-qmax, qmax] with the row's own maximum
    // (the activation quantisers).  There the shortcut needs no clamp: |x| <= amax gives |q'| <= qmax (1 + 3 * 2^-24),
    // which rounds to at most qmax.  Rounding by adding 1.5 * 2^23: the sum's low mantissa bits are rne(q') in two's
    // complement, so its low byte is the code, and sum - 1.5 * 2^23 is rne(q') as a float, exactly.
    __device__ __forceinline__ v2u packed8_own_max(const float (&x)[8]) const {
        constexpr float kShift = 12582912.0f;
        unsigned b[8];
        float off = 0.f;  // largest distance of a q' from its nearest integer
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // fused: t = rne(x * recip) + kShift with the product exact (closer to x / scale than q' is, so the
            // bound above holds a fortiori), and the distance from the same exact product.  With fp16 inputs each is
            // one v_fma_mix_f32, which converts its operand on the way in.
            const float t = fmaf(x[j], recip, kShift);
            off = fmaxf(off, fabsf(fmaf(x[j], recip, kShift - t)));
            b[j] = __float_as_uint(t);
        }
        if (off > 0.5f - 1e-4f) {
#pragma unroll
            for (int j = 0; j < 8; ++j) b[j] = (unsigned)(int)fminf(fmaxf(rintf(__fdiv_rn(x[j], scale)), lo), hi);
        }
        v2u o;  // v_perm_b32: selector bytes 0-3 pick from the second operand, 4-7 from the first, 0x0c gives zero
        const unsigned p01 = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), p23 = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
        const unsigned p45 = __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), p67 = __builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u);
        o.x = __builtin_amdgcn_perm(p23, p01, 0x05040100u);
        o.y = __builtin_amdgcn_perm(p67, p45, 0x05040100u);
        return o;
    }
};

// silu(gate) * up in fp32 from two fp16 values: g / (1 + e^-g) with the hardware's exp2 and reciprocal (about 1 ulp of
// fp32 each), three orders of magnitude below the fp16 rounding that follows.  exp2 overflows to +inf for very negative
// g, the reciprocal of that is 0: silu(-65504) = -0.  One definition for the row-wise kernels and for the GEMM epilogue
// that applies it, so that both give the same fp16 bits.
__device__ __forceinline__ float silu_mul_f32(float gt, float up) {
    return gt * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(gt * -1.4426950408889634f)) * up;
}

// Four (gate, up) pairs held as fp16 pairs in four words (low half = gate, high half = up) -> four fp16 products.
__device__ __forceinline__ v2u silu_mul_pairs4(v4u v) {
    v2u o;
    o.x = pack_f16x2(silu_mul_f32(lo_half(v.x), hi_half(v.x)), silu_mul_f32(lo_half(v.y), hi_half(v.y)));
    o.y = pack_f16x2(silu_mul_f32(lo_half(v.z), hi_half(v.z)), silu_mul_f32(lo_half(v.w), hi_half(v.w)));
    return o;
}

__device__ __forceinline__ void halves8(v4u v, float (&x)[8]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[2 * j] = lo_half(v[j]);
        x[2 * j + 1] = hi_half(v[j]);
    }
}

}  // namespace w4a8
