// Device-side helpers shared by the gfx950 kernels: bf16 <-> fp32, the
// saturating FP8 cast, the SwiGLU product and its derivatives, reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssg {

constexpr int kE4M3 = 0;
constexpr int kE5M2 = 1;
constexpr int kBF16 = 2;            // operand type of the unquantized (bf16) GEMMs, beside the two FP8 formats

template <int FMT> struct Fp8Traits;
// overflow_above = fmax plus half the spacing of the top binade: a magnitude beyond it is kept finite only by
// the clamp of the saturating cast (a value between fmax and it rounds to fmax by itself)
template <> struct Fp8Traits<kE4M3> { static constexpr float fmax = 448.0f, overflow_above = 464.0f; };
template <> struct Fp8Traits<kE5M2> { static constexpr float fmax = 57344.0f, overflow_above = 61440.0f; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Two fp32 -> one packed pair of bf16 (lo in bits 0..15), round to nearest even, with the chip's
// conversion instruction (v_cvt_pk_bf16_f32): one operation instead of a dozen per pair.
typedef __bf16 ssg_bf16x2 __attribute__((ext_vector_type(2)));
typedef float ssg_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const ssg_f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, ssg_bf16x2));
}

// Per-tensor scale (Section 2; Q of Eq. 2): fl32(fmax / amax), 1 for an empty
// range, clamped to the largest finite float; optionally rounded down to a
// power of two by clearing the mantissa.
__device__ __forceinline__ float scale_from_amax(float amax, float fmax, int pow2) {
    float s = 1.0f;
    if (amax > 0.0f) {
        s = __fdiv_rn(fmax, amax);
        s = fminf(s, 3.402823466e+38f);
    }
    if (pow2) s = __uint_as_float(__float_as_uint(s) & 0xff800000u);
    return s;
}

// Two fp32 values -> two FP8 codes in the low 16 bits.  The hardware
// conversion rounds to nearest even through the subnormal range but turns
// out-of-range magnitudes into NaN/Inf codes, so the value is clamped to the
// largest finite magnitude first.  NaN keeps its sign and becomes S.1111111.
template <int FMT>
__device__ __forceinline__ uint32_t satcast_pk2(float a, float b) {
    constexpr float fmax = Fp8Traits<FMT>::fmax;
    float ca = __builtin_amdgcn_fmed3f(a, -fmax, fmax);
    float cb = __builtin_amdgcn_fmed3f(b, -fmax, fmax);
    uint32_t p;
    if (FMT == kE4M3) p = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(ca, cb, 0, false);
    else              p = (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(ca, cb, 0, false);
    p &= 0xffffu;
    if (__builtin_expect(a != a, 0)) p = (p & 0xff00u) | 0x7fu | ((__float_as_uint(a) >> 24) & 0x80u);
    if (__builtin_expect(b != b, 0)) p = (p & 0x00ffu) | ((0x7fu | ((__float_as_uint(b) >> 24) & 0x80u)) << 8);
    return p;
}

template <int FMT>
__device__ __forceinline__ uint32_t satcast_pk4(float a, float b, float c, float d) {
    return satcast_pk2<FMT>(a, b) | (satcast_pk2<FMT>(c, d) << 16);
}

// The same for eight values in ALU-bound epilogues: one NaN test for all eight (x - x is 0 for every finite x and
// NaN for NaN and infinities, and NaN is sticky through the sum), and the per-element NaN patch only when it fires.
template <int FMT>
__device__ __forceinline__ uint2 satcast_pk8(const float (&v)[8]) {
    float probe = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) probe += v[k] - v[k];
    if (__builtin_expect(probe != probe, 0))
        return make_uint2(satcast_pk4<FMT>(v[0], v[1], v[2], v[3]), satcast_pk4<FMT>(v[4], v[5], v[6], v[7]));
    constexpr float fmax = Fp8Traits<FMT>::fmax;
    uint32_t w[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float a = __builtin_amdgcn_fmed3f(v[4 * h], -fmax, fmax), b = __builtin_amdgcn_fmed3f(v[4 * h + 1], -fmax, fmax);
        const float c = __builtin_amdgcn_fmed3f(v[4 * h + 2], -fmax, fmax), d = __builtin_amdgcn_fmed3f(v[4 * h + 3], -fmax, fmax);
        if (FMT == kE4M3)
            w[h] = ((uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xffffu) |
                   ((uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c, d, 0, false) << 16);
        else
            w[h] = ((uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, 0, false) & 0xffffu) |
                   ((uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(c, d, 0, false) << 16);
    }
    return make_uint2(w[0], w[1]);
}

// SwiGLU neuron of Section 4.1 in fp32: u * Swish(g), Swish(g) = g * sigma(g).
// Every operation is a single rounded fp32 operation in a fixed order so that
// the GEMM epilogue and the stand-alone pass produce identical bits.
//
// sigma(g) = 1/(1+e^-g) = e^g/(1+e^g) is evaluated with t = e^-|g| <= 1 so that nothing
// overflows for strongly negative g (the large-|g| regime is the one the method is about).
// t = 2^(y) with y = -|g| * log2(e) carried as a rounded product plus its exact remainder
// (two fused multiply-adds against a split constant), so the hardware exp2 (1 ulp) sees an
// argument that is exact to ~2^-48 and the error does not grow with |g|; the reciprocal is the
// hardware one (1 ulp).  Total error of u*g*sigma(g): < 6 ulp.  t below the smallest normal
// float is flushed to zero by the hardware exp2.
__device__ __forceinline__ float sigmoid_f32(float g) {
    const float x = -fabsf(g);
    constexpr float kLog2eHi = 1.44269502162933349609375f;        // float(log2 e)
    constexpr float kLog2eLo = 1.925963033500011e-08f;            // log2 e - kLog2eHi
    const float y_hi = __fmul_rn(x, kLog2eHi);
    const float y_lo = __fmaf_rn(x, kLog2eLo, __fmaf_rn(x, kLog2eHi, -y_hi));
    // 2^(y_hi + y_lo) = 2^y_hi * (1 + y_lo * ln 2 + ...), |y_lo| < 2^-17
    const float e_hi = __builtin_amdgcn_exp2f(y_hi);
    const float t = __fmaf_rn(e_hi, __fmul_rn(y_lo, 0.693147182464599609375f), e_hi);
    const float r = __builtin_amdgcn_rcpf(__fadd_rn(1.0f, t));
    return g >= 0.0f ? r : __fmul_rn(t, r);
}
__device__ __forceinline__ float swiglu_f32(float u, float g) {
    float sw = __fmul_rn(g, sigmoid_f32(g));
    return __fmul_rn(u, sw);
}
// d h / d u = g*sigma(g);  d h / d g = u * sigma(g) * (1 + g * (1 - sigma(g)))
// The gradients are rounded to bf16 right away and compared with a GEMM-level tolerance, so the
// sigmoid here uses the hardware exp2 / reciprocal (about 2 ulp, plus |g| * 2^-24 from the scaled
// argument) instead of the correctly rounded sequence of the forward pass: ~4x fewer VALU
// instructions in an epilogue that is otherwise ALU bound.
__device__ __forceinline__ float sigmoid_fast_f32(float g) {
    // 1 / (1 + 2^(-g log2 e)); for g below about -88 the power overflows to +inf and the quotient is 0
    // where the true value is below the smallest normal number
    const float t = __builtin_amdgcn_exp2f(g * -1.44269504088896340736f);
    return __builtin_amdgcn_rcpf(1.0f + t);
}
__device__ __forceinline__ void swiglu_grad_f32(float u, float g, float dh, float &du, float &dg) {
    const float sg = sigmoid_fast_f32(g);
    du = dh * (g * sg);
    dg = (dh * u) * (sg * (1.0f + g * (1.0f - sg)));
}

// |x| of a non-NaN float as an unsigned integer orders like the float; NaN -> 0.
__device__ __forceinline__ uint32_t abs_bits_ignore_nan(float v) {
    uint32_t u = __float_as_uint(v) & 0x7fffffffu;
    return u > 0x7f800000u ? 0u : u;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
        v = v > o ? v : o;
    }
    return v;
}

}  // namespace ssg
