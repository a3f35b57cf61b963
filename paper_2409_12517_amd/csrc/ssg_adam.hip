// Adam step with the first moment stored in E4M3 and the second in E5M2 (Section 5).
//
// Two HBM-bound passes over a flat parameter tensor, 16 elements per lane per trip (16-byte
// accesses for the codes as well as for the gradient and the weights):
//   pass 1  new moments from the stored codes and the gradient, their ranges (max|m|, max v)
//           into 64 slotted atomics each;
//   pass 2  the same moments again (bit-identical: same inputs, same operations), the
//           bias-corrected update of the fp32 master weights (optionally a bf16 copy), and the
//           moments re-encoded with the per-tensor scales fmax / range.
// Every arithmetic step is a single rounded fp32 operation in a fixed order (the build disables
// contraction and uses correctly rounded division and square root), so codes, scales and
// weights can be compared bit for bit with a binary32 reference.
//
// State scalars are kept twice, by step parity, so that pass 2 can read the old scales and
// range slots while workgroup 0 writes the new ones and clears the slots of the next step.
#include "ssg_device.h"
#include "ssg_internal.h"

namespace ssg {

struct AdamParams {
    const void *grad;
    float *w;
    uint16_t *w_bf16;
    uint8_t *m_q, *v_q;
    uint32_t *scalars;          // AdamScalars layout below, as words
    int64_t n;
    float b1, b2, omb1, omb2, c1, c2, lr, eps, wd;
    int parity;                 // step & 1: the set written by this step
    int pow2;
};

// word offsets in the scalar block
constexpr int kAdamScaleM = 0, kAdamScaleV = 1, kAdamAmaxM = 2, kAdamAmaxV = 3;   // + 8 * parity
constexpr int kAdamSlotsM = 64;                                                  // + parity * 2 * kAmaxSlotWords
constexpr int kAdamThreads = 256;

template <bool GRAD_BF16>
__device__ __forceinline__ void load_grad8(const void *grad, size_t i, float (&g)[8]) {
    if (GRAD_BF16) {
        const uint4 q = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(grad) + i);
        const uint32_t w4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            g[2 * k] = __uint_as_float(w4[k] << 16);
            g[2 * k + 1] = __uint_as_float(w4[k] & 0xffff0000u);
        }
    } else {
        const float4 a = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(grad) + i);
        const float4 b = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(grad) + i + 4);
        g[0] = a.x; g[1] = a.y; g[2] = a.z; g[3] = a.w; g[4] = b.x; g[5] = b.y; g[6] = b.z; g[7] = b.w;
    }
}

// 8 * HALVES codes as words: one 8- or 16-byte access
template <int HALVES>
__device__ __forceinline__ void load_codes(const uint8_t *src, uint32_t (&q)[2 * HALVES]) {
    if (HALVES == 1) {
        const uint2 t = *reinterpret_cast<const uint2 *>(src);
        q[0] = t.x; q[1] = t.y;
    } else {
        const uint4 t = *reinterpret_cast<const uint4 *>(src);
        q[0] = t.x; q[1] = t.y; q[2 * (HALVES - 1)] = t.z; q[2 * (HALVES - 1) + 1] = t.w;
    }
}
template <int HALVES>
__device__ __forceinline__ void store_codes(uint8_t *dst, const uint32_t (&q)[2 * HALVES]) {
    if (HALVES == 1) *reinterpret_cast<uint2 *>(dst) = make_uint2(q[0], q[1]);
    else *reinterpret_cast<uint4 *>(dst) = make_uint4(q[0], q[1], q[2 * (HALVES - 1)], q[2 * (HALVES - 1) + 1]);
}

// eight stored moments from two words of codes, as fp32: decode(code) * (1 / scale)
__device__ __forceinline__ void decode_moments8(uint32_t m0, uint32_t m1, uint32_t v0, uint32_t v1, float inv_sm,
                                                float inv_sv, float (&m)[8], float (&v)[8]) {
    const uint32_t mw[2] = {m0, m1}, vw[2] = {v0, v1};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        m[4 * h + 0] = __fmul_rn(__builtin_amdgcn_cvt_f32_fp8((int)mw[h], 0), inv_sm);
        m[4 * h + 1] = __fmul_rn(__builtin_amdgcn_cvt_f32_fp8((int)mw[h], 1), inv_sm);
        m[4 * h + 2] = __fmul_rn(__builtin_amdgcn_cvt_f32_fp8((int)mw[h], 2), inv_sm);
        m[4 * h + 3] = __fmul_rn(__builtin_amdgcn_cvt_f32_fp8((int)mw[h], 3), inv_sm);
        v[4 * h + 0] = __fmul_rn(__builtin_amdgcn_cvt_f32_bf8((int)vw[h], 0), inv_sv);
        v[4 * h + 1] = __fmul_rn(__builtin_amdgcn_cvt_f32_bf8((int)vw[h], 1), inv_sv);
        v[4 * h + 2] = __fmul_rn(__builtin_amdgcn_cvt_f32_bf8((int)vw[h], 2), inv_sv);
        v[4 * h + 3] = __fmul_rn(__builtin_amdgcn_cvt_f32_bf8((int)vw[h], 3), inv_sv);
    }
}

// exponential moving averages of the gradient and of its square
__device__ __forceinline__ void new_moments8(const AdamParams &p, const float (&g)[8], float (&m)[8], float (&v)[8]) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        m[k] = __fadd_rn(__fmul_rn(p.b1, m[k]), __fmul_rn(p.omb1, g[k]));
        v[k] = __fadd_rn(__fmul_rn(p.b2, v[k]), __fmul_rn(__fmul_rn(p.omb2, g[k]), g[k]));
    }
}

template <bool GRAD_BF16, int HALVES>
__global__ void __launch_bounds__(kAdamThreads) adam_range_kernel(AdamParams p) {
    const uint32_t *old = p.scalars + 8 * (p.parity ^ 1);
    const float inv_sm = __fdiv_rn(1.0f, __uint_as_float(old[kAdamScaleM])), inv_sv = __fdiv_rn(1.0f, __uint_as_float(old[kAdamScaleV]));
    uint32_t mmax = 0, vmax = 0;
    constexpr int kPer = 8 * HALVES;
    const size_t stride = (size_t)gridDim.x * kAdamThreads * kPer;
    for (size_t i = ((size_t)blockIdx.x * kAdamThreads + threadIdx.x) * kPer; i < (size_t)p.n; i += stride) {
        uint32_t mq[2 * HALVES], vq[2 * HALVES];
        load_codes<HALVES>(p.m_q + i, mq);
        load_codes<HALVES>(p.v_q + i, vq);
        float g[HALVES][8];
#pragma unroll
        for (int h = 0; h < HALVES; ++h) load_grad8<GRAD_BF16>(p.grad, i + 8 * h, g[h]);
#pragma unroll
        for (int h = 0; h < HALVES; ++h) {
            float m[8], v[8];
            decode_moments8(mq[2 * h], mq[2 * h + 1], vq[2 * h], vq[2 * h + 1], inv_sm, inv_sv, m, v);
            new_moments8(p, g[h], m, v);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint32_t a = abs_bits_ignore_nan(m[k]), b = abs_bits_ignore_nan(v[k]);
                mmax = mmax > a ? mmax : a;
                vmax = vmax > b ? vmax : b;
            }
        }
    }
    mmax = wave_max_u32(mmax);
    vmax = wave_max_u32(vmax);
    __shared__ uint32_t red[2 * (kAdamThreads / 64)];
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { red[2 * w] = mmax; red[2 * w + 1] = vmax; }
    __syncthreads();
    if (threadIdx.x < 2) {
        uint32_t r = 0;
#pragma unroll
        for (int k = 0; k < kAdamThreads / 64; ++k) r = r > red[2 * k + threadIdx.x] ? r : red[2 * k + threadIdx.x];
        uint32_t *slots = p.scalars + kAdamSlotsM + (size_t)p.parity * 2 * kAmaxSlotWords + threadIdx.x * kAmaxSlotWords;
        if (r) atomicMax(slots + (blockIdx.x % kAmaxSlots) * kAmaxSlotStride, r);
    }
}

template <bool GRAD_BF16, int HALVES>
__global__ void __launch_bounds__(kAdamThreads) adam_update_kernel(AdamParams p) {
    const uint32_t *old = p.scalars + 8 * (p.parity ^ 1);
    const float inv_sm = __fdiv_rn(1.0f, __uint_as_float(old[kAdamScaleM])), inv_sv = __fdiv_rn(1.0f, __uint_as_float(old[kAdamScaleV]));
    // ranges of the new moments: maximum over the slots (one slot per lane, then across the wave)
    const uint32_t *slots_m = p.scalars + kAdamSlotsM + (size_t)p.parity * 2 * kAmaxSlotWords;
    const uint32_t *slots_v = slots_m + kAmaxSlotWords;
    const int lane = threadIdx.x & 63;
    const float amax_m = __uint_as_float(wave_max_u32(slots_m[lane * kAmaxSlotStride]));
    const float amax_v = __uint_as_float(wave_max_u32(slots_v[lane * kAmaxSlotStride]));
    const float sm = scale_from_amax(amax_m, Fp8Traits<kE4M3>::fmax, p.pow2);
    const float sv = scale_from_amax(amax_v, Fp8Traits<kE5M2>::fmax, p.pow2);
    if (blockIdx.x == 0) {
        uint32_t *cur = p.scalars + 8 * p.parity;
        if (threadIdx.x == 0) {
            cur[kAdamScaleM] = __float_as_uint(sm); cur[kAdamScaleV] = __float_as_uint(sv);
            cur[kAdamAmaxM] = __float_as_uint(amax_m); cur[kAdamAmaxV] = __float_as_uint(amax_v);
        }
        // the other parity's slots were last read by the previous step's update pass: clear them for the next step
        uint32_t *next = p.scalars + kAdamSlotsM + (size_t)(p.parity ^ 1) * 2 * kAmaxSlotWords;
        if (threadIdx.x < 2 * kAmaxSlots)
            next[(threadIdx.x >> 6) * kAmaxSlotWords + (threadIdx.x & 63) * kAmaxSlotStride] = 0u;
    }
    constexpr int kPer = 8 * HALVES;
    const size_t stride = (size_t)gridDim.x * kAdamThreads * kPer;
    for (size_t i = ((size_t)blockIdx.x * kAdamThreads + threadIdx.x) * kPer; i < (size_t)p.n; i += stride) {
        uint32_t mq[2 * HALVES], vq[2 * HALVES];
        load_codes<HALVES>(p.m_q + i, mq);
        load_codes<HALVES>(p.v_q + i, vq);
        float g[HALVES][8];
        float4 wv[2 * HALVES];
#pragma unroll
        for (int h = 0; h < HALVES; ++h) load_grad8<GRAD_BF16>(p.grad, i + 8 * h, g[h]);
#pragma unroll
        for (int q = 0; q < 2 * HALVES; ++q) wv[q] = *reinterpret_cast<const float4 *>(p.w + i + 4 * q);
        uint32_t mo[2 * HALVES], vo[2 * HALVES];
#pragma unroll
        for (int h = 0; h < HALVES; ++h) {
            float m[8], v[8];
            float w[8] = {wv[2 * h].x, wv[2 * h].y, wv[2 * h].z, wv[2 * h].w,
                          wv[2 * h + 1].x, wv[2 * h + 1].y, wv[2 * h + 1].z, wv[2 * h + 1].w};
            decode_moments8(mq[2 * h], mq[2 * h + 1], vq[2 * h], vq[2 * h + 1], inv_sm, inv_sv, m, v);
            new_moments8(p, g[h], m, v);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                // bias-corrected step, decoupled decay
                const float mhat = __fmul_rn(m[k], p.c1);
                const float vhat = __fmul_rn(v[k], p.c2);
                const float denom = __fadd_rn(sqrtf(vhat), p.eps);   // sqrtf, not __fsqrt_rn: only the former is correctly rounded here
                float upd = __fdiv_rn(mhat, denom);
                upd = __fadd_rn(upd, __fmul_rn(p.wd, w[k]));
                w[k] = __fsub_rn(w[k], __fmul_rn(p.lr, upd));
            }
            wv[2 * h] = make_float4(w[0], w[1], w[2], w[3]);
            wv[2 * h + 1] = make_float4(w[4], w[5], w[6], w[7]);
            mo[2 * h] = satcast_pk4<kE4M3>(__fmul_rn(m[0], sm), __fmul_rn(m[1], sm), __fmul_rn(m[2], sm), __fmul_rn(m[3], sm));
            mo[2 * h + 1] = satcast_pk4<kE4M3>(__fmul_rn(m[4], sm), __fmul_rn(m[5], sm), __fmul_rn(m[6], sm), __fmul_rn(m[7], sm));
            vo[2 * h] = satcast_pk4<kE5M2>(__fmul_rn(v[0], sv), __fmul_rn(v[1], sv), __fmul_rn(v[2], sv), __fmul_rn(v[3], sv));
            vo[2 * h + 1] = satcast_pk4<kE5M2>(__fmul_rn(v[4], sv), __fmul_rn(v[5], sv), __fmul_rn(v[6], sv), __fmul_rn(v[7], sv));
        }
#pragma unroll
        for (int q = 0; q < 2 * HALVES; ++q) *reinterpret_cast<float4 *>(p.w + i + 4 * q) = wv[q];
        if (p.w_bf16) {
#pragma unroll
            for (int h = 0; h < HALVES; ++h)
                *reinterpret_cast<uint4 *>(p.w_bf16 + i + 8 * h) =
                    make_uint4(pack_bf16x2(wv[2 * h].x, wv[2 * h].y), pack_bf16x2(wv[2 * h].z, wv[2 * h].w),
                               pack_bf16x2(wv[2 * h + 1].x, wv[2 * h + 1].y), pack_bf16x2(wv[2 * h + 1].z, wv[2 * h + 1].w));
        }
        store_codes<HALVES>(p.m_q + i, mo);
        store_codes<HALVES>(p.v_q + i, vo);
    }
}

__global__ void adam_init_kernel(uint32_t *scalars, size_t scalar_words, uint4 *codes, size_t n16) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t k = i; k < scalar_words; k += stride) {
        // scales 1.0 in both parity sets, everything else (ranges, slots) zero
        const bool is_scale = k == kAdamScaleM || k == kAdamScaleV || k == 8 + kAdamScaleM || k == 8 + kAdamScaleV;
        scalars[k] = is_scale ? 0x3f800000u : 0u;
    }
    for (size_t k = i; k < n16; k += stride) codes[k] = make_uint4(0u, 0u, 0u, 0u);
}

size_t adam_scalar_words() { return (size_t)kAdamSlotsM + 4 * kAmaxSlotWords; }

void launch_adam_init(uint32_t *scalars, uint8_t *codes, size_t code_bytes, hipStream_t st) {
    hipLaunchKernelGGL(adam_init_kernel, dim3(1024), dim3(256), 0, st, scalars, adam_scalar_words(),
                       reinterpret_cast<uint4 *>(codes), code_bytes / 16);
}

void launch_adam_step(const AdamArgs &a, hipStream_t st) {
    AdamParams p;
    p.grad = a.grad; p.w = a.w; p.w_bf16 = (uint16_t *)a.w_bf16; p.m_q = a.m_q; p.v_q = a.v_q; p.scalars = a.scalars;
    p.n = a.n; p.b1 = a.beta1; p.b2 = a.beta2; p.omb1 = a.one_minus_beta1; p.omb2 = a.one_minus_beta2;
    p.c1 = a.c1; p.c2 = a.c2; p.lr = a.lr; p.eps = a.eps; p.wd = a.weight_decay; p.parity = a.step & 1; p.pow2 = a.pow2;
    // range pass: 16 elements per lane (16-byte code loads); update pass: 8 per lane measured faster
    constexpr int kRangeHalves = 2, kUpdateHalves = 1;
    // measured at 45 M elements: the read-only range pass is fastest with one trip per lane (57 us against 67
    // with 4096 looping workgroups), the update pass with 2048 looping workgroups (141 us against 160)
    auto grid = [&](int per_lane, size_t cap) {
        const size_t groups = ((size_t)a.n / per_lane + kAdamThreads - 1) / kAdamThreads;
        return (unsigned)(groups < cap ? groups : cap);
    };
    const unsigned grid_r = grid(8 * kRangeHalves, (size_t)1 << 20), grid_u = grid(8 * kUpdateHalves, 2048);
    // timing records (when enabled): tag 32 = range pass, 33 = update pass
    const double gbytes = a.grad_bf16 ? 2.0 : 4.0;       // algorithmic bytes per element: gradient + two codes; update: + w in/out, bf16 copy, codes out
    profile_before(32, st, (gbytes + 2.0) * (double)a.n);
    if (a.grad_bf16) hipLaunchKernelGGL((adam_range_kernel<true, kRangeHalves>), dim3(grid_r), dim3(kAdamThreads), 0, st, p);
    else hipLaunchKernelGGL((adam_range_kernel<false, kRangeHalves>), dim3(grid_r), dim3(kAdamThreads), 0, st, p);
    profile_after(st);
    profile_before(33, st, (gbytes + 2.0 + 4.0 + 4.0 + (a.w_bf16 ? 2.0 : 0.0) + 2.0) * (double)a.n);
    if (a.grad_bf16) hipLaunchKernelGGL((adam_update_kernel<true, kUpdateHalves>), dim3(grid_u), dim3(kAdamThreads), 0, st, p);
    else hipLaunchKernelGGL((adam_update_kernel<false, kUpdateHalves>), dim3(grid_u), dim3(kAdamThreads), 0, st, p);
    profile_after(st);
}

}  // namespace ssg
