// Diagnostic: the rate the matrix cores sustain on given operand bytes, with no memory traffic.
//
// The published dense FP8 rate assumes the full shader clock.  Under a dense MFMA load the clock
// follows the power the data draws: operands of constant bytes run at the full rate, operands of
// random bytes measurably below it.  This kernel keeps 16 accumulator blocks (256 registers) per
// wave, one wave per SIMD -- the register shape of the 4-wave GEMM -- and issues nothing but
// v_mfma_f32_32x32x64_f8f6f4, so its time is the ceiling any GEMM on that data can approach.
#include "ssg_internal.h"

namespace ssg {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 256, kProbeBlocks = 256, kProbeFrags = 4;

__global__ void __launch_bounds__(kProbeThreads) mfma_rate_kernel(const int *operands, float *sink, int iters) {
    v8i a[kProbeFrags], b[kProbeFrags];
#pragma unroll
    for (int f = 0; f < kProbeFrags; ++f)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[f][i] = operands[(threadIdx.x * kProbeFrags + f) * 16 + i];
            b[f][i] = operands[(threadIdx.x * kProbeFrags + f) * 16 + 8 + i];
        }
    v16f acc[kProbeFrags * kProbeFrags];
#pragma unroll
    for (int j = 0; j < kProbeFrags * kProbeFrags; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kProbeFrags * kProbeFrags; ++j)
            acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[j / kProbeFrags], b[j % kProbeFrags], acc[j],
                                                                     0, 0, 0, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < kProbeFrags * kProbeFrags; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    sink[blockIdx.x * kProbeThreads + threadIdx.x] = s;
}


double mfma_rate_flops(int iters) {
    return (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * (kProbeFrags * kProbeFrags) * 2.0 * 32 * 32 * 64;
}
size_t mfma_rate_operand_bytes() { return (size_t)kProbeThreads * kProbeFrags * 16 * sizeof(int); }     // 64 KiB
size_t mfma_rate_sink_bytes() { return (size_t)kProbeBlocks * kProbeThreads * sizeof(float); }          // 256 KiB
void launch_mfma_rate(const void *operands, void *sink, int iters, hipStream_t st) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, st, (const int *)operands,
                       (float *)sink, iters);
}

}  // namespace ssg
