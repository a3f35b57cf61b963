// Diagnostic: the rate the matrix cores sustain on given operand bytes, with no memory traffic.
//
// The published dense FP8 rate assumes the full shader clock.  Under a dense MFMA load the clock
// follows the power the data draws: operands of constant bytes run at the full rate, operands of
// random bytes measurably below it.  This kernel keeps 16 accumulator blocks (256 registers) per
// wave, one wave per SIMD -- the register shape of the 4-wave GEMM -- and issues nothing but
// v_mfma_f32_32x32x64_f8f6f4, so its time is the ceiling any GEMM on that data can approach.
//
// Built into a library of its own (libssg_probe.so) that only the benchmark loads: it is a
// measurement aid, not part of the block's interface.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

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


}  // namespace

// Launches the loop: `iters` passes of 16 MFMAs per wave on the operand fragments in the first 64 KiB of
// `workspace` (device; the caller fills them); a 256 KiB checksum is written after them, so `workspace_bytes`
// must be at least 320 KiB.  *flops (host, may be NULL) receives the flop count of the launch; the caller
// times it.  Returns 0, or -1 on a bad argument / -4 when the launch reported an error.
extern "C" int ssg_probe_mfma_rate(void *workspace, size_t workspace_bytes, int iters, double *flops, void *stream) {
    const size_t operand_bytes = (size_t)kProbeThreads * kProbeFrags * 16 * sizeof(int);        // 64 KiB
    const size_t sink_bytes = (size_t)kProbeBlocks * kProbeThreads * sizeof(float);             // 256 KiB
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < operand_bytes + sink_bytes ||
        iters <= 0 || iters > (1 << 24))
        return -1;
    if (flops)
        *flops = (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * (kProbeFrags * kProbeFrags) * 2.0 * 32 * 32 * 64;
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const int *>(workspace),
                       reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + operand_bytes), iters);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
