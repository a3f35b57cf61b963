// FP8 MFMA GEMMs for gfx950, one GEMM per launch: the plain store forms of every operand layout (the public
// contraction entry points; y of the block) and the two forward forms with the fused SwiGLU epilogues.
// The backward forms and the grouped launches are instantiated in ssg_gemm_bwd.hip.
#include "ssg_col_range.h"
#include "ssg_gemm_tile.h"

namespace ssg {

// The gate/up GEMM with an independent streaming pass in its grid.  1376 tiles on 256 compute units are 5.4
// rounds: during the last one 160 units would idle.  The workgroups after the last tile take the per-channel range
// of w3 (Section 4.4; it depends on no result of this GEMM and is needed only after it), so that pass costs no time
// of its own.  A workgroup of this kernel owns a whole compute unit (registers, LDS), hence 16 loads in flight per lane.
struct ColRangeParams {
    const uint16_t *src;
    int64_t rows, cols;
    uint32_t *camax_bits;
    int blocks_x;
};
__global__ void __launch_bounds__(kThreads) gemm_swiglu_col_range_kernel(GemmParams p, ColRangeParams r) {
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kUnits * kUnitBytes];
    const int tiles = p.tiles_m * p.tiles_n;
    if ((int)blockIdx.x < tiles) {
        gemm_tile<EPI_SWIGLU, kE4M3, 0, 0>(p, (int)blockIdx.x, smem);
    } else {
        const int b = (int)blockIdx.x - tiles;
        col_range_bf16_block<16>(r.src, r.rows, r.cols, r.camax_bits, b % r.blocks_x, b / r.blocks_x,
                                 reinterpret_cast<uint32_t *>(smem));
    }
}

bool gemm_args_ok(const GemmArgs &a) {
    if (a.epilogue < EPI_STORE || a.epilogue > EPI_SWIGLU_BWD_Q) return false;
    if (!a.A || !a.B || !a.C || a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
    if (a.a_fmt != kE4M3 && a.a_fmt != kE5M2 && a.a_fmt != kBF16) return false;
    // bf16 operands: the two forms the unquantized last layer needs, K-contiguous operands only
    if (a.a_fmt == kBF16 && (a.layout != 0 || a.part != 0 || (a.epilogue != EPI_STORE && a.epilogue != EPI_SWIGLU_BWD))) return false;
    const bool dual = a.epilogue == EPI_SWIGLU || a.epilogue == EPI_SWIGLU_Q;
    if (dual && (!a.B2 || a.a_fmt != kE4M3 || a.layout != 0)) return false;
    if (a.epilogue == EPI_SWIGLU && (!a.C2 || !a.camax_bits)) return false;
    if (a.tail_src && (a.epilogue != EPI_SWIGLU || !a.tail_camax_bits || a.tail_rows <= 0 || a.tail_cols <= 0 ||
                       a.tail_cols % 8 != 0 || (reinterpret_cast<uintptr_t>(a.tail_src) & 15u)))
        return false;
    if (a.part != 0 && a.epilogue != EPI_STORE) return false;
    if (a.layout < 0 || a.layout > 2) return false;
    const bool bwd = a.epilogue == EPI_SWIGLU_BWD || a.epilogue == EPI_SWIGLU_BWD_Q;
    // the backward forms are built for the block's own use: gradient operand E5M2, weight operand K-major
    if (bwd && a.a_fmt != kBF16 && (a.layout != 1 || a.a_fmt != kE5M2)) return false;
    if (a.epilogue == EPI_SWIGLU_BWD_Q && (!a.q_scale || !a.q_scale2 || !a.q_scale_out || !a.q_scale_out2)) return false;
    if (a.part < 0 || a.part > 3) return false;
    if (a.part != 0 && (a.layout != 1 || a.a_fmt != kE5M2)) return false;
    if ((a.part == 2) != (a.add != nullptr)) return false;
    if (a.part == 1 && !a.c_f32) return false;
    if ((a.part == 3) != (a.A_ph2 != nullptr) || (a.part == 3 && (!a.B_ph2 || !a.sa || !a.sb || !a.sa_ph2 || !a.sb_ph2))) return false;
    if (a.part == 3 && !gemm_sum_in_one_launch_ok(a.N, a.K)) return false;
    if ((a.keep_u != nullptr) != (a.keep_g != nullptr) || (a.keep_u && a.epilogue != EPI_SWIGLU_BWD_Q)) return false;
    if (bwd && (!a.U || !a.G || !a.C2 || !a.amax_bits || !a.amax_bits2)) return false;
    return true;
}

// The one-launch form of a sum of two products has no general loop body: whole K steps (at least two) and whole
// tile columns of the K-major B operand only.
bool gemm_sum_in_one_launch_ok(int64_t N, int64_t K) { return K % BK == 0 && K >= 2 * BK && N % BN == 0; }

int gemm_profile_tag(const GemmArgs &a) {
    // 2 * epilogue + A format; the halves of a sum of two products run as two launches get 9 and 10, the sum in
    // one launch 11; the gate/up GEMM with the column range pass in its grid 18
    if (a.part) return 8 + a.part;
    if (a.tail_src) return 18;
    if (a.a_fmt == kBF16) return a.epilogue == EPI_STORE ? 20 : 21;
    return 2 * (a.epilogue == EPI_SWIGLU_BWD_Q ? (int)EPI_SWIGLU_BWD : a.epilogue) + a.a_fmt;
}

template <int EPI, int LAY>
static void launch_fmt(const GemmParams &p, int a_fmt, unsigned blocks, hipStream_t st) {
    if (a_fmt == kE4M3) hipLaunchKernelGGL((gemm_kernel<EPI, kE4M3, 0, LAY>), dim3(blocks), dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((gemm_kernel<EPI, kE5M2, 0, LAY>), dim3(blocks), dim3(kThreads), 0, st, p);
}

bool launch_gemm(const GemmArgs &a, hipStream_t st) {
    if (!gemm_args_ok(a)) return false;
    if (a.part != 0 || a.epilogue == EPI_SWIGLU_BWD || a.epilogue == EPI_SWIGLU_BWD_Q) return launch_gemm_bwd(a, st);
    const GemmParams p = make_gemm_params(a);
    const unsigned blocks = (unsigned)p.tiles_m * (unsigned)p.tiles_n;
    profile_before(gemm_profile_tag(a), st, gemm_flops(a));
    switch (a.epilogue) {
        case EPI_STORE:
            if (a.a_fmt == kBF16) hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kBF16, 0, 0>), dim3(blocks), dim3(kThreads), 0, st, p);
            else if (a.layout == 2) launch_fmt<EPI_STORE, 2>(p, a.a_fmt, blocks, st);
            else if (a.layout == 1) launch_fmt<EPI_STORE, 1>(p, a.a_fmt, blocks, st);
            else launch_fmt<EPI_STORE, 0>(p, a.a_fmt, blocks, st);
            break;
        case EPI_SWIGLU:
            if (a.tail_src) {
                ColRangeParams r{static_cast<const uint16_t *>(a.tail_src), a.tail_rows, a.tail_cols, a.tail_camax_bits,
                                 col_range_blocks_x(a.tail_cols)};
                const unsigned extra = (unsigned)(r.blocks_x * col_range_blocks_y(a.tail_rows));
                hipLaunchKernelGGL(gemm_swiglu_col_range_kernel, dim3(blocks + extra), dim3(kThreads), 0, st, p, r);
            } else {
                hipLaunchKernelGGL((gemm_kernel<EPI_SWIGLU, kE4M3, 0, 0>), dim3(blocks), dim3(kThreads), 0, st, p);
            }
            break;
        default:   // EPI_SWIGLU_Q
            hipLaunchKernelGGL((gemm_kernel<EPI_SWIGLU_Q, kE4M3, 0, 0>), dim3(blocks), dim3(kThreads), 0, st, p);
            break;
    }
    profile_after(st);
    return true;
}

}  // namespace ssg
