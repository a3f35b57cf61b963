// FP8 MFMA GEMMs of the backward pass for gfx950: the single-launch forms (dH with the SwiGLU derivative fused,
// the input gradient as a sum of two products) and the grouped launches, in which the tiles of several
// independent GEMMs share one grid.
//
// Why grouped: every GEMM of the block at the Llama2-7B shape has a tile count that is not a multiple of the 256
// compute units (688 tiles = 2.69 rounds), so each launch ends with a partly empty round; and within one GEMM all
// workgroups reach their epilogue at the same moment, so its global traffic (U, G reads and dU, dG writes of dH;
// 64 MB of fp32 per round of a weight gradient) hits memory in bursts while the matrix cores idle.  In a grouped
// launch the workgroups of the next GEMM follow those of the previous one in dispatch order, so its first tiles
// start on the compute units the previous GEMM's last round leaves idle.  (Alternating the members' workgroups
// instead -- so that tiles of different lengths drift out of phase -- measured 10 % slower for {dH, dW3}: two
// working sets share each XCD's L2 and every member's patch of concurrent tiles is half as large.)
#include "ssg_gemm_tile.h"

namespace ssg {

// Up to three GEMMs in one grid, one after the other in dispatch order.  Workgroups are dealt in sets of 8
// consecutive ids (one per XCD, so that vblock % 8 stays the XCD inside each GEMM and map_tile's per-XCD patches
// survive); sets[i] = number of such sets GEMM i needs.
struct GroupParams {
    GemmParams p[3];
    int sets[3];
};

// dH (with the SwiGLU derivative; EPI = EPI_SWIGLU_BWD or EPI_SWIGLU_BWD_Q), then dW3: both read dY^.
template <int EPI>
__global__ void __launch_bounds__(kThreads) gemm_group_dh_dw3_kernel(GroupParams g) {
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kUnits * kUnitBytes];
    const int G = (int)(blockIdx.x >> 3), x = (int)(blockIdx.x & 7);
    if (G < g.sets[0]) {
        const int vb = G * 8 + x;
        if (vb < g.p[0].tiles_m * g.p[0].tiles_n) gemm_tile<EPI, kE5M2, 0, 1>(g.p[0], vb, smem);
    } else {
        const int vb = (G - g.sets[0]) * 8 + x;
        if (vb < g.p[1].tiles_m * g.p[1].tiles_n) gemm_tile<EPI_STORE, kE5M2, 0, 2>(g.p[1], vb, smem);
    }
}

// dX (sum of two products in one tile: the long tiles, dealt first), then dW1, then dW2.
__global__ void __launch_bounds__(kThreads) gemm_group_dx_dw_kernel(GroupParams g) {
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kUnits * kUnitBytes];
    int G = (int)(blockIdx.x >> 3);
    const int x = (int)(blockIdx.x & 7);
    if (G < g.sets[0]) {
        const int vb = G * 8 + x;
        if (vb < g.p[0].tiles_m * g.p[0].tiles_n) gemm_tile<EPI_STORE, kE5M2, 3, 1>(g.p[0], vb, smem);
        return;
    }
    G -= g.sets[0];
    const bool first = G < g.sets[1];
    const GemmParams &p = first ? g.p[1] : g.p[2];
    const int vb = (first ? G : G - g.sets[1]) * 8 + x;
    if (vb < p.tiles_m * p.tiles_n) gemm_tile<EPI_STORE, kE5M2, 0, 2>(p, vb, smem);
}

static int sets_of(const GemmParams &p) { return (p.tiles_m * p.tiles_n + 7) / 8; }

bool gemm_group_ok(const GemmArgs *const *list, int n) {
    if (n < 2 || n > 3) return false;
    for (int i = 0; i < n; ++i)
        if (!list[i] || !gemm_args_ok(*list[i])) return false;
    auto wgrad = [](const GemmArgs &a) { return a.epilogue == EPI_STORE && a.part == 0 && a.layout == 2 && a.a_fmt == kE5M2; };
    if (n == 2) {
        const GemmArgs &a = *list[0];
        return (a.epilogue == EPI_SWIGLU_BWD || a.epilogue == EPI_SWIGLU_BWD_Q) && a.a_fmt == kE5M2 && wgrad(*list[1]);
    }
    return list[0]->epilogue == EPI_STORE && list[0]->part == 3 && wgrad(*list[1]) && wgrad(*list[2]);
}

bool launch_gemm_group(const GemmArgs *const *list, int n, hipStream_t st) {
    if (!gemm_group_ok(list, n)) return false;
    GroupParams g;
    int total = 0;
    for (int i = 0; i < 3; ++i) {
        g.p[i] = make_gemm_params(*list[i < n ? i : 0]);
        g.sets[i] = i < n ? sets_of(g.p[i]) : 0;
        total += g.sets[i];
    }
    const dim3 grid((unsigned)total * 8u);
    profile_before(n == 2 ? 16 : 17, st);
    if (n == 3) hipLaunchKernelGGL(gemm_group_dx_dw_kernel, grid, dim3(kThreads), 0, st, g);
    else if (list[0]->epilogue == EPI_SWIGLU_BWD)
        hipLaunchKernelGGL(gemm_group_dh_dw3_kernel<EPI_SWIGLU_BWD>, grid, dim3(kThreads), 0, st, g);
    else
        hipLaunchKernelGGL(gemm_group_dh_dw3_kernel<EPI_SWIGLU_BWD_Q>, grid, dim3(kThreads), 0, st, g);
    profile_after(st);
    return true;
}

// The backward forms launched on their own (a.part != 0, or one of the SwiGLU-backward epilogues); the
// argument set has passed gemm_args_ok.
bool launch_gemm_bwd(const GemmArgs &a, hipStream_t st) {
    const GemmParams p = make_gemm_params(a);
    const dim3 grid((unsigned)p.tiles_m * (unsigned)p.tiles_n);
    profile_before(gemm_profile_tag(a), st);
    if (a.epilogue == EPI_SWIGLU_BWD && a.a_fmt == kBF16)
        hipLaunchKernelGGL((gemm_kernel<EPI_SWIGLU_BWD, kBF16, 0, 0>), grid, dim3(kThreads), 0, st, p);
    else if (a.epilogue == EPI_SWIGLU_BWD) hipLaunchKernelGGL((gemm_kernel<EPI_SWIGLU_BWD, kE5M2, 0, 1>), grid, dim3(kThreads), 0, st, p);
    else if (a.epilogue == EPI_SWIGLU_BWD_Q) hipLaunchKernelGGL((gemm_kernel<EPI_SWIGLU_BWD_Q, kE5M2, 0, 1>), grid, dim3(kThreads), 0, st, p);
    else if (a.part == 1) hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE5M2, 1, 1>), grid, dim3(kThreads), 0, st, p);
    else if (a.part == 2) hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE5M2, 2, 1>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE5M2, 3, 1>), grid, dim3(kThreads), 0, st, p);
    profile_after(st);
    return true;
}

}  // namespace ssg
