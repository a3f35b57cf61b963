// FP8 MFMA GEMMs of the backward pass for gfx950: the single-launch forms (dH with the SwiGLU derivative fused,
// the input gradient as a sum of two products) and the grouped launches, in which the tiles of several
// independent GEMMs share one grid.
//
// Why grouped: every GEMM of the block at the Llama2-7B shape has a tile count that is not a multiple of the 256
// compute units (688 tiles = 2.69 rounds), so each launch ends with a partly empty round; and within one GEMM all
// workgroups reach their epilogue at the same moment, so its global traffic (U, G reads and dU, dG writes of dH;
// 64 MB of fp32 per round of a weight gradient) hits memory in bursts while the matrix cores idle.  In a grouped
// launch the workgroups of different GEMMs alternate in dispatch order: the partly empty round is paid once per
// group, and tiles of different lengths drift out of phase, so one workgroup's epilogue traffic runs under the
// others' main loops.
#include <cstdlib>

#include "ssg_gemm_tile.h"

namespace ssg {

// Up to three GEMMs in one grid.  Workgroups are dealt in sets of 8 consecutive ids (one per XCD, so that
// vblock % 8 stays the XCD inside each GEMM and map_tile's per-XCD patches survive); sets[i] = number of such
// sets GEMM i needs.
struct GroupParams {
    GemmParams p[3];
    int sets[3];
    int sequential;      // 1: the GEMMs follow one another in dispatch order; 0: their sets alternate in proportion
};

// The set index G of a workgroup -> (is it GEMM `first`'s, index among that GEMM's sets) for two GEMMs with s0 and s1
// sets interleaved in proportion: GEMM 0 owns set G iff floor((G+1) s0 / (s0+s1)) > floor(G s0 / (s0+s1)).
__device__ __forceinline__ bool interleave2(int G, int s0, int s1, int sequential, int &local) {
    if (sequential) {
        if (G < s0) { local = G; return true; }
        local = G - s0;
        return false;
    }
    const int c0 = (int)(((long long)G * s0) / (s0 + s1)), c0n = (int)(((long long)(G + 1) * s0) / (s0 + s1));
    if (c0n > c0) { local = c0; return true; }
    local = G - c0;
    return false;
}

// dH (with the SwiGLU derivative; EPI = EPI_SWIGLU_BWD or EPI_SWIGLU_BWD_Q) and dW3, interleaved: both read dY^.
template <int EPI>
__global__ void __launch_bounds__(kThreads) gemm_group_dh_dw3_kernel(GroupParams g) {
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kUnits * kUnitBytes];
    const int G = (int)(blockIdx.x >> 3), x = (int)(blockIdx.x & 7);
    int local;
    if (interleave2(G, g.sets[0], g.sets[1], g.sequential, local)) {
        const int vb = local * 8 + x;
        if (vb < g.p[0].tiles_m * g.p[0].tiles_n) gemm_tile<EPI, kE5M2, 0, 1>(g.p[0], vb, smem);
    } else {
        const int vb = local * 8 + x;
        if (vb < g.p[1].tiles_m * g.p[1].tiles_n) gemm_tile<EPI_STORE, kE5M2, 0, 2>(g.p[1], vb, smem);
    }
}

// dX (sum of two products in one tile: the long tiles, dealt first) followed by dW1 and dW2, interleaved.
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
    int local;
    const bool first = interleave2(G, g.sets[1], g.sets[2], g.sequential, local);
    const GemmParams &p = first ? g.p[1] : g.p[2];
    const int vb = local * 8 + x;
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
        return (a.epilogue == EPI_SWIGLU_BWD || a.epilogue == EPI_SWIGLU_BWD_Q) && wgrad(*list[1]);
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
    static const int seq = [] { const char *e = std::getenv("SSG_GEMM_GROUPING"); return (e && e[0] == '2') ? 1 : 0; }();
    g.sequential = seq;
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
    if (a.epilogue == EPI_SWIGLU_BWD) hipLaunchKernelGGL((gemm_kernel<EPI_SWIGLU_BWD, kE5M2, 0, 1>), grid, dim3(kThreads), 0, st, p);
    else if (a.epilogue == EPI_SWIGLU_BWD_Q) hipLaunchKernelGGL((gemm_kernel<EPI_SWIGLU_BWD_Q, kE5M2, 0, 1>), grid, dim3(kThreads), 0, st, p);
    else if (a.part == 1) hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE5M2, 1, 1>), grid, dim3(kThreads), 0, st, p);
    else if (a.part == 2) hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE5M2, 2, 1>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE5M2, 3, 1>), grid, dim3(kThreads), 0, st, p);
    profile_after(st);
    return true;
}

}  // namespace ssg
