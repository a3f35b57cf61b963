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
#include <algorithm>
#include <functional>
#include <vector>

#include "ssg_gemm_tile.h"

namespace ssg {

// Up to four GEMMs in one grid, one after the other in dispatch order.  Workgroups are dealt in sets of 8
// consecutive ids (one per XCD, so that vblock % 8 stays the XCD inside each GEMM and map_tile's per-XCD patches
// survive); member i runs sets [first[i], first[i] + sets[i]) of its GEMM -- a GEMM may be split between two
// launches at a set boundary.
struct GroupParams {
    GemmParams p[4];
    int sets[4];
    int first[4];
};

// dH (with the SwiGLU derivative; EPI = EPI_SWIGLU_BWD or EPI_SWIGLU_BWD_Q), then the first part of dW3: both read dY^.
template <int EPI>
__global__ void __launch_bounds__(kThreads) gemm_group_dh_dw3_kernel(GroupParams g) {
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kUnits * kUnitBytes];
    const int G = (int)(blockIdx.x >> 3), x = (int)(blockIdx.x & 7);
    if (G < g.sets[0]) {
        const int vb = G * 8 + x;
        if (vb < g.p[0].tiles_m * g.p[0].tiles_n) gemm_tile<EPI, kE5M2, 0, 1>(g.p[0], vb, smem);
    } else {
        const int vb = (G - g.sets[0] + g.first[1]) * 8 + x;
        if (vb < g.p[1].tiles_m * g.p[1].tiles_n) gemm_tile<EPI_STORE, kE5M2, 0, 2>(g.p[1], vb, smem);
    }
}

// dX (sum of two products in one tile: the long tiles, dealt first), then dW1, dW2 and the rest of dW3.
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
    int m = 1;
    if (G >= g.sets[1]) { G -= g.sets[1]; m = 2; if (G >= g.sets[2]) { G -= g.sets[2]; m = 3; } }
    const GemmParams &p = g.p[m];
    const int vb = (G + g.first[m]) * 8 + x;
    if (vb < p.tiles_m * p.tiles_n) gemm_tile<EPI_STORE, kE5M2, 0, 2>(p, vb, smem);
}

static int sets_of(const GemmParams &p) { return (p.tiles_m * p.tiles_n + 7) / 8; }
int gemm_tile_sets(const GemmArgs &a) { return sets_of(make_gemm_params(a)); }

static bool is_wgrad(const GemmArgs &a) { return a.epilogue == EPI_STORE && a.part == 0 && a.layout == 2 && a.a_fmt == kE5M2; }

bool gemm_group_ok(const GemmArgs *const *list, int n) {
    if (n < 2 || n > 4) return false;
    for (int i = 0; i < n; ++i)
        if (!list[i] || !gemm_args_ok(*list[i])) return false;
    if (n == 2) {
        const GemmArgs &a = *list[0];
        return (a.epilogue == EPI_SWIGLU_BWD || a.epilogue == EPI_SWIGLU_BWD_Q) && a.a_fmt == kE5M2 && is_wgrad(*list[1]);
    }
    for (int i = 1; i < n; ++i)
        if (!is_wgrad(*list[i])) return false;
    return list[0]->epilogue == EPI_STORE && list[0]->part == 3;
}

// ---- where to split a weight gradient between the two grouped launches of the backward ------------------------
// Workgroups are dispatched in order to whichever compute unit is free, and a tile's time is known well enough
// from its K steps and its epilogue, so the end of a launch can be predicted by replaying that dispatch.  A launch
// whose last tiles start a round of their own pays a whole tile time for them; moving sets of the weight gradient
// from the first launch to the second (or back) shifts work between the two launches' last rounds.
static double tile_cost(const GemmArgs &a) {
    const GemmParams p = make_gemm_params(a);
    // microseconds, from per-workgroup time stamps at the Llama2-7B shape with all compute units busy: 1.33 per K
    // step (1.45 in the long tiles of the one-launch sum, which all run at once), 2.5 before the first step, and the
    // epilogue: 33 with the SwiGLU derivative (42 when it also casts), 10 for an fp32 store, 6 for bf16
    const double ksteps = (double)((p.K + BK - 1) / BK) * (a.part == 3 ? 2.0 : 1.0);
    double epilogue = a.c_f32 ? 10.0 : 6.0;
    if (a.epilogue == EPI_SWIGLU_BWD) epilogue = 33.0;
    if (a.epilogue == EPI_SWIGLU_BWD_Q) epilogue = 42.0;
    return 2.5 + (a.part == 3 ? 1.45 : 1.33) * ksteps + epilogue;
}

static double replay_dispatch(const double *cost, const int *tiles, int n, int units, std::vector<double> &free_at) {
    // free_at: a min-heap of the times at which the compute units become free
    free_at.assign((size_t)units, 0.0);
    double end = 0.0;
    for (int i = 0; i < n; ++i)
        for (int t = 0; t < tiles[i]; ++t) {
            std::pop_heap(free_at.begin(), free_at.end(), std::greater<double>());
            const double done = free_at.back() + cost[i];
            free_at.back() = done;
            std::push_heap(free_at.begin(), free_at.end(), std::greater<double>());
            end = done > end ? done : end;
        }
    return end;
}

int gemm_group_split_sets(const GemmArgs &dh, const GemmArgs &dw_split, const GemmArgs *const *second, int n_second,
                          int units) {
    const int all = gemm_tile_sets(dw_split);
    if (units <= 0 || n_second < 1 || n_second > 3) return all;
    const GemmParams ph = make_gemm_params(dh), pw = make_gemm_params(dw_split);
    const int tiles_w = pw.tiles_m * pw.tiles_n;
    double cost_b[4]; int tiles_b[4];
    for (int i = 0; i < n_second; ++i) {
        const GemmParams p = make_gemm_params(*second[i]);
        cost_b[i] = tile_cost(*second[i]); tiles_b[i] = p.tiles_m * p.tiles_n;
    }
    cost_b[n_second] = tile_cost(dw_split);
    const double cost_a[2] = {tile_cost(dh), tile_cost(dw_split)};
    std::vector<double> heap;
    // the predicted time is a step function of the split.  Of the longest run of equally good splits take a point a
    // quarter of the run below its upper end: measured, the second launch behaves like a fluid (its tiles have
    // drifted out of step, so every set moved there costs its share of time) while the first shows the predicted
    // step, so the best split moves as few sets as make the step, with a margin for tile times that differ a little
    // from the estimates
    std::vector<double> t((size_t)all + 1);
    double best = 0.0;
    for (int s = 0; s <= all; ++s) {
        const int in_a = s * 8 < tiles_w ? s * 8 : tiles_w;
        const int ta[2] = {ph.tiles_m * ph.tiles_n, in_a};
        tiles_b[n_second] = tiles_w - in_a;
        t[(size_t)s] = replay_dispatch(cost_a, ta, 2, units, heap) + replay_dispatch(cost_b, tiles_b, n_second + 1, units, heap);
        if (s == 0 || t[(size_t)s] < best) best = t[(size_t)s];
    }
    if (t[(size_t)all] <= best + 1e-9) return all;             // nothing to gain: dW3 stays whole in the first launch
    int best_lo = all, best_len = 0;
    for (int s = 0; s <= all;) {
        if (t[(size_t)s] > best + 1e-9) { ++s; continue; }
        int e = s;
        while (e + 1 <= all && t[(size_t)(e + 1)] <= best + 1e-9) ++e;
        if (e - s + 1 >= best_len) { best_len = e - s + 1; best_lo = s; }     // of equal runs, the one that moves least
        s = e + 1;
    }
    return best_lo + (best_len - 1) - (best_len - 1) / 4;
}

bool launch_gemm_group(const GemmArgs *const *list, int n, int split_sets, hipStream_t st) {
    if (!gemm_group_ok(list, n)) return false;
    GroupParams g;
    int total = 0;
    double flops = 0.0;
    for (int i = 0; i < 4; ++i) {
        g.p[i] = make_gemm_params(*list[i < n ? i : 0]);
        g.sets[i] = i < n ? sets_of(g.p[i]) : 0;
        g.first[i] = 0;
    }
    // the split member is the last one of either group: the first launch runs its sets [0, split), the second the rest
    if (split_sets >= 0 && (n == 2 || n == 4)) {
        const int all = g.sets[n - 1];
        const int cut = split_sets < all ? split_sets : all;
        if (n == 2) g.sets[1] = cut;
        else { g.first[n - 1] = cut; g.sets[n - 1] = all - cut; }
    }
    // The fp32 weight gradients of the second launch go out through non-temporal stores: nothing reads them before
    // the optimizer, and kept out of the caches they leave in place what the passes after this launch read (measured
    // at the Llama2-7B shape: -10 us per step, in the launches that follow, not in this one).  In the first launch,
    // beside dH's epilogue traffic, the same stores cost 3-7 us: left as they are.
    if (n >= 3)
        for (int i = 1; i < n; ++i) g.p[i].nt_store = 1;
    for (int i = 0; i < n; ++i) {
        // flops of the tiles this launch runs (a last set may be partly beyond the GEMM's tile count)
        const int tiles = g.p[i].tiles_m * g.p[i].tiles_n;
        int hi = (g.first[i] + g.sets[i]) * 8, lo = g.first[i] * 8;
        hi = hi < tiles ? hi : tiles; lo = lo < tiles ? lo : tiles;
        flops += gemm_flops(*list[i]) * (double)(hi - lo) / (double)tiles;
        total += g.sets[i];
    }
    if (total == 0) return true;
    const dim3 grid((unsigned)total * 8u);
    profile_before(n == 2 ? 16 : 17, st, flops);
    if (n >= 3) hipLaunchKernelGGL(gemm_group_dx_dw_kernel, grid, dim3(kThreads), 0, st, g);
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
    profile_before(gemm_profile_tag(a), st, gemm_flops(a));
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
