// FP8 MFMA GEMM for gfx950 with the block's fused epilogues.
//
//   C[m,n] = sum_k A[m,k] * B[n,k]      A [M,K], B [N,K] FP8 codes, K contiguous
//
// (the inner products of Eq. 2, the last linear layer of the display after it,
// and their gradient contractions).  fp32 accumulation on the matrix cores with
// v_mfma_f32_32x32x64_f8f6f4, the only FP8 form that reaches the full rate on
// this chip; its per-operand format selectors take E4M3 or E5M2.
//
// Workgroup: 512 threads = 8 waves as 2 (M) x 4 (N); tile 256 x 256 x 128; each
// wave owns 128 x 64 outputs = 4 x 2 MFMA blocks (128 accumulator registers).
// Tiles are streamed global -> LDS with 16-byte direct-to-LDS loads (no
// staging registers), two LDS stages of 64 KB, one barrier per K step.  A row
// of a tile is 128 bytes; the eight 16-byte chunks of a row are stored XOR-
// permuted by the row index so that the 32 lanes that read the same logical
// chunk of 32 different rows spread over all banks.
//
// Epilogues:
//   STORE       C = acc / (sa*sb) [* col_scale[n]], bf16 or fp32; optional second
//               K segment with its own scales (input gradient: two products summed).
//   SWIGLU      B tile = 128 rows of W1 and the same 128 rows of W2, so a wave
//               holds u and g of the same (t,i): stores bf16 U, G and folds
//               max_t |u * Swish(g)| into the per-channel maxima (Section 4.4).
//   SWIGLU_BWD  acc -> dH (times the channel factor s_i), reads bf16 U, G, stores
//               bf16 dU, dG and folds their amax.
#include "ssg_device.h"
#include "ssg_internal.h"

namespace ssg {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef __attribute__((address_space(1))) const void *global_void_ptr;

#ifndef SSG_GEMM_EXPERIMENT
#define SSG_GEMM_EXPERIMENT 0   /* timing experiments only (results are wrong): 1 = no DMA after the prologue, 2 = no LDS reads */
#endif
constexpr int BM = 256, BN = 256, BK = 128;
constexpr int kThreads = 512;
constexpr int kUnitBytes = BM * BK;               // one operand tile of one K step: 256 rows x 128 B = 32 KB
constexpr int kUnits = 5;                         // ring of operand tiles in LDS: all 160 KB

__device__ uint4 g_zero_chunk = {0u, 0u, 0u, 0u}; // source of the zero fill of a ragged K tail

struct GemmParams {
    const uint8_t *A, *B, *A2, *B2;
    int64_t M, N, K, K2;
    const float *sa, *sb, *sa2, *sb2, *col_scale;
    void *C, *C2;
    const uint16_t *U, *G;
    uint32_t *camax_bits, *amax_bits, *amax_bits2;
    int c_f32;
    int tiles_m, tiles_n;
};

// An LDS row holds the 128 bytes (eight 16-byte chunks, one full cache line) of one matrix row for one
// K step.  Two rows fill the 256-byte bank period, so rows r, r+2, r+4, ... would collide when 16
// lanes read the same chunk of 16 consecutive rows; XOR-ing the chunk index with (r >> 1) & 7
// spreads 16 consecutive rows over the sixteen 16-byte bank groups.
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// Direct-to-LDS loads are issued through inline assembly: the compiler would otherwise wait for
// ALL outstanding LDS-DMA loads before every ds_read (it cannot tell the two LDS stages apart),
// which serialises memory latency with the MFMA work.  M0 carries the wave-uniform LDS
// destination; lane i lands at M0 + 16*i.  The vmcnt waits are placed by hand in the main loop.
__device__ __forceinline__ void dma16(const uint8_t *g, uint32_t lds_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_addr), "v"(g) : "memory");
#else
    (void)g; (void)lds_addr;
#endif
}

// Same with a wave-uniform 64-bit base in SGPRs and a 32-bit per-lane byte offset: no VALU work per issue.
__device__ __forceinline__ void dma16_s(const uint8_t *base_uniform, uint32_t lane_off, uint32_t lds_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base_uniform) : "memory");
#else
    (void)base_uniform; (void)lane_off; (void)lds_addr;
#endif
}

template <int AFMT>
__device__ __forceinline__ v16f mfma(const v8i &a, const v8i &b, const v16f &c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, AFMT, 0, 0, 0, 0, 0);
}

__device__ __forceinline__ float inv_scale_product(const float *sa, const float *sb) {
    float p = 1.0f;
    if (sa) p = *sa;
    if (sb) p = __fmul_rn(p, *sb);
    return __fdiv_rn(1.0f, p);
}

template <int EPI, int AFMT, bool TWO_SEG>
__global__ void __launch_bounds__(kThreads) gemm_kernel(GemmParams p) {
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kUnits * kUnitBytes];

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;   // wave index is uniform: keep it scalar
    const int wm = w >> 2, wn = w & 3;

    // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with
    // its own L2, so give every XCD a contiguous range of a tile order in which any 32 consecutive
    // tiles (one per CU of the XCD) form a 4 x 8 patch: 12 operand tiles fetched for 32 computed.
    int tile_m, tile_n;
    {
        const int total = p.tiles_m * p.tiles_n;
        const int per_xcd = (total + 7) / 8;
        int t = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
        if ((total & 7) != 0) {
            // ranges are uneven: fall back to the identity when the remapped id would leave the grid
            const int full = total & ~7;
            t = (int)blockIdx.x < full ? (int)(blockIdx.x & 7) * (full >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
        }
        constexpr int kGroupM = 4;
        const int group_tiles = kGroupM * p.tiles_n;
        const int gidx = t / group_tiles;
        const int first_m = gidx * kGroupM;
        const int gsize = (p.tiles_m - first_m) < kGroupM ? (p.tiles_m - first_m) : kGroupM;
        const int in_group = t - gidx * group_tiles;
        tile_m = first_m + in_group % gsize;
        tile_n = in_group / gsize;
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    // SWIGLU: a tile covers 128 channels (128 rows of W1 + the same 128 rows of W2)
    const int64_t n0 = (int64_t)tile_n * (EPI == EPI_SWIGLU ? BN / 2 : BN);

    // ---- global -> LDS slots of this lane.  One DMA instruction fills 1 KB = 8 rows x 128 B (eight
    // full cache lines); an operand tile ("unit") is 32 instructions, 4 per wave.  Lane l lands at
    // row (l >> 3), position (l & 7) of its 8-row group and fetches the logical chunk that the
    // swizzle puts there: group j of wave w starts at row (4w+j)*8, so swz(row) = (4*(j&1) + (l>>4)) & 7.
    const int lrow = l >> 3;
    const int chunk_even = (l & 7) ^ swz(lrow), chunk_odd = (l & 7) ^ swz(8 + lrow);
    uint32_t a_lane[4], b_lane[4];             // byte offset of this lane's chunk in K step 0, per DMA slot
    const uint8_t *b_src = p.B;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = (w * 4 + j) * 8 + lrow;
        const int ck = ((j & 1) ? chunk_odd : chunk_even) * 16;
        int64_t gm = m0 + row;
        gm = gm < p.M ? gm : p.M - 1;
        a_lane[j] = (uint32_t)(gm * p.K) + ck;
        int64_t gn;
        if (EPI == EPI_SWIGLU) gn = n0 + (row & 127);
        else gn = n0 + row;
        gn = gn < p.N ? gn : p.N - 1;
        b_lane[j] = (uint32_t)(gn * p.K) + ck;
    }
    if (EPI == EPI_SWIGLU && w >= 4) b_src = p.B2;      // waves 4..7 fill tile rows 128..255
    const uint32_t lds_w = (uint32_t)(w * 4) * 1024u;   // + j*1024 + unit offset

    // ---- LDS -> register fragment offsets (same pattern for A and B): for K half kh lane l holds
    // row l%32 and logical chunks kh*4 + 2*(l/32) and the next one
    uint32_t frag_off[2][2];
#pragma unroll
    for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int e = 0; e < 2; ++e)
            frag_off[kh][e] = (uint32_t)((l & 31) * BK + (((kh * 4 + (l >> 5) * 2 + e) ^ swz(l & 31)) << 4));
    const uint32_t a_frag_base = (uint32_t)(wm * 128) * BK;
    uint32_t b_frag_base[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
        b_frag_base[nb] = (uint32_t)(EPI == EPI_SWIGLU ? nb * 128 + wn * 32 : wn * 64 + nb * 32) * BK;

    v16f acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.0f;

    // One K loop over both products when there are two (input gradient): steps 0..nk1-1 come from
    // (A, B), steps nk1.. from (A2, B2); the accumulators are rescaled by alpha1/alpha2 where the
    // second product starts, so a single dequantization by alpha2 at the end serves both.
    constexpr int n_seg = TWO_SEG ? 2 : 1;
    const int nk1 = (int)((p.K + BK - 1) / BK);
    const int nk = nk1 + (TWO_SEG ? (int)((p.K2 + BK - 1) / BK) : 0);
    {
        const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void_ptr)smem;
        uint32_t a2_lane[4] = {0, 0, 0, 0}, b2_lane[4] = {0, 0, 0, 0};
        if (TWO_SEG) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {          // row pitch of the second pair is K2
                const int row = (w * 4 + j) * 8 + lrow;
                const int ck = ((j & 1) ? chunk_odd : chunk_even) * 16;
                int64_t gm = m0 + row; gm = gm < p.M ? gm : p.M - 1;
                int64_t gn = n0 + row; gn = gn < p.N ? gn : p.N - 1;
                a2_lane[j] = (uint32_t)(gm * p.K2) + ck;
                b2_lane[j] = (uint32_t)(gn * p.K2) + ck;
            }
        }
        // The LDS ring holds 5 operand tiles ("units") of 32 KB: unit u is the A tile (u even) or B tile
        // (u odd) of K step u/2 and lives in ring slot u % 5.  While step k is being read (2 units)
        // three more are in flight.  Unit u = DMA of 256 rows x 128 B: 4 instructions per wave, the
        // source is a wave-uniform base (SGPRs) plus this lane's 32-bit offset.  In the last,
        // partial K step the chunks past K come from a 16-byte zero word instead.
        auto issue_unit = [&](int u) {
            const int k = u >> 1;
            if (k >= nk) return;                   // nothing left to fetch (the waits below account for it)
            if ((SSG_GEMM_EXPERIMENT & 1) && u >= kUnits) return;
            const uint32_t dst = smem_base + (uint32_t)(u % kUnits) * kUnitBytes + lds_w;
            const bool second = TWO_SEG && k >= nk1;
            const int64_t kbase = (int64_t)(second ? k - nk1 : k) * BK;
            const int64_t Kseg = second ? p.K2 : p.K;
            const bool is_b = (u & 1) != 0;
            const uint8_t *base = is_b ? (second ? p.B2 : b_src) : (second ? p.A2 : p.A);
            if (kbase + BK <= Kseg) {              // whole step in range (uniform branch)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t off = is_b ? (second ? b2_lane[j] : b_lane[j]) : (second ? a2_lane[j] : a_lane[j]);
                    dma16_s(base + kbase, off, dst + j * 1024);
                }
            } else {
                const uint8_t *zero = reinterpret_cast<const uint8_t *>(&g_zero_chunk);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t off = is_b ? (second ? b2_lane[j] : b_lane[j]) : (second ? a2_lane[j] : a_lane[j]);
                    const int ck = ((j & 1) ? chunk_odd : chunk_even) * 16;
                    const bool k_ok = kbase + ck < Kseg;       // K is a multiple of 16: a chunk is all in or all out
                    dma16(k_ok ? base + kbase + off : zero, dst + j * 1024);
                }
            }
        };
        auto rescale_for_second_product = [&]() {
            const float r = __fdiv_rn(inv_scale_product(p.sa, p.sb), inv_scale_product(p.sa2, p.sb2));
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[mb][nb][i] *= r;
        };

        // Schedule.  The two waves that share a SIMD (w and w+4) run one slot out of phase: while
        // one feeds the matrix core from registers (8 MFMAs on one 64-wide K half, ~512 cycles) the
        // other pulls its next fragments out of LDS and issues DMA.  Slots are separated by
        // workgroup barriers.  Group 0 (waves 0-3) runs K step k in slots 4k..4k+3 as load(kh0)
        // compute(kh0) load(kh1) compute(kh1); group 1 (waves 4-7) does the same one slot later.
        // Units 2k+3 and 2k+4 reuse the ring slots of step k-1, which group 1 read last in slot
        // 4k-1; each wave issues its share of them in its own load(kh0) slot of step k (4k / 4k+1).
        // Before the barrier that ends slot 4k+3 every wave waits until all but its newest 4 DMA
        // instructions have landed, i.e. until units 2k+2 and 2k+3 (step k+1) are complete.
        v8i fa[4], fb[2];
        auto load_frags = [&](int k, int kh) {
            if (SSG_GEMM_EXPERIMENT & 2) return;
            const uint8_t *sA = smem + ((2 * k) % kUnits) * kUnitBytes + a_frag_base;
            const uint8_t *sB = smem + ((2 * k + 1) % kUnits) * kUnitBytes;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                const uint4 lo = *reinterpret_cast<const uint4 *>(sA + mb * 32 * BK + frag_off[kh][0]);
                const uint4 hi = *reinterpret_cast<const uint4 *>(sA + mb * 32 * BK + frag_off[kh][1]);
                fa[mb] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const uint4 lo = *reinterpret_cast<const uint4 *>(sB + b_frag_base[nb] + frag_off[kh][0]);
                const uint4 hi = *reinterpret_cast<const uint4 *>(sB + b_frag_base[nb] + frag_off[kh][1]);
                fb[nb] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            }
        };
        auto compute = [&]() {
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) acc[mb][nb] = mfma<AFMT>(fa[mb], fb[nb], acc[mb][nb]);
        };
        // A first-half load slot has two jobs on different pipes: 12 LDS reads and 8 DMA instructions.
        // Half of the waves do them in one order and half in the other, so both pipes are busy at once.
        auto load_and_issue = [&](int k) {
            if (wn & 1) {
                load_frags(k, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (k >= 1) { issue_unit(2 * k + 3); issue_unit(2 * k + 4); }
            } else {
                if (k >= 1) { issue_unit(2 * k + 3); issue_unit(2 * k + 4); }
                __builtin_amdgcn_sched_barrier(0);
                load_frags(k, 0);
            }
        };
        auto wait_next_step = [&](int k) {         // units 2k+2, 2k+3 landed; unit 2k+4 may still be in flight
            if (2 * k + 4 < 2 * nk) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        };
        auto slot_end = [&]() {                    // every wave executes the same number of these
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        };

#pragma unroll
        for (int u = 0; u < kUnits; ++u) issue_unit(u);
        if (nk >= 3) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");       // units 0 and 1 have landed
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        slot_end();
        if (wm == 0) {
            for (int k = 0; k < nk; ++k) {
                load_and_issue(k);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                slot_end();
                if (TWO_SEG && k == nk1) rescale_for_second_product();
                compute();
                slot_end();
                load_frags(k, 1);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                slot_end();
                compute();
                wait_next_step(k);
                slot_end();
            }
            slot_end();
        } else {
            for (int k = 0; k < nk; ++k) {
                if (k > 0) compute();              // second half of step k-1
                slot_end();
                load_and_issue(k);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                slot_end();
                if (TWO_SEG && k == nk1) rescale_for_second_product();
                compute();
                slot_end();
                load_frags(k, 1);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                wait_next_step(k);
                slot_end();
            }
            compute();
            slot_end();
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- epilogue.  Block (mb, nb), register i, lane l holds
    //      row = wm*128 + mb*32 + (i/4)*8 + (l/32)*4 + i%4,  column = colbase(nb) + l%32,
    // i.e. one column and scattered rows per lane.  Each wave re-lays its accumulators out through
    // a private LDS patch, one 32 x 64 slab (mb) at a time, so that a lane then owns 8 consecutive
    // columns of one row and every global access is a 16-byte vector on a full 64/128-byte run.
    __syncthreads();                                   // main-loop LDS is no longer read by anyone
    constexpr int kPitch = 72;                         // floats; 4 rows apart lands on the other 32 banks
    float *stg = reinterpret_cast<float *>(smem) + w * (32 * kPitch);
    const int lcol = l & 31;
    const int lrow4 = (l >> 5) * 4;
    auto stage_slab = [&](int mb) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                stg[((i >> 2) * 8 + lrow4 + (i & 3)) * kPitch + nb * 32 + lcol] = acc[mb][nb][i];
    };
    auto load8 = [&](int r, int c, float (&v)[8]) {
        const float4 a = *reinterpret_cast<const float4 *>(stg + r * kPitch + c);
        const float4 b = *reinterpret_cast<const float4 *>(stg + r * kPitch + c + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    };
    auto pack_bf16x8 = [&](const float (&v)[8]) {
        uint32_t q[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) q[k] = f32_to_bf16_bits(v[2 * k]) | (f32_to_bf16_bits(v[2 * k + 1]) << 16);
        return make_uint4(q[0], q[1], q[2], q[3]);
    };
    auto unpack_bf16x8 = [&](const uint4 q, float (&v)[8]) {
        const uint32_t w4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = __uint_as_float(w4[k] << 16);
            v[2 * k + 1] = __uint_as_float(w4[k] & 0xffff0000u);
        }
    };

    if (EPI == EPI_STORE || EPI == EPI_SWIGLU_BWD) {
        // lane -> (row r of the slab in 4 passes of 8 rows, 8 columns c8 of the wave's 64)
        const int c8 = (l & 7) * 8;
        const int64_t col = n0 + wn * 64 + c8;
        const bool col_ok = col < p.N;                 // N is a multiple of 16: the 8 columns are all in or all out
        const float alpha = (EPI == EPI_STORE && n_seg == 2) ? inv_scale_product(p.sa2, p.sb2)
                                                             : inv_scale_product(p.sa, p.sb);
        float f[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) f[k] = alpha;
        if (p.col_scale && col_ok) {
#pragma unroll
            for (int k = 0; k < 8; ++k) f[k] = __fmul_rn(alpha, p.col_scale[col + k]);
        }
        uint32_t du_max = 0, dg_max = 0;
        // SWIGLU_BWD: the stored U, G of slab mb+1 are fetched while slab mb is processed, so that
        // their memory latency is not paid once per pass
        uint4 ru[2][4], rg[2][4];
        auto fetch_ug = [&](int mb, int buf) {
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int64_t row = m0 + wm * 128 + mb * 32 + pass * 8 + (l >> 3);
                if (col_ok && row < p.M) {
                    const size_t at = (size_t)row * (size_t)p.N + (size_t)col;
                    ru[buf][pass] = *reinterpret_cast<const uint4 *>(p.U + at);
                    rg[buf][pass] = *reinterpret_cast<const uint4 *>(p.G + at);
                }
            }
        };
        if (EPI == EPI_SWIGLU_BWD) fetch_ug(0, 0);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
            if (EPI == EPI_SWIGLU_BWD && mb + 1 < 4) fetch_ug(mb + 1, (mb + 1) & 1);
            stage_slab(mb);
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int r = pass * 8 + (l >> 3);
                const int64_t row = m0 + wm * 128 + mb * 32 + r;
                float v[8];
                load8(r, c8, v);
                if (!col_ok || row >= p.M) continue;
                const size_t at = (size_t)row * (size_t)p.N + (size_t)col;
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = __fmul_rn(v[k], f[k]);
                if (EPI == EPI_STORE) {
                    if (p.c_f32) {
                        float *out = reinterpret_cast<float *>(p.C) + at;
                        *reinterpret_cast<float4 *>(out) = make_float4(v[0], v[1], v[2], v[3]);
                        *reinterpret_cast<float4 *>(out + 4) = make_float4(v[4], v[5], v[6], v[7]);
                    } else {
                        *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(p.C) + at) = pack_bf16x8(v);
                    }
                } else {
                    float u[8], g[8], du[8], dg[8];
                    unpack_bf16x8(ru[mb & 1][pass], u);
                    unpack_bf16x8(rg[mb & 1][pass], g);
#pragma unroll
                    for (int k = 0; k < 8; ++k) swiglu_grad_f32(u[k], g[k], v[k], du[k], dg[k]);
                    const uint4 qu = pack_bf16x8(du), qg = pack_bf16x8(dg);
                    *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(p.C) + at) = qu;
                    *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(p.C2) + at) = qg;
                    // amax of the stored bf16 values: compare the 15-bit magnitudes (NaN -> 0)
                    const uint32_t wu[4] = {qu.x, qu.y, qu.z, qu.w}, wg[4] = {qg.x, qg.y, qg.z, qg.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        uint32_t a0 = wu[k] & 0x7fffu, a1 = (wu[k] >> 16) & 0x7fffu;
                        uint32_t b0 = wg[k] & 0x7fffu, b1 = (wg[k] >> 16) & 0x7fffu;
                        a0 = a0 > 0x7f80u ? 0u : a0; a1 = a1 > 0x7f80u ? 0u : a1;
                        b0 = b0 > 0x7f80u ? 0u : b0; b1 = b1 > 0x7f80u ? 0u : b1;
                        a0 = a0 > a1 ? a0 : a1; b0 = b0 > b1 ? b0 : b1;
                        du_max = du_max > a0 ? du_max : a0;
                        dg_max = dg_max > b0 ? dg_max : b0;
                    }
                }
            }
        }
        if (EPI == EPI_SWIGLU_BWD) {
            // one atomic pair per workgroup: same-address atomics serialise in L2
            du_max = wave_max_u32(du_max);
            dg_max = wave_max_u32(dg_max);
            uint32_t *red = reinterpret_cast<uint32_t *>(smem + 8 * 32 * kPitch * 4);   // past the staging patches
            if (l == 0) { red[2 * w] = du_max; red[2 * w + 1] = dg_max; }
            __syncthreads();
            if (tid < 2) {
                uint32_t m = 0;
#pragma unroll
                for (int k = 0; k < 8; ++k) m = m > red[2 * k + tid] ? m : red[2 * k + tid];
                uint32_t *dst = tid == 0 ? p.amax_bits : p.amax_bits2;
                if (m) atomicMax(dst + (blockIdx.x % kAmaxSlots) * kAmaxSlotStride, m << 16);
            }
        }
    } else {   // EPI_SWIGLU: slab columns 0..31 are u, 32..63 are g of the same 32 channels
        const int c8 = (l & 3) * 8;
        const int64_t col = n0 + wn * 32 + c8;
        const bool col_ok = col < p.N;
        const float alpha_u = inv_scale_product(p.sa, p.sb);
        const float alpha_g = inv_scale_product(p.sa, p.sb2);
        uint32_t hmax[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
            stage_slab(mb);
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const int r = pass * 16 + (l >> 2);
                const int64_t row = m0 + wm * 128 + mb * 32 + r;
                float u[8], g[8];
                load8(r, c8, u);
                load8(r, 32 + c8, g);
                if (!col_ok || row >= p.M) continue;
                const size_t at = (size_t)row * (size_t)p.N + (size_t)col;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    u[k] = __fmul_rn(u[k], alpha_u);
                    g[k] = __fmul_rn(g[k], alpha_g);
                }
                const uint4 qu = pack_bf16x8(u), qg = pack_bf16x8(g);
                *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(p.C) + at) = qu;
                *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(p.C2) + at) = qg;
                unpack_bf16x8(qu, u);                  // h is formed from the stored (rounded) values
                unpack_bf16x8(qg, g);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t hb = abs_bits_ignore_nan(swiglu_f32(u[k], g[k]));
                    hmax[k] = hmax[k] > hb ? hmax[k] : hb;
                }
            }
        }
        // lanes with equal (l & 3) hold the same 8 channels: fold over the 16 row lanes
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int off = 4; off < 64; off <<= 1) {
                const uint32_t o = (uint32_t)__shfl_xor((int)hmax[k], off, 64);
                hmax[k] = hmax[k] > o ? hmax[k] : o;
            }
        if (l < 4 && col_ok) {
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (hmax[k]) atomicMax(&p.camax_bits[col + k], hmax[k]);
        }
    }
}

template <int EPI>
static void launch_epi(const GemmParams &p, int a_fmt, unsigned blocks, hipStream_t st) {
    if (EPI == EPI_STORE && p.A2) {        // two K segments: only the E5M2 x E4M3 input-gradient product uses it
        if (a_fmt == kE4M3)
            hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE4M3, true>), dim3(blocks), dim3(kThreads), 0, st, p);
        else
            hipLaunchKernelGGL((gemm_kernel<EPI_STORE, kE5M2, true>), dim3(blocks), dim3(kThreads), 0, st, p);
        return;
    }
    if (a_fmt == kE4M3)
        hipLaunchKernelGGL((gemm_kernel<EPI, kE4M3, false>), dim3(blocks), dim3(kThreads), 0, st, p);
    else
        hipLaunchKernelGGL((gemm_kernel<EPI, kE5M2, false>), dim3(blocks), dim3(kThreads), 0, st, p);
}

void launch_gemm(const GemmArgs &a, hipStream_t st) {
    GemmParams p;
    p.A = a.A; p.B = a.B; p.A2 = a.A2; p.B2 = a.B2;
    p.M = a.M; p.N = a.N; p.K = a.K; p.K2 = a.K2;
    p.sa = a.sa; p.sb = a.sb; p.sa2 = a.sa2; p.sb2 = a.sb2; p.col_scale = a.col_scale;
    p.C = a.C; p.C2 = a.C2;
    p.U = (const uint16_t *)a.U; p.G = (const uint16_t *)a.G;
    p.camax_bits = a.camax_bits; p.amax_bits = a.amax_bits; p.amax_bits2 = a.amax_bits2;
    p.c_f32 = a.c_f32;
    p.tiles_m = (int)((a.M + BM - 1) / BM);
    const int n_per_tile = a.epilogue == EPI_SWIGLU ? BN / 2 : BN;
    p.tiles_n = (int)((a.N + n_per_tile - 1) / n_per_tile);
    const unsigned blocks = (unsigned)p.tiles_m * (unsigned)p.tiles_n;
    profile_before(2 * a.epilogue + a.a_fmt + (a.epilogue == EPI_STORE && a.A2 ? 8 : 0), st);
    switch (a.epilogue) {
        case EPI_STORE: launch_epi<EPI_STORE>(p, a.a_fmt, blocks, st); break;
        case EPI_SWIGLU: launch_epi<EPI_SWIGLU>(p, a.a_fmt, blocks, st); break;
        default: launch_epi<EPI_SWIGLU_BWD>(p, a.a_fmt, blocks, st); break;
    }
    profile_after(st);
}

}  // namespace ssg
