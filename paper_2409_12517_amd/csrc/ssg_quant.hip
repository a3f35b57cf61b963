// HBM-bound passes of the FP8 Smooth-SwiGLU block for gfx950:
//   amax (Section 2: per-tensor range), the scale + saturating cast Q of Eq. 2
//   with an optional transposed copy, per-channel maxima and factors of
//   Section 4.4, and the SwiGLU product of Section 4.1 for tests.
// All loads and stores are 16-byte (8-byte for row-major code stores) vectors
// along the contiguous index; reductions use one atomic max per workgroup or
// per column on the float's bit pattern (|x| orders like an unsigned integer).
#include <type_traits>

#include "ssg_col_range.h"
#include "ssg_device.h"
#include "ssg_internal.h"

namespace ssg {

// ------------------------------------------------------------------ fill
__global__ void __launch_bounds__(256) fill_u32_kernel(uint32_t *p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}
void launch_fill_u32(uint32_t *p, size_t n, uint32_t value, hipStream_t st) {
    if (n == 0) return;
    profile_before(kTagSmall, st, 4.0 * (double)n);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, value);
    profile_after(st);
}

// Zero selected scalar slots (bit i of mask -> slot i) and up to two vectors in one launch.
__global__ void __launch_bounds__(256)
reset_kernel(uint32_t *scalars, uint32_t mask, uint32_t *v1, size_t n1, uint32_t *v2, size_t n2) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < 32 && ((mask >> i) & 1u)) scalars[i] = 0u;
    if (i < n1) v1[i] = 0u;
    if (i < n2) v2[i] = 0u;
}
void launch_reset(uint32_t *scalars, uint32_t mask, uint32_t *v1, size_t n1, uint32_t *v2, size_t n2, hipStream_t st) {
    size_t n = n1 > n2 ? n1 : n2;
    if (n < 32) n = 32;
    profile_before(kTagSmall, st, 4.0 * (double)(n1 + n2));
    hipLaunchKernelGGL(reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, scalars, mask, v1, n1, v2, n2);
    profile_after(st);
}

// ------------------------------------------------------------------ loaders
// Each loader returns 8 consecutive elements of one row as fp32.
struct LoadBf16 {
    const uint16_t *p;
    // (a streaming read: the non-temporal hint keeps the source from displacing what later kernels read again)
    __device__ __forceinline__ uint4 load8_raw(size_t off) const {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + off));
        return make_uint4(q[0], q[1], q[2], q[3]);
    }
    static __device__ __forceinline__ void widen(const uint4 q, float (&v)[8]) {
        uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ __forceinline__ void load8(size_t off, float (&v)[8]) const {
        uint4 q = load8_raw(off);
        uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
struct LoadF32 {
    const float *p;
    __device__ __forceinline__ void load8(size_t off, float (&v)[8]) const {
        float4 a = *reinterpret_cast<const float4 *>(p + off);
        float4 b = *reinterpret_cast<const float4 *>(p + off + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};
struct LoadSwiglu {          // h = u * Swish(g) from stored bf16 U, G
    const uint16_t *u, *g;
    __device__ __forceinline__ void load8(size_t off, float (&v)[8]) const {
        // plain loads: U and G were just written by the GEMM and are read again by the backward pass
        float uu[8], gg[8];
        LoadBf16::widen(*reinterpret_cast<const uint4 *>(u + off), uu);
        LoadBf16::widen(*reinterpret_cast<const uint4 *>(g + off), gg);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = swiglu_f32(uu[i], gg[i]);
    }
};

// ------------------------------------------------------------------ amax
template <class Loader>
__global__ void __launch_bounds__(256) amax_kernel(Loader ld, size_t n8, uint32_t *amax_bits, int slots) {
    uint32_t m = 0;
    // work is cut into units of 2048 chunks (32 KB of bf16): 8 independent 16-byte loads per lane,
    // 4 KB apart; workgroup b takes units b, b + gridDim.x, ... (the launch picks gridDim.x so that
    // every workgroup gets the same number of units)
    const size_t units = (n8 + 2047) / 2048;
    for (size_t unit = blockIdx.x; unit < units; unit += gridDim.x) {
        const size_t i = unit * 2048 + threadIdx.x;
        float v[8][8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t j = i + u * 256;
            if (j < n8) ld.load8(j * 8, v[u]);
            else {
#pragma unroll
                for (int k = 0; k < 8; ++k) v[u][k] = 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                uint32_t b = abs_bits_ignore_nan(v[u][k]);
                m = m > b ? m : b;
            }
    }
    m = wave_max_u32(m);
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t r = part[0];
        for (int w = 1; w < 4; ++w) r = r > part[w] ? r : part[w];
        if (r) atomicMax(amax_bits + (blockIdx.x % slots) * kAmaxSlotStride, r);
    }
}

// bf16 source: the range is taken on the raw 16-bit patterns, two per operation (biased_abs_pk, ssg_col_range.h).
// A pure streaming read: every workgroup walks contiguous runs of 4 x 256 16-byte pieces (4 independent loads per
// lane), grid-stride.  Measured on a 90 MB tensor: 13 us (6.9 TB/s) against 27-41 us for the generic kernel above
// (which widens every element to fp32 and walks 32 KB units); more loads per lane or larger workgroups are slower.
constexpr int kAmaxBf16Loads = 4;
struct AmaxBatch {
    const ssg_u32x4 *src[3];
    size_t n16[3];
    uint32_t *amax_bits[3];
};
// (up to three tensors per launch, blockIdx.y picks one: the ranges of x, W1, W2 share a launch)
__global__ void __launch_bounds__(256)
amax_bf16_kernel(const AmaxBatch batch, int slots) {
    const ssg_u32x4 *__restrict__ src = batch.src[blockIdx.y];
    const size_t n16 = batch.n16[blockIdx.y];
    uint32_t *amax_bits = batch.amax_bits[blockIdx.y];
    ssg_i16x2 m = {0x7f, 0x7f};
    const size_t run = (size_t)kAmaxBf16Loads * 256;
    for (size_t base = (size_t)blockIdx.x * run; base < n16; base += (size_t)gridDim.x * run) {
        ssg_u32x4 v[kAmaxBf16Loads];
#pragma unroll
        for (int u = 0; u < kAmaxBf16Loads; ++u) {
            const size_t j = base + (size_t)u * 256 + threadIdx.x;
            v[u] = j < n16 ? __builtin_nontemporal_load(src + j) : ssg_u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kAmaxBf16Loads; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) m = __builtin_elementwise_max(m, biased_abs_pk(v[u][k]));
    }
    uint32_t r = wave_max_u32(unbias_max_pk(m));
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) r = r > part[w] ? r : part[w];
        r = r > part[0] ? r : part[0];
        if (r) atomicMax(amax_bits + (blockIdx.x % slots) * kAmaxSlotStride, r);
    }
}

void launch_amax_batch(const void *const *src, const size_t *n, uint32_t *const *amax_bits, int count, hipStream_t st) {
    AmaxBatch batch;
    size_t largest = 0;
    double bytes = 0.0;
    int m = 0;
    for (int i = 0; i < count && m < 3; ++i) {
        if (n[i] / 8 == 0) continue;
        batch.src[m] = (const ssg_u32x4 *)src[i]; batch.n16[m] = n[i] / 8; batch.amax_bits[m] = amax_bits[i];
        largest = batch.n16[m] > largest ? batch.n16[m] : largest;
        bytes += 2.0 * (double)n[i];
        ++m;
    }
    if (m == 0) return;
    for (int i = m; i < 3; ++i) { batch.src[i] = batch.src[0]; batch.n16[i] = 0; batch.amax_bits[i] = batch.amax_bits[0]; }
    const size_t runs = (largest + kAmaxBf16Loads * 256 - 1) / (kAmaxBf16Loads * 256);
    const unsigned blocks = (unsigned)(runs < 1024 ? runs : 1024);
    profile_before(kTagAmax, st, bytes);
    hipLaunchKernelGGL(amax_bf16_kernel, dim3(blocks, (unsigned)m), dim3(256), 0, st, batch, kAmaxSlots);
    profile_after(st);
}

void launch_amax(const void *src, SrcKind kind, size_t n, uint32_t *amax_bits, int slots, hipStream_t st) {
    size_t n8 = n / 8;      // n is a multiple of 16 at every call site (rows, cols multiples of 16)
    if (n8 == 0) return;
    profile_before(kTagAmax, st, (kind == SRC_BF16 ? 2.0 : 4.0) * (double)n);
    if (kind == SRC_BF16) {
        AmaxBatch batch;
        for (int i = 0; i < 3; ++i) { batch.src[i] = (const ssg_u32x4 *)src; batch.n16[i] = n8; batch.amax_bits[i] = amax_bits; }
        const size_t runs = (n8 + kAmaxBf16Loads * 256 - 1) / (kAmaxBf16Loads * 256);
        const unsigned blocks = (unsigned)(runs < 1024 ? runs : 1024);
        hipLaunchKernelGGL(amax_bf16_kernel, dim3(blocks), dim3(256), 0, st, batch, slots);
    } else {
        const size_t units = (n8 + 2047) / 2048;
        const size_t cap = slots > 1 ? 2048 : 512;
        const size_t per_block = (units + cap - 1) / cap;               // units per workgroup, the same for all
        unsigned blocks = (unsigned)((units + per_block - 1) / per_block);
        hipLaunchKernelGGL(amax_kernel<LoadF32>, dim3(blocks), dim3(256), 0, st,
                           LoadF32{(const float *)src}, n8, amax_bits, slots);
    }
    profile_after(st);
}

// ------------------------------------------------------------------ cast
// One workgroup converts a 128 x 128 tile.  A thread owns two 4-row x 8-column
// blocks: it loads 8 elements from each of 4 rows, scales, casts, stores the
// 8 codes of each row (8 bytes, 16 lanes cover 128 contiguous bytes), and, if
// the transposed copy is wanted, transposes its 4x4 byte blocks in registers
// and parks them in LDS as [column][row] so that the copy is written in
// 16-byte pieces that are contiguous along the source's row index.
constexpr int kTile = 128;
constexpr int kTPitchWords = 33;     // LDS pitch of one transposed column, in 32-bit words

__device__ __forceinline__ void transpose4x4_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d,
                                                   uint32_t (&o)[4]) {
    uint32_t ab_lo = __builtin_amdgcn_perm(b, a, 0x05010400u);   // a0 b0 a1 b1
    uint32_t ab_hi = __builtin_amdgcn_perm(b, a, 0x07030602u);   // a2 b2 a3 b3
    uint32_t cd_lo = __builtin_amdgcn_perm(d, c, 0x05010400u);
    uint32_t cd_hi = __builtin_amdgcn_perm(d, c, 0x07030602u);
    o[0] = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x05040100u);     // a0 b0 c0 d0
    o[1] = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x07060302u);
}

// COUNT: also count, into counters[0] and counters[1], the elements whose scaled magnitude lies beyond the
// rounding interval of the largest finite value (only the clamp keeps them finite: overflow, Section 3) and
// the nonzero elements whose code is +-0 (underflow).
// Up to three tensors per launch (blockIdx.z picks the item; workgroups beyond an item's own tile grid leave at
// once): the casts of x, W1, W2 -- and of dU, dG -- share a launch, which saves the ramp-up and drain of two launches.
template <class Loader>
struct CastItem {
    Loader ld;
    int64_t rows, cols;
    const float *col_scale, *amax;
    int amax_slots;
    float *amax_out;
    const float *scale_in;
    float *scale_out;
    uint8_t *dst, *dst_t;
    uint32_t *record;
    unsigned long long *counters;
};
template <class Loader>
struct CastBatch {
    CastItem<Loader> item[3];
    int pow2;
};
// The work of one workgroup: tile (bx, by) of item `it`.
template <class Loader, int FMT, bool COLSCALE, bool TRANSPOSED, bool RECORD = false, bool COUNT = false>
__device__ __forceinline__ void cast_block(const CastItem<Loader> &it, const int pow2, const unsigned bx, const unsigned by) {
    const Loader ld = it.ld;
    const int64_t rows = it.rows, cols = it.cols;
    if ((int64_t)bx * kTile >= cols || (int64_t)by * kTile >= rows) return;
    const float *__restrict__ col_scale = it.col_scale;
    const float *__restrict__ amax = it.amax;
    const int amax_slots = it.amax_slots;
    float *__restrict__ amax_out = it.amax_out;
    const float *__restrict__ scale_in = it.scale_in;
    float *__restrict__ scale_out = it.scale_out;
    uint8_t *__restrict__ dst = it.dst, *__restrict__ dst_t = it.dst_t;
    uint32_t *__restrict__ record = it.record;
    unsigned long long *__restrict__ counters = it.counters;
    __shared__ uint32_t tile[TRANSPOSED ? kTile * kTPitchWords : 1];
    uint32_t n_sat = 0, n_flush = 0;

    float sigma = 1.0f;
    bool tensor_scale = false;
    if (scale_in) { sigma = *scale_in; tensor_scale = true; }
    else if (amax) {
        // maximum over the slots the producers folded into: lane i of every wave takes slot i
        // (kAmaxSlots = wave size), then a wave-wide maximum
        const uint32_t *ab = reinterpret_cast<const uint32_t *>(amax);
        const int lane = threadIdx.x & 63;
        uint32_t mbits = lane < amax_slots ? ab[lane * kAmaxSlotStride] : 0u;
        mbits = wave_max_u32(mbits);
        const float m = __uint_as_float(mbits);
        sigma = scale_from_amax(m, Fp8Traits<FMT>::fmax, pow2);
        tensor_scale = true;
        if (amax_out && bx == 0 && by == 0 && threadIdx.x == 0) *amax_out = m;
    }
    if (scale_out && bx == 0 && by == 0 && threadIdx.x == 0) *scale_out = sigma;

    const int64_t row0 = (int64_t)by * kTile;
    const int64_t col0 = (int64_t)bx * kTile;
    const int c8 = threadIdx.x & 15;       // which 8-column chunk
    const int r4 = threadIdx.x >> 4;       // which 4-row group (0..15) inside a 64-row half
    const int64_t col = col0 + c8 * 8;
    const bool col_ok = col < cols;

    float cs[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) cs[i] = 1.0f;
    if (COLSCALE && col_ok) {
        float4 a = *reinterpret_cast<const float4 *>(col_scale + col);
        float4 b = *reinterpret_cast<const float4 *>(col_scale + col + 4);
        cs[0] = a.x; cs[1] = a.y; cs[2] = a.z; cs[3] = a.w;
        cs[4] = b.x; cs[5] = b.y; cs[6] = b.z; cs[7] = b.w;
    }

    ssg_i16x2 seen2 = {0x7f, 0x7f};                     // RECORD: largest (|bf16 pattern| + 0x7f) this lane met, per half
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int lr = half * 64 + r4 * 4;             // local row of the 4-row group
        uint32_t lo[4] = {0, 0, 0, 0}, hi[4] = {0, 0, 0, 0};
        if (col_ok && row0 + lr < rows) {              // rows is a multiple of 16: the group is all in or all out
            // the four row loads of the group first: four requests in flight per lane (measured: one at a time is
            // 5-10 % slower, all eight of the lane at once is slower again)
            float v[4][8];
            if constexpr (RECORD) {
                // bf16 source: the range is taken on the raw 16-bit patterns, two per operation.  |x| + 0x7f is
                // below 0x8000 for every number and infinity and at or above it for NaN, so a signed 16-bit
                // maximum ignores NaN, as the range pass does.
                uint4 raw[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) raw[r] = ld.load8_raw((size_t)(row0 + lr + r) * (size_t)cols + (size_t)col);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t w4[4] = {raw[r].x, raw[r].y, raw[r].z, raw[r].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const ssg_i16x2 b = __builtin_bit_cast(ssg_i16x2, (w4[i] & 0x7fff7fffu) + 0x007f007fu);
                        seen2 = __builtin_elementwise_max(seen2, b);
                    }
                    LoadBf16::widen(raw[r], v[r]);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) ld.load8((size_t)(row0 + lr + r) * (size_t)cols + (size_t)col, v[r]);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const size_t off = (size_t)(row0 + lr + r) * (size_t)cols + (size_t)col;
                uint32_t nonzero = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (COUNT) nonzero |= (v[r][i] != 0.0f ? 1u : 0u) << i;
                    if (COLSCALE) v[r][i] = __fmul_rn(v[r][i], cs[i]);
                    if (tensor_scale) v[r][i] = __fmul_rn(v[r][i], sigma);
                    if (COUNT) n_sat += fabsf(v[r][i]) > Fp8Traits<FMT>::overflow_above ? 1u : 0u;
                }
                lo[r] = satcast_pk4<FMT>(v[r][0], v[r][1], v[r][2], v[r][3]);
                hi[r] = satcast_pk4<FMT>(v[r][4], v[r][5], v[r][6], v[r][7]);
                if (COUNT) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const uint32_t code = ((i < 4 ? lo[r] : hi[r]) >> (8 * (i & 3))) & 0x7fu;
                        n_flush += (code == 0u && ((nonzero >> i) & 1u)) ? 1u : 0u;
                    }
                }
                *reinterpret_cast<uint2 *>(dst + off) = make_uint2(lo[r], hi[r]);
            }
        }
        if (TRANSPOSED) {
            uint32_t t[4];
            transpose4x4_bytes(lo[0], lo[1], lo[2], lo[3], t);
#pragma unroll
            for (int j = 0; j < 4; ++j) tile[(c8 * 8 + j) * kTPitchWords + (lr >> 2)] = t[j];
            transpose4x4_bytes(hi[0], hi[1], hi[2], hi[3], t);
#pragma unroll
            for (int j = 0; j < 4; ++j) tile[(c8 * 8 + 4 + j) * kTPitchWords + (lr >> 2)] = t[j];
        }
    }
    if (RECORD) {
        // the range this pass saw, for the history of delayed scaling: one atomic per workgroup (atomics on
        // one address from many workgroups serialise, and across XCDs they are slow: one per wave cost 20 us
        // on a 45 M element tensor)
        __shared__ uint32_t wave_seen[4];
        const uint32_t lo16 = (uint32_t)(uint16_t)seen2[0] - 0x7fu, hi16 = (uint32_t)(uint16_t)seen2[1] - 0x7fu;
        uint32_t seen = (lo16 > hi16 ? lo16 : hi16) << 16;          // bf16 pattern -> fp32 pattern of the same number
        seen = wave_max_u32(seen);
        if ((threadIdx.x & 63) == 0) wave_seen[threadIdx.x >> 6] = seen;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t m = wave_seen[0];
#pragma unroll
            for (int k = 1; k < 4; ++k) m = m > wave_seen[k] ? m : wave_seen[k];
            if (m) atomicMax(record + ((by * gridDim.x + bx) % kAmaxSlots) * kAmaxSlotStride, m);
        }
    }
    if (COUNT) {
        // one atomic per workgroup and counter, and none for a zero count
        __shared__ uint32_t wave_counts[4][2];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            n_sat += (uint32_t)__shfl_xor((int)n_sat, off, 64);
            n_flush += (uint32_t)__shfl_xor((int)n_flush, off, 64);
        }
        if ((threadIdx.x & 63) == 0) { wave_counts[threadIdx.x >> 6][0] = n_sat; wave_counts[threadIdx.x >> 6][1] = n_flush; }
        __syncthreads();
        if (threadIdx.x < 2) {
            const uint32_t c = wave_counts[0][threadIdx.x] + wave_counts[1][threadIdx.x] + wave_counts[2][threadIdx.x] +
                               wave_counts[3][threadIdx.x];
            if (c) atomicAdd(counters + threadIdx.x, (unsigned long long)c);
        }
    }
    if (TRANSPOSED) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = threadIdx.x + 256 * j;
            const int c = q >> 3;                      // local column = row of the transposed copy
            const int rc = q & 7;                      // 16-row chunk
            if (col0 + c < cols && row0 + rc * 16 < rows) {
                const uint32_t *src = &tile[c * kTPitchWords + rc * 4];
                uint4 o = make_uint4(src[0], src[1], src[2], src[3]);
                *reinterpret_cast<uint4 *>(dst_t + (size_t)(col0 + c) * (size_t)rows + (size_t)(row0 + rc * 16)) = o;
            }
        }
    }
}

template <class Loader, int FMT, bool COLSCALE, bool TRANSPOSED, bool RECORD = false, bool COUNT = false>
__global__ void __launch_bounds__(256)
cast_kernel(const CastBatch<Loader> batch) {
    cast_block<Loader, FMT, COLSCALE, TRANSPOSED, RECORD, COUNT>(batch.item[blockIdx.z], batch.pow2, blockIdx.x, blockIdx.y);
}

// The two casts between the gate/up GEMM and the last GEMM of the Smooth-SwiGLU forward in one launch: h^ =
// cast(s_i h) from bf16 U, G (Eq. 2; blockIdx.z = 0) and w3~ = Q(s^-1 w3) (the display after Eq. 2; blockIdx.z = 1).
// Both depend only on the channel factors, neither on the other.
template <bool COUNT>
__global__ void __launch_bounds__(256)
cast_h_w3_kernel(const CastItem<LoadSwiglu> h, const CastItem<LoadBf16> w3, const int pow2) {
    if (blockIdx.z == 0) cast_block<LoadSwiglu, kE4M3, true, false, false, COUNT>(h, pow2, blockIdx.x, blockIdx.y);
    else cast_block<LoadBf16, kE4M3, true, false, false, false>(w3, pow2, blockIdx.x, blockIdx.y);
}

template <class Loader>
static CastItem<Loader> cast_item(const Loader &ld, const CastArgs &a) {
    return CastItem<Loader>{ld, a.rows, a.cols, a.col_scale, a.amax, a.amax_slots, a.amax_out, a.scale_in, a.scale_out,
                            a.dst, a.dst_t, a.record, a.counters};
}

// All items of a batch share the source kind, the format and the presence of every optional part (per-column
// factor, transposed copy, range record, counters): one kernel instantiation serves them.
static bool same_cast_form(const CastArgs &a, const CastArgs &b) {
    return a.kind == b.kind && a.fmt == b.fmt && a.pow2 == b.pow2 && (a.col_scale != nullptr) == (b.col_scale != nullptr) &&
           (a.dst_t != nullptr) == (b.dst_t != nullptr) && (a.record != nullptr) == (b.record != nullptr) &&
           (a.counters != nullptr) == (b.counters != nullptr);
}

template <class Loader, int FMT, class MakeLoader>
static void launch_cast_l(const CastArgs *list, int n, MakeLoader make, hipStream_t st) {
    const CastArgs &a = list[0];
    CastBatch<Loader> batch;
    int64_t rows = 0, cols = 0;
    for (int i = 0; i < 3; ++i) {
        const CastArgs &x = list[i < n ? i : 0];
        batch.item[i] = cast_item<Loader>(make(x), x);
        if (i < n) { rows = x.rows > rows ? x.rows : rows; cols = x.cols > cols ? x.cols : cols; }
    }
    batch.pow2 = a.pow2;
    dim3 grid((unsigned)((cols + kTile - 1) / kTile), (unsigned)((rows + kTile - 1) / kTile), (unsigned)n);
    const bool cs = a.col_scale != nullptr, tr = a.dst_t != nullptr;
#define SSG_CAST(...) hipLaunchKernelGGL((cast_kernel<Loader, FMT, __VA_ARGS__>), grid, dim3(256), 0, st, batch)
    if constexpr (std::is_same<Loader, LoadBf16>::value) {
        if (a.record && !cs) {
            if (tr) SSG_CAST(false, true, true);
            else SSG_CAST(false, false, true);
            return;
        }
    }
    if (a.counters && !tr) {
        if (cs) SSG_CAST(true, false, false, true);
        else SSG_CAST(false, false, false, true);
        return;
    }
    if (cs && tr) SSG_CAST(true, true);
    else if (cs) SSG_CAST(true, false);
    else if (tr) SSG_CAST(false, true);
    else SSG_CAST(false, false);
#undef SSG_CAST
}

template <int FMT>
static void launch_cast_f(const CastArgs *list, int n, hipStream_t st) {
    switch (list[0].kind) {
        case SRC_BF16:
            launch_cast_l<LoadBf16, FMT>(list, n, [](const CastArgs &x) { return LoadBf16{(const uint16_t *)x.src}; }, st);
            break;
        case SRC_F32:
            launch_cast_l<LoadF32, FMT>(list, n, [](const CastArgs &x) { return LoadF32{(const float *)x.src}; }, st);
            break;
        case SRC_SWIGLU:
            launch_cast_l<LoadSwiglu, FMT>(list, n, [](const CastArgs &x) {
                return LoadSwiglu{(const uint16_t *)x.src, (const uint16_t *)x.src2}; }, st);
            break;
    }
}

static double cast_bytes(const CastArgs &a) {
    // algorithmic bytes: the source once (bf16 2, fp32 4, bf16 U and G 4), one code per element (two with a transposed copy)
    return ((a.kind == SRC_BF16 ? 2.0 : 4.0) + (a.dst_t ? 2.0 : 1.0)) * (double)a.rows * (double)a.cols;
}

void launch_cast_batch(const CastArgs *list, int n, hipStream_t st) {
    // items that are empty or of another form than the first go on their own
    int m = 0;
    CastArgs same[3];
    for (int i = 0; i < n; ++i) {
        if (list[i].rows == 0 || list[i].cols == 0) continue;
        if (m < 3 && (m == 0 || same_cast_form(same[0], list[i]))) same[m++] = list[i];
        else launch_cast(list[i], st);
    }
    if (m == 0) return;
    double bytes = 0.0;
    for (int i = 0; i < m; ++i) bytes += cast_bytes(same[i]);
    const CastArgs &a = same[0];
    profile_before(a.kind == SRC_SWIGLU ? kTagCastSwiglu : a.col_scale ? kTagCastColscale : kTagCast, st, bytes);
    if (a.fmt == kE4M3) launch_cast_f<kE4M3>(same, m, st);
    else launch_cast_f<kE5M2>(same, m, st);
    profile_after(st);
}

void launch_cast(const CastArgs &a, hipStream_t st) { launch_cast_batch(&a, 1, st); }

bool cast_h_w3_ok(const CastArgs &h, const CastArgs &w3) {
    return h.kind == SRC_SWIGLU && w3.kind == SRC_BF16 && h.fmt == kE4M3 && w3.fmt == kE4M3 && h.col_scale && w3.col_scale &&
           !h.dst_t && !w3.dst_t && !h.record && !w3.record && !w3.counters && h.rows > 0 && w3.rows > 0 && h.cols > 0 &&
           w3.cols > 0;
}

void launch_cast_h_w3(const CastArgs &h, const CastArgs &w3, hipStream_t st) {
    if (!cast_h_w3_ok(h, w3)) {             // not the pair this launch is built for: one after the other
        launch_cast(h, st);
        launch_cast(w3, st);
        return;
    }
    const CastItem<LoadSwiglu> hi = cast_item<LoadSwiglu>(LoadSwiglu{(const uint16_t *)h.src, (const uint16_t *)h.src2}, h);
    const CastItem<LoadBf16> wi = cast_item<LoadBf16>(LoadBf16{(const uint16_t *)w3.src}, w3);
    const int64_t rows = h.rows > w3.rows ? h.rows : w3.rows, cols = h.cols > w3.cols ? h.cols : w3.cols;
    dim3 grid((unsigned)((cols + kTile - 1) / kTile), (unsigned)((rows + kTile - 1) / kTile), 2u);
    profile_before(kTagCastHW3, st, cast_bytes(h) + cast_bytes(w3));
    if (h.counters) hipLaunchKernelGGL(cast_h_w3_kernel<true>, grid, dim3(256), 0, st, hi, wi, w3.pow2);
    else hipLaunchKernelGGL(cast_h_w3_kernel<false>, grid, dim3(256), 0, st, hi, wi, w3.pow2);
    profile_after(st);
}

// ------------------------------------------------------------------ per-column amax
// Grid (cols/512, rows/128).  A wave reads 1 KB of a row per load; a lane keeps 8 running column
// maxima over its wave's share of the slab's rows; the four waves of a workgroup meet in LDS and
// one atomic per column goes to memory.
constexpr int kSlabRows = 128;

template <class Loader>
__global__ void __launch_bounds__(256)
col_amax_kernel(Loader ld, int64_t rows, int64_t cols, uint32_t *__restrict__ camax_bits) {
    __shared__ uint32_t cmax[kColTile];
    cmax[threadIdx.x] = 0;
    cmax[threadIdx.x + 256] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.x * kColTile + lane * 8;
    const int64_t row0 = (int64_t)blockIdx.y * kSlabRows;
    const int64_t row1 = row0 + kSlabRows < rows ? row0 + kSlabRows : rows;
    if (col < cols) {
        uint32_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int64_t r = row0 + w; r < row1; r += 16) {        // four independent row loads in flight per lane
            float v[4][8];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t rr = r + 4 * u;
                if (rr < row1) ld.load8((size_t)rr * (size_t)cols + (size_t)col, v[u]);
                else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[u][i] = 0.0f;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    uint32_t b = abs_bits_ignore_nan(v[u][i]);
                    m[i] = m[i] > b ? m[i] : b;
                }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (m[i]) atomicMax(&cmax[lane * 8 + i], m[i]);
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int t = threadIdx.x + 256 * h;
        const int64_t c = (int64_t)blockIdx.x * kColTile + t;
        if (c < cols && cmax[t]) atomicMax(&camax_bits[c], cmax[t]);
    }
}

// bf16 source: the workgroup's work is col_range_bf16_block (ssg_col_range.h), shared with the gate/up GEMM's grid.
__global__ void __launch_bounds__(256)
col_amax_bf16_kernel(const uint16_t *__restrict__ src, int64_t rows, int64_t cols, uint32_t *__restrict__ camax_bits) {
    __shared__ uint32_t cmax[kColTile];
    col_range_bf16_block<8>(src, rows, cols, camax_bits, (int)blockIdx.x, (int)blockIdx.y, cmax);
}

void launch_col_amax(const void *src, const void *src2, SrcKind kind, int64_t rows, int64_t cols,
                     uint32_t *camax_bits, hipStream_t st) {
    if (rows == 0 || cols == 0) return;
    dim3 grid((unsigned)((cols + kColTile - 1) / kColTile), (unsigned)((rows + kSlabRows - 1) / kSlabRows));
    profile_before(kTagColAmax, st, (double)rows * (double)cols * (kind == SRC_F32 ? 4.0 : kind == SRC_SWIGLU ? 4.0 : 2.0));
    switch (kind) {
        case SRC_BF16:
            grid.y = (unsigned)col_range_blocks_y(rows);
            hipLaunchKernelGGL(col_amax_bf16_kernel, grid, dim3(256), 0, st, (const uint16_t *)src, rows, cols, camax_bits);
            break;
        case SRC_F32:
            hipLaunchKernelGGL(col_amax_kernel<LoadF32>, grid, dim3(256), 0, st, LoadF32{(const float *)src},
                               rows, cols, camax_bits);
            break;
        case SRC_SWIGLU:
            hipLaunchKernelGGL(col_amax_kernel<LoadSwiglu>, grid, dim3(256), 0, st,
                               LoadSwiglu{(const uint16_t *)src, (const uint16_t *)src2}, rows, cols, camax_bits);
            break;
    }
    profile_after(st);
}

// ------------------------------------------------------------------ per-channel factors
// Smooth-SwiGLU (Section 4.4): s_i = fl32(448 / a_i), sinv_i = fl32(a_i / 448),
// both 1 for an all-zero channel.  The range of s^-1 * w3 needs no pass over
// W3: rounding is monotone, so max_j fl32(|w_ji| * sinv_i) = fl32(max_j |w_ji| * sinv_i).
__global__ void __launch_bounds__(256)
channel_factors_kernel(const float *__restrict__ h_camax, const float *__restrict__ w3_camax, int64_t f,
                       int smooth, const uint32_t *__restrict__ hmax_bits, const float *__restrict__ h_scale_given,
                       float *__restrict__ s, float *__restrict__ sinv, uint32_t *__restrict__ amax_w3s_bits) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t wbits = 0;
    if (i < f) {
        float si, sv;
        if (smooth) {
            const float a = h_camax[i];
            si = scale_from_amax(a, 448.0f, 0);
            sv = a > 0.0f ? __fdiv_rn(a, 448.0f) : 1.0f;
        } else {
            // plain block: one scale for the whole tensor, from its own range or as the caller gives it
            si = h_scale_given ? *h_scale_given : scale_from_amax(__uint_as_float(*hmax_bits), 448.0f, 0);
            sv = 1.0f;
        }
        s[i] = si;
        sinv[i] = sv;
        wbits = abs_bits_ignore_nan(__fmul_rn(w3_camax[i], sv));
    }
    wbits = wave_max_u32(wbits);
    if ((threadIdx.x & 63) == 0 && wbits) atomicMax(amax_w3s_bits, wbits);
}

__global__ void __launch_bounds__(256)
vec_max_kernel(const float *__restrict__ v, int64_t n, uint32_t *__restrict__ out_bits) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t b = i < n ? abs_bits_ignore_nan(v[i]) : 0u;
    b = wave_max_u32(b);
    if ((threadIdx.x & 63) == 0 && b) atomicMax(out_bits, b);
}

void launch_channel_factors(const float *h_camax, const float *w3_camax, int64_t f, int smooth, float *s,
                            float *sinv, uint32_t *amax_w3s_bits, uint32_t *hmax_bits, const float *h_scale_given,
                            hipStream_t st) {
    const unsigned blocks = (unsigned)((f + 255) / 256);
    if (!smooth) {
        profile_before(kTagSmall, st, 4.0 * (double)f);
        hipLaunchKernelGGL(vec_max_kernel, dim3(blocks), dim3(256), 0, st, h_camax, f, hmax_bits);
        profile_after(st);
    }
    profile_before(kTagSmall, st, 16.0 * (double)f);
    hipLaunchKernelGGL(channel_factors_kernel, dim3(blocks), dim3(256), 0, st, h_camax, w3_camax, f, smooth,
                       hmax_bits, smooth ? nullptr : h_scale_given, s, sinv, amax_w3s_bits);
    profile_after(st);
}

__global__ void __launch_bounds__(256)
fold_range_kernel(const float *__restrict__ w3_camax, const float *__restrict__ sinv, int64_t f,
                  uint32_t *__restrict__ amax_bits) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t b = i < f ? abs_bits_ignore_nan(__fmul_rn(w3_camax[i], sinv[i])) : 0u;
    b = wave_max_u32(b);
    if ((threadIdx.x & 63) == 0 && b) atomicMax(amax_bits, b);
}
void launch_fold_range(const float *w3_camax, const float *sinv, int64_t f, uint32_t *amax_bits, hipStream_t st) {
    hipLaunchKernelGGL(fold_range_kernel, dim3((unsigned)((f + 255) / 256)), dim3(256), 0, st, w3_camax, sinv, f,
                       amax_bits);
}

// ------------------------------------------------------------------ SwiGLU product (tests)
__global__ void __launch_bounds__(256)
swiglu_kernel(LoadSwiglu ld, size_t n8, float *__restrict__ h) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    float v[8];
    ld.load8(i * 8, v);
    *reinterpret_cast<float4 *>(h + i * 8) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(h + i * 8 + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
void launch_swiglu(const void *U, const void *G, int64_t n, float *h, hipStream_t st) {
    const size_t n8 = (size_t)n / 8;
    if (n8 == 0) return;
    hipLaunchKernelGGL(swiglu_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st,
                       LoadSwiglu{(const uint16_t *)U, (const uint16_t *)G}, n8, h);
}

// ------------------------------------------------------------------ bf16 transposes (last layer left in bf16)
// The comparison variant of Section 4.3 runs the last linear layer and its two gradient contractions on bf16
// operands; those contract over the index that is not contiguous in W3 [d,f], dY [T,d] and h [T,f], so transposed
// bf16 copies are written (64 x 64 tiles through LDS, 16-byte accesses on both sides).  SWIGLU: the source is the
// SwiGLU product of bf16 U, G, rounded once to bf16; it is written both as it stands and transposed.
template <bool SWIGLU>
__global__ void __launch_bounds__(256)
transpose_bf16_kernel(const uint16_t *__restrict__ src, const uint16_t *__restrict__ src2, int64_t rows, int64_t cols,
                      uint16_t *__restrict__ dst, uint16_t *__restrict__ dst_t) {
    __shared__ uint16_t tile[64][64 + 8];
    const int64_t row0 = (int64_t)blockIdx.y * 64, col0 = (int64_t)blockIdx.x * 64;
    const int c8 = (threadIdx.x & 7) * 8, r = threadIdx.x >> 3;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int64_t row = row0 + r + 32 * half, col = col0 + c8;
        uint4 q = make_uint4(0u, 0u, 0u, 0u);
        if (row < rows && col < cols) {
            const size_t at = (size_t)row * (size_t)cols + (size_t)col;
            if (SWIGLU) {
                float v[8];
                LoadSwiglu{src, src2}.load8(at, v);
                q = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                *reinterpret_cast<uint4 *>(dst + at) = q;
            } else {
                q = *reinterpret_cast<const uint4 *>(src + at);
            }
        }
        *reinterpret_cast<uint4 *>(&tile[r + 32 * half][c8]) = q;
    }
    __syncthreads();
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int c = r + 32 * half;                          // source column = row of the transposed copy
        const int64_t col = col0 + c, row = row0 + c8;        // c8 now counts source rows
        if (col < cols && row < rows) {
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) w[k] = (uint32_t)tile[c8 + 2 * k][c] | ((uint32_t)tile[c8 + 2 * k + 1][c] << 16);
            *reinterpret_cast<uint4 *>(dst_t + (size_t)col * (size_t)rows + (size_t)row) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}
void launch_transpose_bf16(const void *src, int64_t rows, int64_t cols, void *dst_t, hipStream_t st) {
    if (rows == 0 || cols == 0) return;
    const dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
    profile_before(kTagTranspose, st, 4.0 * (double)rows * (double)cols);
    hipLaunchKernelGGL(transpose_bf16_kernel<false>, grid, dim3(256), 0, st, (const uint16_t *)src, nullptr, rows, cols,
                       nullptr, (uint16_t *)dst_t);
    profile_after(st);
}
void launch_swiglu_bf16(const void *U, const void *G, int64_t rows, int64_t cols, void *h, void *h_t, hipStream_t st) {
    if (rows == 0 || cols == 0) return;
    const dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
    profile_before(kTagTranspose, st, 8.0 * (double)rows * (double)cols);
    hipLaunchKernelGGL(transpose_bf16_kernel<true>, grid, dim3(256), 0, st, (const uint16_t *)U, (const uint16_t *)G, rows, cols,
                       (uint16_t *)h, (uint16_t *)h_t);
    profile_after(st);
}

// ------------------------------------------------------------------ per-row factor, then per-tensor Q
// w1~ = Q(s_i * w1_i) of the inference form (end of Section 4.4): row i of a [rows, cols] bf16 matrix is
// multiplied by rs[i] (one fp32 multiply), the result is quantized per tensor to E4M3.  Run once per
// set of weights, so two plain elementwise passes: range, then cast.  cols is a multiple of 16, so
// the 8 elements of a lane share a row.
__global__ void __launch_bounds__(256)
rowscale_amax_kernel(const uint16_t *__restrict__ w, const float *__restrict__ rs, int64_t rows, int64_t cols,
                     uint32_t *__restrict__ slots) {
    const size_t n = (size_t)rows * (size_t)cols, stride = (size_t)gridDim.x * 256 * 8;
    uint32_t m = 0;
    for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8; i < n; i += stride) {
        float v[8];
        LoadBf16{w}.load8(i, v);
        const float f = rs[i / (size_t)cols];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t b = abs_bits_ignore_nan(__fmul_rn(v[k], f));
            m = m > b ? m : b;
        }
    }
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0 && m) atomicMax(slots + (blockIdx.x % kAmaxSlots) * kAmaxSlotStride, m);
}
__global__ void __launch_bounds__(256)
rowscale_cast_kernel(const uint16_t *__restrict__ w, const float *__restrict__ rs, int64_t rows, int64_t cols,
                     const uint32_t *__restrict__ slots, int pow2, float *__restrict__ scale_out,
                     float *__restrict__ amax_out, uint8_t *__restrict__ dst) {
    const float amax = __uint_as_float(wave_max_u32(slots[(threadIdx.x & 63) * kAmaxSlotStride]));
    const float sigma = scale_from_amax(amax, Fp8Traits<kE4M3>::fmax, pow2);
    if (blockIdx.x == 0 && threadIdx.x == 0) { *scale_out = sigma; if (amax_out) *amax_out = amax; }
    const size_t n = (size_t)rows * (size_t)cols, stride = (size_t)gridDim.x * 256 * 8;
    for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8; i < n; i += stride) {
        float v[8];
        LoadBf16{w}.load8(i, v);
        const float f = rs[i / (size_t)cols];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __fmul_rn(__fmul_rn(v[k], f), sigma);
        *reinterpret_cast<uint2 *>(dst + i) = make_uint2(satcast_pk4<kE4M3>(v[0], v[1], v[2], v[3]),
                                                         satcast_pk4<kE4M3>(v[4], v[5], v[6], v[7]));
    }
}
void launch_rowscale_quantize(const void *w, const float *row_scale, int64_t rows, int64_t cols, uint32_t *slots,
                              int pow2, float *scale_out, float *amax_out, uint8_t *dst, hipStream_t st) {
    const size_t groups = ((size_t)rows * (size_t)cols / 8 + 255) / 256;
    const unsigned blocks = (unsigned)(groups < 4096 ? groups : 4096);
    hipLaunchKernelGGL(rowscale_amax_kernel, dim3(blocks), dim3(256), 0, st, (const uint16_t *)w, row_scale, rows, cols, slots);
    hipLaunchKernelGGL(rowscale_cast_kernel, dim3(blocks), dim3(256), 0, st, (const uint16_t *)w, row_scale, rows, cols,
                       slots, pow2, scale_out, amax_out, dst);
}

// ------------------------------------------------------------------ delayed scaling state
__global__ void __launch_bounds__(256) scaling_init_kernel(uint32_t *state, size_t words) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= words) return;
    const bool is_scale = i < (size_t)kScalingTensors * kScalingStride && (i % kScalingStride) == 0;
    state[i] = is_scale ? 0x3f800000u : 0u;            // empty history: scale 1
}
void launch_scaling_init(uint32_t *state, hipStream_t st) {
    hipLaunchKernelGGL(scaling_init_kernel, dim3((unsigned)((kScalingWords + 255) / 256)), dim3(256), 0, st, state,
                       kScalingWords);
}

// One wave per tensor: the range of the call just made (maximum over its slots, which are cleared
// for the next call) replaces the oldest history entry; the next call's scale is fmax over the
// largest entry (Section 2, delayed scaling).
__global__ void __launch_bounds__(64) scaling_update_kernel(uint32_t *state, ScalingUpdate u) {
    const int k = blockIdx.x, lane = threadIdx.x;
    uint32_t *slots = u.slots[k];
    const uint32_t seen = wave_max_u32(slots[lane * kAmaxSlotStride]);
    slots[lane * kAmaxSlotStride] = 0u;
    uint32_t *w = state + (size_t)u.tensor[k] * kScalingStride;
    const uint32_t pos = w[1] % kScalingHistory;
    uint32_t h = lane < kScalingHistory ? w[8 + lane] : 0u;
    if (lane == (int)pos) h = seen;
    const float largest = __uint_as_float(wave_max_u32(h));
    const float fmax = u.fmt[k] == kE4M3 ? Fp8Traits<kE4M3>::fmax : Fp8Traits<kE5M2>::fmax;
    if (lane == 0) {
        w[8 + pos] = seen;
        w[1] = (pos + 1) % kScalingHistory;
        w[2] = seen;
        w[0] = __float_as_uint(scale_from_amax(largest, fmax, u.pow2));
    }
}
void launch_scaling_update(uint32_t *state, const ScalingUpdate &u, hipStream_t st) {
    if (u.count <= 0) return;
    profile_before(kTagSmall, st, 0.0);
    hipLaunchKernelGGL(scaling_update_kernel, dim3((unsigned)u.count), dim3(64), 0, st, state, u);
    profile_after(st);
}

}  // namespace ssg
