// Per-column range of a bf16 matrix [rows, cols] (Section 4.4: the per-channel maxima of w3 that give the
// range of s^-1 * w3 without a pass over the product), as the work of ONE workgroup of 256 threads, so that it can
// run as a kernel of its own or as extra workgroups at the end of another kernel's grid.
//
// The range is taken on the raw 16-bit patterns, two per operation: (|x| pattern) + 0x7f is below 0x8000 for
// every number and for infinity and at or above it for NaN, so a signed 16-bit maximum ignores NaN.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssg {

typedef short ssg_i16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int ssg_u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ ssg_i16x2 biased_abs_pk(uint32_t w) {
    return __builtin_bit_cast(ssg_i16x2, (w & 0x7fff7fffu) + 0x007f007fu);
}
// the larger of the two biased patterns as the fp32 bit pattern of the same number
__device__ __forceinline__ uint32_t unbias_max_pk(ssg_i16x2 m) {
    const uint32_t lo = (uint32_t)(uint16_t)m[0] - 0x7fu, hi = (uint32_t)(uint16_t)m[1] - 0x7fu;
    return (lo > hi ? lo : hi) << 16;
}

constexpr int kColTile = 512;          // one wave reads 1 KB of a row per load: 64 lanes x 8 bf16
constexpr int kColSlabBf16 = 256;      // rows per workgroup

// Grid of the pass: (cols / 512, rows / 256) workgroups, rounded up
inline __host__ __device__ int col_range_blocks_x(int64_t cols) { return (int)((cols + kColTile - 1) / kColTile); }
inline __host__ __device__ int col_range_blocks_y(int64_t rows) { return (int)((rows + kColSlabBf16 - 1) / kColSlabBf16); }

// Workgroup (bx, by): a lane owns 8 columns (one 16-byte piece per row), a wave 512 columns, and walks down its share
// of a 256-row slab with LOADS non-temporal row loads in flight; the four waves take every fourth row.  The running
// maxima stay packed (two columns per register); the waves meet in `cmax` (512 words of LDS) and one atomic per
// column goes to camax_bits (fp32 bit patterns, zeroed by the caller).  cols must be a multiple of 8.
template <int LOADS>
__device__ __forceinline__ void col_range_bf16_block(const uint16_t *__restrict__ src, int64_t rows, int64_t cols,
                                                     uint32_t *__restrict__ camax_bits, int bx, int by, uint32_t *cmax) {
    cmax[threadIdx.x] = 0;
    cmax[threadIdx.x + 256] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t col = (int64_t)bx * kColTile + lane * 8;
    const int64_t row0 = (int64_t)by * kColSlabBf16;
    const int64_t row1 = row0 + kColSlabBf16 < rows ? row0 + kColSlabBf16 : rows;
    if (col < cols) {
        ssg_i16x2 m[4] = {{0x7f, 0x7f}, {0x7f, 0x7f}, {0x7f, 0x7f}, {0x7f, 0x7f}};
        for (int64_t r = row0 + w; r < row1; r += 4 * LOADS) {
            ssg_u32x4 v[LOADS];
#pragma unroll
            for (int u = 0; u < LOADS; ++u) {
                const int64_t rr = r + 4 * u;
                v[u] = rr < row1 ? __builtin_nontemporal_load(reinterpret_cast<const ssg_u32x4 *>(src + (size_t)rr * (size_t)cols + (size_t)col))
                                 : ssg_u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < LOADS; ++u)
#pragma unroll
                for (int k = 0; k < 4; ++k) m[k] = __builtin_elementwise_max(m[k], biased_abs_pk(v[u][k]));
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t lo = ((uint32_t)(uint16_t)m[k][0] - 0x7fu) << 16, hi = ((uint32_t)(uint16_t)m[k][1] - 0x7fu) << 16;
            if (lo) atomicMax(&cmax[lane * 8 + 2 * k], lo);
            if (hi) atomicMax(&cmax[lane * 8 + 2 * k + 1], hi);
        }
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int t = threadIdx.x + 256 * h;
        const int64_t c = (int64_t)bx * kColTile + t;
        if (c < cols && cmax[t]) atomicMax(&camax_bits[c], cmax[t]);
    }
}

}  // namespace ssg
