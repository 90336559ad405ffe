// The Canny detector's threshold stencil (Table 2): no border region, a float matrix in and a
// byte matrix out - the one kernel here whose output type differs from its input type.  The
// skeleton's decomposition stays: workgroups of w_r x w_c work-items tile the matrix, a work-item
// owns CR x CC adjacent cells; with CC = 4 it moves one 16-byte vector in and four bytes out.
#pragma once
#include "tile_kernel.h"

namespace sk {

struct ThresholdArgs {
    const float *in;
    uint8_t *out;
    int rows, cols;
    int tiles_c, n_tiles;
    int xcd_chunk;   // > 0: tiles are dealt to the 8 XCDs in contiguous chunks of this many
    int vec_ok;      // rows of `in` start 16-byte aligned, rows of `out` 4-byte aligned, cols % 4 == 0
    float level;
};

// 1 where the value reaches the level, else 0 (a NaN reaches nothing)
__device__ __forceinline__ uint32_t reaches(float v, float level) { return v >= level ? 1u : 0u; }

template <int CR, int CC, int MAXT>
__global__ __launch_bounds__(MAXT) void threshold_kernel(const ThresholdArgs a) {
    int t = blockIdx.x;
    if (a.xcd_chunk > 0) t = (t & 7) * a.xcd_chunk + (t >> 3);
    if (t >= a.n_tiles) return;
    const int tile_r = t / a.tiles_c, tile_c = t - tile_r * a.tiles_c;
    const int r0 = (tile_r * (int)blockDim.y + (int)threadIdx.y) * CR;
    const int c0 = (tile_c * (int)blockDim.x + (int)threadIdx.x) * CC;
    if (c0 >= a.cols) return;
#pragma unroll
    for (int cr = 0; cr < CR; ++cr) {
        const int r = r0 + cr;
        if (r >= a.rows) break;
        const float *src = a.in + (size_t)r * a.cols + c0;
        uint8_t *dst = a.out + (size_t)r * a.cols + c0;
        if constexpr (CC == 4) {
            if (a.vec_ok && c0 + CC <= a.cols) {
                float v[4];
                load_vec(v, src);
                *reinterpret_cast<uint32_t *>(dst) = reaches(v[0], a.level) | (reaches(v[1], a.level) << 8) |
                                                     (reaches(v[2], a.level) << 16) | (reaches(v[3], a.level) << 24);
                continue;
            }
        }
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
            if (c0 + cc < a.cols) dst[cc] = (uint8_t)reaches(src[cc], a.level);
    }
}

}  // namespace sk
