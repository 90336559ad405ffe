// Temporal blocking in registers for iterated stencils with the 1/1/1/1 border region:
// one launch advances the matrix by DEPTH applications without local memory or barriers.
//
// A wavefront owns a strip of the matrix: its 64 lanes hold 64 consecutive 4-cell vectors of a
// row (256 columns) and it walks down H + 2*DEPTH rows.  Every lane keeps, for each of the
// DEPTH time levels, the last three rows of its vector; as soon as input row t has arrived,
// level 1 can produce its row t - 1, level 2 its row t - 2, and so on (each level lags one row
// behind the one below), and level DEPTH's rows go straight to global memory.  Row neighbours
// come from the adjacent lanes by cross-lane moves.  What a level computes within k cells of the
// strip's edge is stale after k applications, so the first and the last lane (4 cells each,
// DEPTH <= 4) are rim lanes and the strip's 62 inner vectors (248 columns) are written; strips
// therefore advance by 248 columns, rows by H.
//
// Borders: periodic copies evolve like their originals, so WRAP needs nothing beyond wrapped
// loads; under CONSTANT the out-of-matrix cells of every level are set back to the padding
// value.  (CLAMP would need a clamped row's new value before the marching order produces it;
// it stays with the local-memory temporal kernel.)  The per-cell arithmetic is the same fold as
// everywhere else: results are bit-identical to DEPTH single launches.
#pragma once
#include "tile_kernel.h"

namespace sk {

constexpr int kStreamLanes = 64;                    // vectors per strip row, rim included
constexpr int kStreamCols = (kStreamLanes - 2) * 4; // columns a strip writes

template <class Op, int B, int DEPTH, int MAXT>
__global__ __launch_bounds__(MAXT) void stream_kernel(const TileArgs<Op, HaloC<1, 1, 1, 1>> a, const int H) {
    using T = typename Op::T;
    static_assert(B == kWrap || B == kConstant, "wrap and constant borders only");
    static_assert(DEPTH >= 1 && DEPTH <= 4, "one rim lane covers at most four applications");
    static_assert(Op::kPlanes == 1 && sizeof(T) == 4, "fp32, one value per cell");
    constexpr int CC = 4;

    const int tid = (int)threadIdx.y * (int)blockDim.x + (int)threadIdx.x;
    const int lane = tid & 63;
    const int waves_per_block = ((int)blockDim.x * (int)blockDim.y) >> 6;
    // a wavefront's index is the same in all its lanes: keep it, and all that follows from it, scalar
    const int wave = __builtin_amdgcn_readfirstlane((int)blockIdx.x * waves_per_block + (tid >> 6));
    if (wave >= a.n_tiles) return;
    const int seg = wave / a.tiles_c, strip = wave - seg * a.tiles_c;
    const int rows = a.rows, cols = a.cols;
    const int r0 = seg * H;
    const int gc0 = strip * kStreamCols - CC + lane * CC;      // first of this lane's four columns

    // this lane's columns after border resolution (-1: padding), and whether one vector load serves
    int col[CC];
#pragma unroll
    for (int j = 0; j < CC; ++j) col[j] = resolve<B>(gc0 + j, cols);
    const bool vec = a.vec_ok && col[0] >= 0 && col[0] + CC <= cols && col[3] == col[0] + 3;
    bool outside_c[CC];   // CONSTANT: cells that are not matrix cells
#pragma unroll
    for (int j = 0; j < CC; ++j) outside_c[j] = (unsigned)(gc0 + j) >= (unsigned)cols;

    auto load_row = [&](int t, T (&v)[CC]) {
        const int gr = resolve<B>(r0 - DEPTH + t, rows);
        if (gr < 0) {
#pragma unroll
            for (int j = 0; j < CC; ++j) v[j] = a.pad;
        } else if (vec) {
            load_vec(v, a.in + (size_t)gr * cols + col[0]);
        } else {
#pragma unroll
            for (int j = 0; j < CC; ++j) v[j] = col[j] < 0 ? a.pad : a.in[(size_t)gr * cols + col[j]];
        }
    };

    // lv[k][s]: level k's row that was produced at a time step with t % 3 == s  (level 0 = input)
    T lv[DEPTH][3][CC];
#pragma unroll
    for (int k = 0; k < DEPTH; ++k)
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int j = 0; j < CC; ++j) lv[k][s][j] = 0;
    T pf[3][CC];          // rows on their way from memory, three time steps ahead
#pragma unroll
    for (int s = 0; s < 3; ++s) load_row(s, pf[s]);

    const int kSteps = H + 2 * DEPTH;
    for (int t0 = 0; t0 < kSteps; t0 += 3) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int t = t0 + u;
            if (t < kSteps) {                       // same for every lane
#pragma unroll
                for (int j = 0; j < CC; ++j) lv[0][u][j] = pf[u][j];
                if (t + 3 < kSteps) load_row(t + 3, pf[u]);
#pragma unroll
                for (int k = 1; k <= DEPTH; ++k) {
                    // level k's row r0 - DEPTH + t - k from level k-1's three newest rows
                    const T(&up)[CC] = lv[k - 1][(u + 1) % 3];
                    const T(&mid)[CC] = lv[k - 1][(u + 2) % 3];
                    const T(&dn)[CC] = lv[k - 1][u];
                    typename Op::State st[CC];
#pragma unroll
                    for (int cc = 0; cc < CC; ++cc) Op::init(st[cc]);
#pragma unroll
                    for (int dr = -1; dr <= 1; ++dr) {
                        const T(&q)[CC] = dr < 0 ? up : (dr == 0 ? mid : dn);
                        const T row[6] = {__uint_as_float(from_lane_below(__float_as_uint(q[3]))), q[0], q[1], q[2],
                                          q[3], __uint_as_float(from_lane_above(__float_as_uint(q[0])))};
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc)
                            fold_row<Op>(
                                st[cc], dr, 1, 1, [&](int dc) { return a.w[(dr + 1) * 3 + dc + 1]; },
                                [&](int dc) { return row[1 + cc + dc]; });
                    }
                    T res[CC];
#pragma unroll
                    for (int cc = 0; cc < CC; ++cc) res[cc] = Op::finish(st[cc], a.scalar0);
                    const int gr = r0 - DEPTH + t - k;      // the matrix row just produced
                    if (B == kConstant) {
                        const bool outside_r = (unsigned)gr >= (unsigned)rows;
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc)
                            if (outside_r || outside_c[cc]) res[cc] = a.pad;
                    }
                    if (k < DEPTH) {
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc) lv[k][u][cc] = res[cc];
                    } else if (t >= 2 * DEPTH && gr < rows && lane > 0 && lane < kStreamLanes - 1 && gc0 < cols) {
                        // gr = r0 + t - 2*DEPTH runs over this segment's rows
                        T *out = a.out + (size_t)gr * cols + gc0;
                        if (a.vec_ok && gc0 + CC <= cols) {
                            store_vec(out, res);
                        } else {
#pragma unroll
                            for (int cc = 0; cc < CC; ++cc)
                                if (gc0 + cc < cols) out[cc] = res[cc];
                        }
                    }
                }
            }
        }
    }
}

}  // namespace sk
