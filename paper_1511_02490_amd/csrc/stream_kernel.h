// Temporal blocking in registers for iterated stencils with the 1/1/1/1 border region:
// one launch advances the matrix by DEPTH applications without local memory or barriers.
//
// A wavefront owns a strip of the matrix: its 64 lanes hold 64 consecutive 4-cell vectors of a
// row (256 columns) and it walks down H + 2*DEPTH rows.  Every lane keeps, for each of the
// DEPTH time levels, the last three rows of its vector; as soon as input row t has arrived,
// level 1 can produce its row t - 1, level 2 its row t - 2, and so on (each level lags one row
// behind the one below), and level DEPTH's rows go straight to global memory.  Row neighbours
// come from the adjacent lanes by cross-lane moves.  What a level computes within k cells of the
// strip's edge is stale after k applications, so the outermost lanes are rim lanes (4 cells each:
// one lane per side up to 4 applications, two up to 8) and the strip's 62 or 60 inner vectors are
// written; strips therefore advance by 248 or 240 columns, rows by H.
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
constexpr int kStreamMaxDepth = 8;
// rim lanes per side, and the columns a strip writes, for `depth` applications per launch
__host__ __device__ constexpr int stream_rim(int depth) { return (depth + 3) / 4; }
__host__ __device__ constexpr int stream_cols(int depth) { return (kStreamLanes - 2 * stream_rim(depth)) * 4; }

// FAST: rows are whole aligned vectors (cols % 4 == 0, 16-byte aligned pointers).  A lane's four
// columns then lie either all inside the matrix or all outside it, every input row is one vector
// load at a per-lane column plus a wavefront-uniform row address, issued without a branch three
// steps ahead, and the time loop is straight-line code.  Otherwise elements are loaded one by one.
template <class Op, int B, int DEPTH, bool FAST>
__device__ __forceinline__ void stream_body(const TileArgs<Op, HaloC<1, 1, 1, 1>> &a, const int H) {
    using T = typename Op::T;
    static_assert(B == kWrap || B == kConstant, "wrap and constant borders only");
    static_assert(DEPTH >= 1 && DEPTH <= kStreamMaxDepth, "a rim lane covers four applications");
    static_assert(Op::kPlanes == 1 && sizeof(T) == 4, "fp32, one value per cell");
    constexpr int CC = 4;
    constexpr int R = 3;                            // rows of a level kept
    constexpr int PF = 6;                           // input rows in flight = steps per round (a multiple of R)
    constexpr int kRim = stream_rim(DEPTH);
    constexpr int kCols = stream_cols(DEPTH);

    const int tid = (int)threadIdx.y * (int)blockDim.x + (int)threadIdx.x;
    const int lane = tid & 63;
    const int waves_per_block = ((int)blockDim.x * (int)blockDim.y) >> 6;
    // a wavefront's index is the same in all its lanes: keep it, and all that follows from it, scalar
    const int wave = __builtin_amdgcn_readfirstlane((int)blockIdx.x * waves_per_block + (tid >> 6));
    if (wave >= a.n_tiles) return;
    const int seg = wave / a.tiles_c, strip = wave - seg * a.tiles_c;
    const int rows = a.rows, cols = a.cols;
    const int r0 = seg * H;
    const int gc0 = strip * kCols - kRim * CC + lane * CC;     // first of this lane's four columns
    const bool writes = lane >= kRim && lane < kStreamLanes - kRim && gc0 < cols;

    // FAST: the column the lane's vector load starts at (wrapped, or any valid one for padding)
    const bool outside = (unsigned)gc0 >= (unsigned)cols;
    const int vcol = !outside ? gc0 : (B == kWrap ? resolve<B>(gc0, cols) : 0);
    const bool edge_wave = __any(outside) != 0;     // the same for the whole wavefront
    const unsigned in_off = (unsigned)vcol * (unsigned)sizeof(T);    // byte offsets inside a row
    const unsigned out_off = (unsigned)gc0 * (unsigned)sizeof(T);
    // otherwise: the lane's columns after border resolution (-1: padding)
    int col[CC];
#pragma unroll
    for (int j = 0; j < CC; ++j) col[j] = resolve<B>(gc0 + j, cols);
    bool outside_c[CC];   // CONSTANT: cells that are not matrix cells
#pragma unroll
    for (int j = 0; j < CC; ++j) outside_c[j] = (unsigned)(gc0 + j) >= (unsigned)cols;

    // A segment consumes kSteps input rows; the march makes whole rounds of PF steps (what the
    // steps past kSteps compute is never stored).
    const int kSteps = H + 2 * DEPTH;
    const int kRounds = (kSteps + PF - 1) / PF;

    // issue the loads of input row r0 - DEPTH + t
    auto load_row = [&](int t, T (&v)[CC]) {
        const int tt = t < kSteps ? t : kSteps - 1;
        const int gr = resolve<B>(r0 - DEPTH + tt, rows);      // the same for the whole wavefront
        if (FAST) {
            const char *rowp = reinterpret_cast<const char *>(a.in + (size_t)(gr < 0 ? 0 : gr) * cols);
            load_vec(v, reinterpret_cast<const T *>(rowp + in_off));
        } else {
#pragma unroll
            for (int j = 0; j < CC; ++j)
                v[j] = (gr >= 0 && col[j] >= 0) ? a.in[(size_t)gr * cols + col[j]] : a.pad;
        }
    };
    // CONSTANT: cells of matrix row gr (any time level) that are not matrix cells hold the padding
    auto pad_outside = [&](int gr, T (&v)[CC]) {
        if (B != kConstant) return;
        const bool outside_r = (unsigned)gr >= (unsigned)rows;
        if (FAST) {
            if (outside_r || edge_wave) {
#pragma unroll
                for (int j = 0; j < CC; ++j) v[j] = (outside_r || outside) ? a.pad : v[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < CC; ++j)
                if (outside_r || outside_c[j]) v[j] = a.pad;
        }
    };

    // lv[k][s]: level k's row that was produced at a time step with t % 3 == s  (level 0 = input)
    T lv[DEPTH][R][CC];
#pragma unroll
    for (int k = 0; k < DEPTH; ++k)
#pragma unroll
        for (int s = 0; s < R; ++s)
#pragma unroll
            for (int j = 0; j < CC; ++j) lv[k][s][j] = 0;
    T pf[PF][CC];         // rows on their way from memory, PF time steps ahead
#pragma unroll
    for (int s = 0; s < PF; ++s) {
        load_row(s, pf[s]);
        // in the order the march consumes them: were the scheduler to issue the first-needed row
        // last, every round of the loop would begin by waiting for all loads in flight
        __builtin_amdgcn_sched_barrier(0);
    }

    for (int round = 0; round < kRounds; ++round) {
#pragma unroll
        for (int v = 0; v < PF; ++v) {
            const int t = round * PF + v;
            const int u = v % R;                    // = t % R
#pragma unroll
            for (int j = 0; j < CC; ++j) lv[0][u][j] = pf[v][j];
            pad_outside(r0 - DEPTH + t, lv[0][u]);
            load_row(t + PF, pf[v]);
#pragma unroll
            for (int k = 1; k <= DEPTH; ++k) {
                // level k's first row that anything depends on is r0 - DEPTH + k, due at step 2k:
                // before that the level has nothing to do (a wavefront-uniform test)
                if (t < 2 * k) continue;
                // level k's row r0 - DEPTH + t - k from level k-1's three newest rows
                const T(&up)[CC] = lv[k - 1][(u + 1) % R];
                const T(&mid)[CC] = lv[k - 1][(u + 2) % R];
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
                            st[cc], dr, dr + 1, 3, 1, 1, [&](int dc) { return a.w[(dr + 1) * 3 + dc + 1]; },
                            [&](int dc) { return row[1 + cc + dc]; });
                }
                T res[CC];
#pragma unroll
                for (int cc = 0; cc < CC; ++cc) res[cc] = Op::finish(st[cc], a.scalar0);
                const int gr = r0 - DEPTH + t - k;      // the matrix row just produced
                if (k < DEPTH) {
                    pad_outside(gr, res);
#pragma unroll
                    for (int cc = 0; cc < CC; ++cc) lv[k][u][cc] = res[cc];
                } else if (t >= 2 * DEPTH && t < kSteps && gr < rows && writes) {
                    // gr = r0 + t - 2*DEPTH runs over this segment's rows
                    if (FAST) {
                        char *rowp = reinterpret_cast<char *>(a.out + (size_t)gr * cols);
                        store_out_vec(reinterpret_cast<T *>(rowp + out_off), res, a.nt_store != 0);
                    } else {
                        T *out = a.out + (size_t)gr * cols + gc0;
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc)
                            if (gc0 + cc < cols) out[cc] = res[cc];
                    }
                }
            }
        }
    }
}

template <class Op, int B, int DEPTH, bool FAST, int MAXT>
__global__ __launch_bounds__(MAXT) void stream_kernel(const TileArgs<Op, HaloC<1, 1, 1, 1>> a, const int H) {
    stream_body<Op, B, DEPTH, FAST>(a, H);
}

}  // namespace sk
