// One application of a stencil with a compile-time border region, marched down the matrix in
// registers: no local memory, no barrier, every input element is loaded and pre-processed once
// per strip (the tile kernel stages the N + S rows above and below each tile again).
//
// A wavefront owns a strip: its 64 lanes hold 64 consecutive 4-cell vectors of a row and it
// walks down H + N + S input rows.  When input row t arrives, each lane pre-processes its vector
// (Op::stage_vec, e.g. sine and cosine), fetches the W cells to its west and the E cells to its
// east from the adjacent lanes by cross-lane moves, and folds that row into the N + S + 1
// output rows whose border region contains it; the output row that just received its
// southernmost region row is finished and stored.  A cell therefore sees the rows of its
// region north to south and, inside a row, west to east - the order of the fold everywhere else,
// so results are bit-identical to the other mappings.  Lanes at a strip's end whose neighbour
// sits in another wavefront only feed their neighbours (one rim lane per side for up to four
// cells of border region there, two for up to eight), so strips advance by 60 to 64 vectors.
//
// All three border modes: a single application never needs a cell's new value, only resolved
// loads.
#pragma once
#include "tile_kernel.h"

namespace sk {

// Rim lanes at a side whose region extent is h cells (four cells per lane), and the vectors of a
// strip that are written, given the region's west / east extents.
__host__ __device__ constexpr int march_rim(int h) { return (h + 3) / 4; }
__host__ __device__ constexpr int march_vectors(int W, int E) { return 64 - march_rim(W) - march_rim(E); }

// FAST: rows are whole aligned vectors (cols % 4 == 0, 16-byte aligned pointers).  A lane's four
// columns then lie either all inside the matrix or all outside it, every row is one vector load
// at a per-lane column plus a wavefront-uniform row address, and what the border mode asks for
// beyond that is a per-lane fix-up of the loaded vector.  Otherwise elements are loaded one by one.
template <class Op, int B, class Halo, bool FAST>
__device__ __forceinline__ void march_body(const TileArgs<Op, Halo> &a, const int H) {
    using T = typename Op::T;
    using L = typename Op::L;
    static_assert(Halo::kStatic, "compile-time border regions only");
    static_assert(sizeof(T) == 4 && sizeof(L) == 4, "32-bit elements");
    constexpr int N = Halo::N, S = Halo::S, E = Halo::E, W = Halo::W;
    constexpr int CC = 4;
    static_assert(E <= 2 * CC && W <= 2 * CC, "row neighbours come from the two adjacent lanes at each side");
    constexpr int NP = Op::kPlanes;
    constexpr int R = N + S + 1;          // output rows in flight = rows of the region
    constexpr int WCOLS = E + W + 1;
    constexpr int kRimW = march_rim(W);
    constexpr int kCols = march_vectors(W, E) * CC;

    const int tid = (int)threadIdx.y * (int)blockDim.x + (int)threadIdx.x;
    const int lane = tid & 63;
    const int waves_per_block = ((int)blockDim.x * (int)blockDim.y) >> 6;
    int b = (int)blockIdx.x;
    if (a.xcd_chunk > 0) b = (b & 7) * a.xcd_chunk + (b >> 3);
    // a wavefront's index is the same in all its lanes: keep it, and all that follows from it, scalar
    const int wave = __builtin_amdgcn_readfirstlane(b * waves_per_block + (tid >> 6));
    if (wave >= a.n_tiles) return;
    const int seg = wave / a.tiles_c, strip = wave - seg * a.tiles_c;
    const int rows = a.rows, cols = a.cols;
    const int r0 = seg * H;
    const int gc0 = strip * kCols - kRimW * CC + lane * CC;    // first of this lane's four columns
    const bool writes = lane >= kRimW && lane < kRimW + march_vectors(W, E) && gc0 < cols;

    // FAST: the column the lane's vector load starts at, and its fix-up
    const bool outside = (unsigned)gc0 >= (unsigned)cols;
    int vcol = gc0;
    if (outside) vcol = B == kWrap ? resolve<B>(gc0, cols) : (gc0 < 0 ? 0 : cols - CC);
    const bool edge_wave = __any(outside) != 0;     // the same for the whole wavefront
    const unsigned in_off = (unsigned)vcol * (unsigned)sizeof(T);    // byte offsets inside a row
    const unsigned out_off = (unsigned)gc0 * (unsigned)sizeof(T);
    // otherwise: the lane's columns after border resolution (-1: padding)
    int col[CC];
#pragma unroll
    for (int j = 0; j < CC; ++j) col[j] = resolve<B>(gc0 + j, cols);
    const bool wanted = gc0 < cols + E;             // beyond that nobody reads this lane's cells

    // A segment needs kSteps input rows; the march makes whole rounds of R steps (what the steps
    // past kSteps compute is never stored) and the fast body issues exactly one load per step,
    // without a branch, so that the loads of the next R rows stay in flight behind the arithmetic.
    const int kSteps = H + N + S;
    const int kRounds = (kSteps + R - 1) / R;

    // issue the loads of input row r0 - N + t
    auto load_row = [&](int t, T (&v)[CC]) {
        const int tt = t < kSteps ? t : kSteps - 1;
        const int gr = resolve<B>(r0 - N + tt, rows);   // the same for the whole wavefront
        if (FAST) {
            // scalar row address + 32-bit lane offset; a padding row is fixed up later
            const char *rowp = reinterpret_cast<const char *>(a.in + (size_t)(gr < 0 ? 0 : gr) * cols);
            load_vec(v, reinterpret_cast<const T *>(rowp + in_off));
        } else {
#pragma unroll
            for (int j = 0; j < CC; ++j)
                v[j] = (gr >= 0 && wanted && col[j] >= 0) ? a.in[(size_t)gr * cols + col[j]] : a.pad;
        }
    };
    // what the border mode substitutes in a row that has arrived
    auto fix_row = [&](int t, T (&v)[CC]) {
        const bool row_outside = B == kConstant && (unsigned)(r0 - N + t) >= (unsigned)rows;
        if (FAST) {
            if (B == kConstant) {
                if (row_outside || edge_wave) {
#pragma unroll
                    for (int j = 0; j < CC; ++j) v[j] = (row_outside || outside) ? a.pad : v[j];
                }
            } else if (B == kClamp) {
                if (edge_wave) {
                    const T rep = gc0 < 0 ? v[0] : v[CC - 1];
#pragma unroll
                    for (int j = 0; j < CC; ++j) v[j] = outside ? rep : v[j];
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < CC; ++j)
                if (row_outside || col[j] < 0 || !wanted) v[j] = a.pad;
        }
    };

    // rows on their way from memory, R time steps ahead; output rows being accumulated
    T pf[R][CC];
    typename Op::State st[R][CC];
    [[maybe_unused]] float ring[3][R][CC] = {};   // operators with a tree of row sums: see below
#pragma unroll
    for (int u = 0; u < R; ++u) {
        load_row(u, pf[u]);
        // Keep these loads in the order the march consumes them.  Left to itself the scheduler may
        // issue them last-needed first; the march's first step would then have to wait for every
        // load in flight, and since waits are counted in issue order that wait (for all loads rather
        // than for the oldest) would stand at the head of every round of the loop.
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) Op::init(st[u][cc]);
    }

    for (int round = 0; round < kRounds; ++round) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const int t = round * R + u;            // input row r0 - N + t
            {
                fix_row(t, pf[u]);
                L sv[NP][CC];
                Op::template stage_vec<CC>(pf[u], sv);
                load_row(t + R, pf[u]);
                // the row as this lane's cells see it: W cells from the lane below, its own four,
                // E cells from the lane above
                L row[NP][W + CC + E];
#pragma unroll
                for (int p = 0; p < NP; ++p) {
#pragma unroll
                    for (int k = 0; k < W; ++k) {
                        // the cell d columns west of this lane's first: in the lane one below, or (d > 4) two below
                        const int d = W - k, hops = (d + CC - 1) / CC;
                        uint32_t x = from_lane_below(__float_as_uint(sv[p][hops * CC - d]));
                        if (hops == 2) x = from_lane_below(x);
                        row[p][k] = __uint_as_float(x);
                    }
#pragma unroll
                    for (int k = 0; k < CC; ++k) row[p][W + k] = sv[p][k];
#pragma unroll
                    for (int k = 0; k < E; ++k) {
                        const int hops = k / CC + 1;
                        uint32_t x = from_lane_above(__float_as_uint(sv[p][k - (hops - 1) * CC]));
                        if (hops == 2) x = from_lane_above(x);
                        row[p][W + CC + k] = __uint_as_float(x);
                    }
                }
                auto value_at = [&](int i) {
                    L parts[NP];
#pragma unroll
                    for (int p = 0; p < NP; ++p) parts[p] = row[p][i];
                    return Op::combine(parts);
                };
                // Operators that fold a row at a time and sum one of its parts as a tree of row sums
                // (the cosines): the row sum h(t) of every cell, the pair h(t-1) + h(t) and the four
                // pair(t-2) + pair(t) are formed once per input row and serve all the output rows
                // whose trees contain them; ring[level][t mod R].
                if constexpr (Op::kRowFold) {
#pragma unroll
                    for (int cc = 0; cc < CC; ++cc) {
                        const float h = Op::row_cos(W, E, [&](int dc) { return value_at(W + cc + dc); });
                        const float pair = __fadd_rn(ring[0][(u + R - 1) % R][cc], h);
                        ring[0][u][cc] = h;
                        ring[2][u][cc] = __fadd_rn(ring[1][(u + R - 2) % R][cc], pair);
                        ring[1][u][cc] = pair;
                    }
                }
                // this input row is region row dr of output row j = t - N - dr
#pragma unroll
                for (int dr = -N; dr <= S; ++dr) {
                    // Output rows above or below the segment belong to other wavefronts: nothing has
                    // to be folded for them (a wavefront-uniform test).  Worth it for short segments
                    // of a light function (5x5 sum, 10 rows: a quarter of the folds); the sin/cos
                    // stencil marches tall segments and keeps its straight-line code.
                    if (!Op::kRowFold && (unsigned)(t - N - dr) >= (unsigned)H) continue;
                    constexpr int kBig = 64 * R;    // keeps the remainder's operand positive
                    const int slot = (u - N - dr + kBig) % R;
#pragma unroll
                    for (int cc = 0; cc < CC; ++cc) {
                        if (dr == -N) Op::init(st[slot][cc]);
                        if constexpr (Op::kRowFold) {
                            Op::fold_sines(
                                st[slot][cc], W, E, [&](int dc) { return a.w[(dr + N) * WCOLS + dc + W]; },
                                [&](int dc) { return value_at(W + cc + dc); });
                            if (dr == S)
                                Op::set_cos(st[slot][cc], Op::template window_cos<R>([&](int level, int back) {
                                                return ring[level][(u + R - back) % R][cc];
                                            }));
                        } else {
                            fold_row<Op>(
                                st[slot][cc], dr, dr + N, R, W, E, [&](int dc) { return a.w[(dr + N) * WCOLS + dc + W]; },
                                [&](int dc) { return value_at(W + cc + dc); });
                        }
                    }
                    if (dr == S) {
                        const int gr = r0 + t - N - S;      // the output row that is complete now
                        if (t >= N + S && t < kSteps && gr < rows && writes) {
                            T res[CC];
#pragma unroll
                            for (int cc = 0; cc < CC; ++cc) res[cc] = Op::finish(st[slot][cc], a.scalar0);
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
    }
}

template <class Op, int B, class Halo, bool FAST, int MAXT>
__global__ __launch_bounds__(MAXT) void march_kernel(const TileArgs<Op, Halo> a, const int H) {
    march_body<Op, B, Halo, FAST>(a, H);
}

}  // namespace sk
