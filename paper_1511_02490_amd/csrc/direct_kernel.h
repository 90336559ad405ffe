// Stencil kernels that stage nothing in local memory: each work-item pulls the rows of its
// window straight from global memory as 16-byte vectors and keeps them in registers, and the
// reuse between neighbouring work-items that the paper's local-memory tile provides
// (Section 2) is left to the vector L1 and the XCD's L2.  For light customising functions
// with a small border region this is faster on CDNA4 than the tile, because there is no
// barrier between a workgroup's loads and its stores and every wavefront is independent.
// The workgroup shape w_r x w_c still decides which cells share a compute unit's L1.
#pragma once
#include "tile_kernel.h"

namespace sk {

// Window row `gr_raw` for the CC cells starting at column c0: W values to the west, the CC
// cells, E values to the east, border-resolved.
template <class Op, int B, int CC, int W, int E>
__device__ __forceinline__ void fetch_row(typename Op::V (&row)[W + CC + E], const typename Op::T *in, int gr_raw,
                                          int c0, int rows, int cols, bool fast_cols, typename Op::T pad) {
    using T = typename Op::T;
    static_assert(W <= CC && E <= CC, "direct kernels reach at most one vector to each side");
    const int gr = resolve<B>(gr_raw, rows);
    T v[W + CC + E];
    if (gr >= 0 && fast_cols) {
        const T *p = in + (size_t)gr * cols + c0;
        T ctr[CC];
        load_vec(ctr, p);
#pragma unroll
        for (int k = 0; k < CC; ++k) v[W + k] = ctr[k];
        if constexpr (W == 1) v[0] = p[-1];
        if constexpr (W > 1) {
            T side[CC];
            load_vec(side, p - CC);
#pragma unroll
            for (int k = 0; k < W; ++k) v[k] = side[CC - W + k];
        }
        if constexpr (E == 1) v[W + CC] = p[CC];
        if constexpr (E > 1) {
            T side[CC];
            load_vec(side, p + CC);
#pragma unroll
            for (int k = 0; k < E; ++k) v[W + CC + k] = side[k];
        }
    } else {
#pragma unroll
        for (int k = 0; k < W + CC + E; ++k) {
            const int gc = resolve<B>(c0 - W + k, cols);
            v[k] = (gr < 0 || gc < 0) ? pad : in[(size_t)gr * cols + gc];
        }
    }
#pragma unroll
    for (int k = 0; k < W + CC + E; ++k) {
        typename Op::L parts[Op::kPlanes];
        Op::stage(v[k], parts);
        row[k] = Op::combine(parts);
    }
}

// Work-item (ty, tx) of workgroup (tile_r, tile_c) owns rows (tile_r*w_r + ty)*CR .. +CR-1 and
// columns (tile_c*w_c + tx)*CC .. +CC-1.  Same fold, in the same order, as the tile kernel.
template <class Op, int B, class Halo, int CR, int CC, int MAXT>
__global__ __launch_bounds__(MAXT) void direct_kernel(const TileArgs<Op, Halo> a) {
    static_assert(Halo::kStatic, "direct kernels are compiled per border region");
    using T = typename Op::T;
    using V = typename Op::V;
    constexpr int N = Halo::N, S = Halo::S, E = Halo::E, W = Halo::W;
    constexpr int WCOLS = E + W + 1;

    int t = blockIdx.x;
    if (a.xcd_chunk > 0) t = (t & 7) * a.xcd_chunk + (t >> 3);
    if (t >= a.n_tiles) return;
    const int tile_r = t / a.tiles_c, tile_c = t - tile_r * a.tiles_c;
    const int rows = a.rows, cols = a.cols;
    const int r0 = (tile_r * (int)blockDim.y + (int)threadIdx.y) * CR;
    const int c0 = (tile_c * (int)blockDim.x + (int)threadIdx.x) * CC;
    if (r0 >= rows || c0 >= cols) return;

    const bool fast_cols = a.vec_ok && c0 >= (W > 0 ? CC : 0) && c0 + CC + (E > 0 ? CC : 0) <= cols;

    typename Op::State st[CR][CC];
#pragma unroll
    for (int cr = 0; cr < CR; ++cr)
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) Op::init(st[cr][cc]);

    // A small window is fetched whole before its first row is used (rows below the matrix resolve
    // like any other out-of-matrix row): no branch separates the loads, so all of them are in
    // flight together instead of one memory round trip per row.  A large window would cost
    // registers, and with them resident wavefronts: its rows are fetched as they are needed.
    constexpr bool kWhole = (CR + N + S) * (W + CC + E) <= 32;
    V win[kWhole ? CR + N + S : 1][W + CC + E];
    if constexpr (kWhole) {
#pragma unroll
        for (int wi = 0; wi < CR + N + S; ++wi)
            fetch_row<Op, B, CC, W, E>(win[wi], a.in, r0 - N + wi, c0, rows, cols, fast_cols, a.pad);
    }
#pragma unroll
    for (int wi = 0; wi < CR + N + S; ++wi) {
        if constexpr (!kWhole) {
            // the first cell-row this window row feeds; stop once that lies below the matrix
            const int first_cr = wi - N - S > 0 ? wi - N - S : 0;
            if (r0 + first_cr >= rows) break;
            fetch_row<Op, B, CC, W, E>(win[0], a.in, r0 - N + wi, c0, rows, cols, fast_cols, a.pad);
        }
        const V(&row)[W + CC + E] = win[kWhole ? wi : 0];
#pragma unroll
        for (int cr = 0; cr < CR; ++cr) {
            const int dr = wi - N - cr;
            if (dr < -N || dr > S) continue;
#pragma unroll
            for (int cc = 0; cc < CC; ++cc)
                fold_row<Op>(
                    st[cr][cc], dr, dr + N, N + S + 1, W, E, [&](int dc) { return a.w[(dr + N) * WCOLS + dc + W]; },
                    [&](int dc) { return row[W + cc + dc]; });
        }
    }

#pragma unroll
    for (int cr = 0; cr < CR; ++cr) {
        const int r = r0 + cr;
        if (r >= rows) break;
        T res[CC];
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) res[cc] = Op::finish(st[cr][cc], a.scalar0);
        T *dst = a.out + (size_t)r * cols + c0;
        if (a.vec_ok && c0 + CC <= cols) {
            store_out_vec(dst, res, a.nt_store != 0);
        } else {
#pragma unroll
            for (int cc = 0; cc < CC; ++cc)
                if (c0 + cc < cols) dst[cc] = res[cc];
        }
    }
}

// ---- Game of Life on packed bytes -----------------------------------------------------------
// 16 cells per work-item and row, four per 32-bit register.  Cells are 0/1, so byte-wise sums
// of up to nine cells never carry into the next byte.  For each cell: s = sum of the 3x3
// block (centre included), n = s - self, alive' = ((n | self) == 3), i.e. B3/S23.
struct LifeRow {
    uint32_t w[4];   // 16 cells
    uint32_t l, r;   // the cell west of w[0]'s first byte, the cell east of w[3]'s last byte
};

// Next generation of the 16 cells of `cur`, given the rows above and below.
__device__ __forceinline__ void life_rule(uint32_t (&o)[4], const LifeRow &above, const LifeRow &cur,
                                          const LifeRow &below) {
    uint32_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = above.w[k] + cur.w[k] + below.w[k];   // column sums
    const uint32_t vl = above.l + cur.l + below.l, vr = above.r + cur.r + below.r;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t west = (v[k] << 8) | (k == 0 ? vl : (v[k - 1] >> 24));
        const uint32_t east = (v[k] >> 8) | ((k == 3 ? vr : v[k + 1]) << 24);
        const uint32_t s = v[k] + west + east;        // 3x3 block sums, <= 9 per byte
        const uint32_t n = s - cur.w[k];              // neighbours only
        o[k] = zero_bytes((n | cur.w[k]) ^ 0x03030303u);    // zero byte <=> alive next
    }
}

// Loads one row of 16 cells and the two cells just west and east of them (columns gcw / gce after
// border resolution, -1 for padding).  All three loads are unconditional and independent of each
// other, so the loads of every row a work-item needs can be in flight together.
template <int B>
__device__ __forceinline__ LifeRow life_fetch(const uint8_t *in, int gr_raw, int c0, int rows, int cols,
                                              bool fast_cols, uint8_t pad, int gcw, int gce) {
    LifeRow x;
    const int gr = resolve<B>(gr_raw, rows);
    const uint8_t *row = in + (size_t)(gr < 0 ? 0 : gr) * cols;
    if (gr >= 0 && fast_cols) {
        const uint4 v = *reinterpret_cast<const uint4 *>(row + c0);
        x.w[0] = v.x; x.w[1] = v.y; x.w[2] = v.z; x.w[3] = v.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t word = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int gc = resolve<B>(c0 + 4 * k + b, cols);
                const uint32_t cell = (gr < 0 || gc < 0) ? pad : row[gc];
                word |= cell << (8 * b);
            }
            x.w[k] = word;
        }
    }
    const uint32_t west = row[gcw < 0 ? 0 : gcw], east = row[gce < 0 ? 0 : gce];
    x.l = (gr < 0 || gcw < 0) ? pad : west;
    x.r = (gr < 0 || gce < 0) ? pad : east;
    return x;
}

template <int B, int CR, int MAXT>
__global__ __launch_bounds__(MAXT) void life_direct_kernel(const TileArgs<OpLife, HaloC<1, 1, 1, 1>> a) {
    constexpr int CC = 16;
    int t = blockIdx.x;
    if (a.xcd_chunk > 0) t = (t & 7) * a.xcd_chunk + (t >> 3);
    if (t >= a.n_tiles) return;
    const int tile_r = t / a.tiles_c, tile_c = t - tile_r * a.tiles_c;
    const int rows = a.rows, cols = a.cols;
    const int r0 = (tile_r * (int)blockDim.y + (int)threadIdx.y) * CR;
    const int c0 = (tile_c * (int)blockDim.x + (int)threadIdx.x) * CC;
    if (r0 >= rows || c0 >= cols) return;
    const bool fast_cols = a.vec_ok && c0 + CC <= cols;
    // the columns just west and east of this work-item's cells, the same for every row
    const int gcw = resolve<B>(c0 - 1, cols), gce = resolve<B>(c0 + CC, cols);

    // all CR + 2 rows before the first is used (rows below the matrix resolve like any other
    // out-of-matrix row): every load of the work-item is in flight at once
    LifeRow win[CR + 2];
#pragma unroll
    for (int k = 0; k < CR + 2; ++k)
        win[k] = life_fetch<B>(a.in, r0 - 1 + k, c0, rows, cols, fast_cols, a.pad, gcw, gce);
#pragma unroll
    for (int cr = 0; cr < CR; ++cr) {
        const int r = r0 + cr;
        if (r >= rows) break;
        uint32_t o[4];
        life_rule(o, win[cr], win[cr + 1], win[cr + 2]);
        uint8_t *dst = a.out + (size_t)r * cols + c0;
        if (a.vec_ok && c0 + CC <= cols) {
            store_word4(dst, make_uint4(o[0], o[1], o[2], o[3]), a.nt_store != 0);
        } else {
#pragma unroll
            for (int k = 0; k < CC; ++k)
                if (c0 + k < cols) dst[k] = (uint8_t)(o[k >> 2] >> (8 * (k & 3)));
        }
    }
}

}  // namespace sk
