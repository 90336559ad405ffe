// The stencil skeleton's kernel (Section 2 and Figure 1 of the paper): the matrix is cut
// into workgroups of w_r x w_c work-items; each workgroup stages its tile plus the perimeter
// border region in local memory (LDS), waits, and every work-item folds the customising
// function over the border region of its cells.
//
// Beyond the paper's one-element-per-work-item mapping, a work-item may own a CR x CC block
// of adjacent cells (register blocking): the workgroup then covers (w_r*CR) x (w_c*CC)
// elements, rows of the window are pulled from LDS once and reused by all the cells they
// touch, and with CC*sizeof(T) = 16 bytes HBM and LDS traffic moves as 128-bit accesses.
#pragma once
#include "stencil_ops.h"

namespace sk {

template <class Op, class Halo, bool Static = Halo::kStatic>
struct WeightStore;
// Compile-time region: the weight table travels in the kernel arguments (scalar registers).
template <class Op, class Halo>
struct WeightStore<Op, Halo, true> {
    static constexpr int kCount = Op::kWeights ? (Halo::N + Halo::S + 1) * (Halo::E + Halo::W + 1) : 1;
    using W = typename weight_type_of<Op>::type;
    W v[kCount];
    __device__ __forceinline__ W operator[](int k) const { return Op::kWeights ? v[k] : W(0); }
};
// Run-time region: table in device memory (uniform index -> scalar loads).
template <class Op, class Halo>
struct WeightStore<Op, Halo, false> {
    const float *v;
    __device__ __forceinline__ float operator[](int k) const { return Op::kWeights ? v[k] : 0.0f; }
};

template <class Op, class Halo>
struct TileArgs {
    const typename Op::T *in;
    typename out_type_of<Op>::type *out;
    int rows, cols;
    int tiles_c;     // tiles per row of tiles
    int n_tiles;
    int xcd_chunk;   // > 0: tiles are dealt to the 8 XCDs in contiguous chunks of this many
    int pitch;       // LDS tile pitch, in staged elements
    int plane;       // elements per LDS plane (tile rows x pitch)
    unsigned stage_magic;   // ceil(2^32 / items per staged row): tid / items by one multiply
    int vec_ok;      // rows of `in` / `out` start at multiples of a work-item's load / store width and cols % CC == 0
    int nt_store;    // vector stores of output cells are non-temporal
    typename Op::T pad;
    float scalar0;
    Halo halo;
    WeightStore<Op, Halo> w;
};

__host__ __device__ constexpr int round_up(int x, int m) { return (x + m - 1) / m * m; }
__host__ __device__ constexpr int round_down(int x, int m) { return x / m * m; }

// 16-byte moves between global memory / LDS and register arrays (a load may also be one 4-byte
// word: four byte cells that are widened to floats afterwards).
template <class E, int CNT>
__device__ __forceinline__ void load_vec(E (&dst)[CNT], const E *src) {
    if constexpr (sizeof(E) * CNT == 4) {
        const uint32_t tmp = *reinterpret_cast<const uint32_t *>(src);
        __builtin_memcpy(dst, &tmp, 4);
    } else {
        static_assert(sizeof(E) * CNT % 16 == 0, "vector moves are whole 16-byte words");
        constexpr int NV = sizeof(E) * CNT / 16;
        uint4 tmp[NV];
#pragma unroll
        for (int k = 0; k < NV; ++k) tmp[k] = reinterpret_cast<const uint4 *>(src)[k];
        __builtin_memcpy(dst, tmp, sizeof(tmp));
    }
}
template <class E, int CNT>
__device__ __forceinline__ void store_vec(E *dst, const E (&src)[CNT]) {
    static_assert(sizeof(E) * CNT % 16 == 0, "vector moves are whole 16-byte words");
    constexpr int NV = sizeof(E) * CNT / 16;
    uint4 tmp[NV];
    __builtin_memcpy(tmp, src, sizeof(tmp));
#pragma unroll
    for (int k = 0; k < NV; ++k) reinterpret_cast<uint4 *>(dst)[k] = tmp[k];
}
// The same to global memory, optionally as non-temporal stores: output cells are not read again
// by the launch that writes them, and on matrices beyond the caches keeping them out of the way
// of the input pays (measured on a plain copy: +20 % on 256 MiB, nothing on 64 MiB).
typedef unsigned int nt_word4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_word4(void *dst, uint4 v, bool nt) {
    if (nt) {
        nt_word4 t;
        t.x = v.x, t.y = v.y, t.z = v.z, t.w = v.w;
        __builtin_nontemporal_store(t, reinterpret_cast<nt_word4 *>(dst));
    } else {
        *reinterpret_cast<uint4 *>(dst) = v;
    }
}
template <class E, int CNT>
__device__ __forceinline__ void store_out_vec(E *dst, const E (&src)[CNT], bool nt) {
    static_assert(sizeof(E) * CNT % 16 == 0, "vector moves are whole 16-byte words");
    constexpr int NV = sizeof(E) * CNT / 16;
    uint4 tmp[NV];
    __builtin_memcpy(tmp, src, sizeof(tmp));
#pragma unroll
    for (int k = 0; k < NV; ++k) store_word4(reinterpret_cast<uint4 *>(dst) + k, tmp[k], nt);
}

// What a cell keeps while one row of its region goes by (operators that fold a row at a time).
struct NoRowState {};
template <class Op, bool = Op::kRowFold>
struct row_state_of { using type = NoRowState; };
template <class Op>
struct row_state_of<Op, true> { using type = typename Op::RowState; };

// Cross-lane moves inside a wavefront: the value the lane one below / one above holds.
// (Lane 0 has no lane below and lane 63 none above; they get 0 - the move's bound control -
// and must look elsewhere.)
__device__ __forceinline__ uint32_t from_lane_below(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x138 /* wave_shr:1 */, 0xf, 0xf, true);
}
__device__ __forceinline__ uint32_t from_lane_above(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x130 /* wave_shl:1 */, 0xf, 0xf, true);
}

// Columns staged left / right of the tile: the border region's extent, widened to whole
// 16-byte vectors when the work-items move vectors.
template <int CC>
__host__ __device__ constexpr int staged_halo(int h) { return CC == 1 ? h : round_up(h, CC); }

// Stages `n_rows` rows of a tile into LDS with border resolution (Section 2).  Tile row i is
// matrix row row_first + i, tile column j is matrix column col_first + j; each plane of the
// staged values has `pitch` elements per row.  The rows are walked as one linear sequence of
// 16-byte vectors (single elements when CC = 1), work-item k taking items k, k + n, k + 2n, ...
// so that the halo columns cost a fraction of a pass rather than a whole extra pass with most
// lanes idle.  Vectors starting at or beyond matrix column `col_end` are not needed and skipped.
// `magic` = ceil(2^32 / (pitch / CC)) turns the one division into a multiply.
template <class Op, int B, int CC>
__device__ __forceinline__ void stage_tile(typename Op::L *tile, int plane, int pitch, const typename Op::T *in,
                                           int rows, int cols, int row_first, int col_first, int n_rows,
                                           int col_end, typename Op::T pad, int vec_ok, unsigned magic, int tid,
                                           int nthreads) {
    using T = typename Op::T;
    using L = typename Op::L;
    constexpr int NP = Op::kPlanes;
    const int n_items = pitch / CC;   // per staged row
    int i = (int)__umulhi((unsigned)tid, magic);
    int q = tid - i * n_items;
    const int di = (int)__umulhi((unsigned)nthreads, magic), dq = nthreads - di * n_items;
    // Vectors are taken kBatch at a time: the loads of a batch are all issued before the first of
    // them is waited for and written to LDS, so a work-item with several items pays one memory
    // round trip per batch, not one per item.  (Single elements gain nothing from it.)
    constexpr int kBatch = CC == 1 ? 1 : 4;
    while (i < n_rows) {
        T v[kBatch][CC];
        int at_i[kBatch], at_q[kBatch];
        bool have[kBatch];
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            at_i[b] = i;
            at_q[b] = q;
            have[b] = i < n_rows;
            if (have[b]) {
                const int gr = resolve<B>(row_first + i, rows);
                if constexpr (CC == 1) {
                    const int gc = resolve<B>(col_first + q, cols);
                    v[b][0] = (gr < 0 || gc < 0) ? pad : in[(size_t)gr * cols + gc];
                } else {
                    const int gc0 = col_first + q * CC;
                    have[b] = gc0 < col_end;
                    if (have[b]) {
                        if (gr >= 0 && vec_ok && gc0 >= 0 && gc0 + CC <= cols) {
                            load_vec(v[b], in + (size_t)gr * cols + gc0);
                        } else {
#pragma unroll
                            for (int k = 0; k < CC; ++k) {
                                const int gc = resolve<B>(gc0 + k, cols);
                                v[b][k] = (gr < 0 || gc < 0) ? pad : in[(size_t)gr * cols + gc];
                            }
                        }
                    }
                }
            }
            i += di;
            q += dq;
            if (q >= n_items) {
                q -= n_items;
                ++i;
            }
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            if (!have[b]) continue;
            if constexpr (CC == 1) {
                L sv[NP];
                Op::stage(v[b][0], sv);
#pragma unroll
                for (int p = 0; p < NP; ++p) tile[p * plane + at_i[b] * pitch + at_q[b]] = sv[p];
            } else {
                L sv[NP][CC];
                Op::template stage_vec<CC>(v[b], sv);
#pragma unroll
                for (int p = 0; p < NP; ++p) store_vec(tile + p * plane + at_i[b] * pitch + at_q[b] * CC, sv[p]);
            }
        }
    }
}

template <class Op, int B, class Halo, int CR, int CC, int MAXT>
__global__ __launch_bounds__(MAXT) void tile_kernel(const TileArgs<Op, Halo> a) {
    using O = typename out_type_of<Op>::type;
    using L = typename Op::L;
    constexpr int NP = Op::kPlanes;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    L *tile = reinterpret_cast<L *>(lds_raw);   // NP planes of a.plane elements each

    const int wr = blockDim.y, wc = blockDim.x;
    const int tx = threadIdx.x, ty = threadIdx.y;

    int t = blockIdx.x;
    if (a.xcd_chunk > 0) t = (t & 7) * a.xcd_chunk + (t >> 3);
    if (t >= a.n_tiles) return;
    const int tile_r = t / a.tiles_c, tile_c = t - tile_r * a.tiles_c;

    const Halo h = a.halo;
    const int hn = h.n(), hs = h.s(), he = h.e(), hw = h.w();
    const int th = wr * CR, tw = wc * CC;
    const int r0 = tile_r * th, c0 = tile_c * tw;
    const int hwa = staged_halo<CC>(hw);
    const int pitch = a.pitch;
    const int rows = a.rows, cols = a.cols;
    // the whole tile height is staged, also where the last tile hangs over the matrix edge (those
    // rows resolve like any other out-of-matrix row): no window row ever needs a range check
    const int TH = th + hn + hs;

    stage_tile<Op, B, CC>(tile, a.plane, pitch, a.in, rows, cols, r0 - hn, c0 - hwa, TH, cols + he, a.pad,
                          a.vec_ok, a.stage_magic, ty * wc + tx, wr * wc);
    __syncthreads();

    // ---- fold the customising function over the border region ----------------------------
    const int lr0 = ty * CR, lc0 = tx * CC;
    if (r0 + lr0 >= rows || c0 + lc0 >= cols) return;

    typename Op::State st[CR][CC];
#pragma unroll
    for (int cr = 0; cr < CR; ++cr)
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) Op::init(st[cr][cc]);

    if constexpr (Halo::kStatic) {
        constexpr int N = Halo::N, S = Halo::S, E = Halo::E, W = Halo::W;
        constexpr int HWA = staged_halo<CC>(W);
        constexpr int VL = CC == 1 ? 1 : (16 / (int)sizeof(L) < 1 ? 1 : 16 / (int)sizeof(L));
        constexpr int LO = round_down(HWA - W, VL);
        constexpr int HI = round_up(HWA + CC + E, VL);
        constexpr int WW = HI - LO;
        constexpr int WCOLS = E + W + 1;
        // window rows stream through registers; row wi feeds cell-row cr with dr = wi - N - cr
#pragma unroll
        for (int wi = 0; wi < CR + N + S; ++wi) {
            L row[NP][WW];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const L *src = tile + p * a.plane + (lr0 + wi) * pitch + lc0 + LO;
                if constexpr (CC == 1) {
#pragma unroll
                    for (int k = 0; k < WW; ++k) row[p][k] = src[k];
                } else {
                    load_vec(row[p], src);
                }
            }
            auto value_at = [&](int i) {
                L parts[NP];
#pragma unroll
                for (int p = 0; p < NP; ++p) parts[p] = row[p][i];
                return Op::combine(parts);
            };
#pragma unroll
            for (int cr = 0; cr < CR; ++cr) {
                const int dr = wi - N - cr;
                if (dr < -N || dr > S) continue;
#pragma unroll
                for (int cc = 0; cc < CC; ++cc)
                    fold_row<Op>(
                        st[cr][cc], dr, dr + N, N + S + 1, W, E, [&](int dc) { return a.w[(dr + N) * WCOLS + dc + W]; },
                        [&](int dc) { return value_at(HWA - LO + cc + dc); });
            }
        }
    } else {
        // Run-time region: the cells of a work-item walk through the region together, so that a
        // tap's weight (a uniform, scalar load) is fetched once for all of them; every cell still
        // sees its taps in row-major order.
        const int wcols = he + hw + 1, wrows = hn + hs + 1;
        constexpr bool kVec = CC > 1 && (sizeof(L) * CC) % 16 == 0;
        if constexpr (kVec) {
            // Columns are counted from the staged tile's aligned west edge (column kk of the window
            // of cell (cr, 0) is dc = kk - hwa) and taken CC at a time: the cells of a row need
            // window columns kk .. kk + CC - 1 for tap kk, i.e. two aligned vectors per chunk, of
            // which one is the previous chunk's.  Taps outside [k_lo, k_hi] are not in the region.
            const int k_lo = hwa - hw, k_hi = hwa + he;
            const L *west[CR];
#pragma unroll
            for (int cr = 0; cr < CR; ++cr) west[cr] = tile + (lr0 + cr) * pitch + lc0;
            for (int i = 0; i < wrows; ++i) {
                const int dr = i - hn;
                [[maybe_unused]] typename row_state_of<Op>::type rs[CR][CC] = {};
                L va[CR][NP][CC], vb[CR][NP][CC];
                auto load_chunk = [&](L (&v)[CR][NP][CC], int j) {
#pragma unroll
                    for (int cr = 0; cr < CR; ++cr)
#pragma unroll
                        for (int p = 0; p < NP; ++p) load_vec(v[cr][p], west[cr] + p * a.plane + i * pitch + CC * j);
                };
                // taps CC * j .. CC * j + CC - 1: `lo` holds window columns CC * j .., `hi` the next CC
                auto chunk = [&](const L (&lo)[CR][NP][CC], L (&hi)[CR][NP][CC], int j) {
                    if (CC * j + 1 <= k_hi) load_chunk(hi, j + 1);
#pragma unroll
                    for (int t = 0; t < CC; ++t) {
                        const int kk = CC * j + t;
                        if (kk < k_lo || kk > k_hi) continue;
                        const auto w = a.w[i * wcols + kk - k_lo];
#pragma unroll
                        for (int cr = 0; cr < CR; ++cr)
#pragma unroll
                            for (int cc = 0; cc < CC; ++cc) {
                                L parts[NP];
#pragma unroll
                                for (int p = 0; p < NP; ++p)
                                    parts[p] = t + cc < CC ? lo[cr][p][(t + cc) % CC] : hi[cr][p][(t + cc) % CC];
                                if constexpr (Op::kRowFold)
                                    Op::row_visit(st[cr][cc], rs[cr][cc], kk - k_lo, w, Op::combine(parts));
                                else
                                    Op::visit(st[cr][cc], dr, kk - hwa, w, Op::combine(parts));
                            }
                    }
                };
                int j = k_lo / CC;
                load_chunk(va, j);
                for (; CC * j <= k_hi; j += 2) {
                    chunk(va, vb, j);
                    if (CC * (j + 1) <= k_hi) chunk(vb, va, j + 1);
                }
                if constexpr (Op::kRowFold) {
#pragma unroll
                    for (int cr = 0; cr < CR; ++cr)
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc) Op::row_end(st[cr][cc], rs[cr][cc], wcols, i, wrows);
                }
            }
        } else {
            const L *nw[CR];      // the north-west corner of the region of cell (cr, 0)
#pragma unroll
            for (int cr = 0; cr < CR; ++cr) nw[cr] = tile + (lr0 + cr) * pitch + (hwa - hw) + lc0;
            for (int i = 0; i < wrows; ++i) {
                const int dr = i - hn;
                [[maybe_unused]] typename row_state_of<Op>::type rs[CR][CC] = {};
                for (int k = 0; k < wcols; ++k) {
                    const auto w = a.w[i * wcols + k];
#pragma unroll
                    for (int cr = 0; cr < CR; ++cr)
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc) {
                            L parts[NP];
#pragma unroll
                            for (int p = 0; p < NP; ++p) parts[p] = nw[cr][p * a.plane + i * pitch + k + cc];
                            if constexpr (Op::kRowFold)
                                Op::row_visit(st[cr][cc], rs[cr][cc], k, w, Op::combine(parts));
                            else
                                Op::visit(st[cr][cc], dr, k - hw, w, Op::combine(parts));
                        }
                }
                if constexpr (Op::kRowFold) {
#pragma unroll
                    for (int cr = 0; cr < CR; ++cr)
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc) Op::row_end(st[cr][cc], rs[cr][cc], wcols, i, wrows);
                }
            }
        }
    }

    // ---- store ------------------------------------------------------------------------------
#pragma unroll
    for (int cr = 0; cr < CR; ++cr) {
        const int r = r0 + lr0 + cr;
        if (r >= rows) break;
        O res[CC];
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) res[cc] = Op::finish(st[cr][cc], a.scalar0);
        O *dst = a.out + (size_t)r * cols + c0 + lc0;
        if constexpr (CC > 1) {
            if (a.vec_ok && c0 + lc0 + CC <= cols) {
                store_out_vec(dst, res, a.nt_store != 0);
                continue;
            }
        }
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
            if (c0 + lc0 + cc < cols) dst[cc] = res[cc];
    }
}

}  // namespace sk
