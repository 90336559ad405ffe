// Temporal blocking for iterated stencils with the 1/1/1/1 border region: one launch
// advances the matrix by `depth` applications (1 <= depth <= 4).  The workgroup stages its tile
// plus a border region `depth` cells deep (rows) and one 16-byte vector wide (columns) in local
// memory, then ping-pongs between two LDS buffers: after application k the values within k
// cells of the staged rim are stale, and after `depth` applications exactly the tile itself is
// still right and is written out.  HBM traffic per application falls by the depth; the price is
// the redundant rim work and one barrier per application.
//
// Out-of-matrix positions inside the staged tile are re-resolved after every application: a
// periodic copy evolves like its original (nothing to do), a padded position is set back to the
// padding value, a clamped position is copied from the nearest in-matrix cell's new value.
// The per-cell arithmetic is the same fold as in the single-application kernels, so results
// are bit-identical to `depth` separate launches.
#pragma once
#include "direct_kernel.h"
#include "tile_kernel.h"

namespace sk {

// Rows of an item handled by one work-item per pass through a time step: the window rolls down
// over them, so R + 2 LDS rows are read for R rows written.
constexpr int kTemporalRows = 2;

// Four cells of one LDS row plus the cells west and east of them.  Work-items with consecutive
// ids hold consecutive vectors of a row, so the two neighbours normally sit in the adjacent
// lanes; where they do not (first / last lane of a wavefront, or the caller says so) the
// adjoining LDS words are read instead.  At the two ends of a staged row the "neighbour" is
// whatever lies beside it in memory - values that only ever reach rim cells that are stale.
struct QuadRow {
    float v[4];
    float w, e;
};
__device__ __forceinline__ QuadRow load_quad_row(const float *rp, bool west_in_lane, bool east_in_lane) {
    QuadRow r;
    load_vec(r.v, rp);
    r.w = __uint_as_float(from_lane_below(__float_as_uint(r.v[3])));
    r.e = __uint_as_float(from_lane_above(__float_as_uint(r.v[0])));
    if (!west_in_lane) r.w = rp[-1];
    if (!east_in_lane) r.e = rp[4];
    return r;
}

// One application for the four cells of `mid`, given the rows above and below.
template <class Op>
__device__ __forceinline__ void temporal_quad(typename Op::T (&res)[4], const QuadRow &up, const QuadRow &mid,
                                              const QuadRow &dn, const WeightStore<Op, HaloC<1, 1, 1, 1>> &w,
                                              float scalar0) {
    typename Op::State st[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) Op::init(st[cc]);
#pragma unroll
    for (int dr = -1; dr <= 1; ++dr) {
        const QuadRow &q = dr < 0 ? up : (dr == 0 ? mid : dn);
        const float row[6] = {q.w, q.v[0], q.v[1], q.v[2], q.v[3], q.e};
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
            fold_row<Op>(
                st[cc], dr, dr + 1, 3, 1, 1, [&](int dc) { return w[(dr + 1) * 3 + dc + 1]; },
                [&](int dc) { return row[1 + cc + dc]; });
    }
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) res[cc] = Op::finish(st[cc], scalar0);
}

template <class Op, int B, int CR, int MAXT>
__global__ __launch_bounds__(MAXT) void temporal_kernel(const TileArgs<Op, HaloC<1, 1, 1, 1>> a, const int depth) {
    using T = typename Op::T;
    static_assert(Op::kPlanes == 1 && sizeof(T) == 4 && sizeof(typename Op::L) == 4, "fp32, one plane");
    constexpr int CC = 4, HC = 4;   // cells per vector; staged columns each side of the tile
    constexpr int R = kTemporalRows;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    // [one spare vector][buffer][buffer][one spare vector]: the reads one word before a row's
    // first vector and one word after its last stay inside the allocation
    float *src = reinterpret_cast<float *>(lds_raw) + CC;
    float *dst = src + a.plane;

    const int wr = blockDim.y, wc = blockDim.x;
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int tid = ty * wc + tx, nthreads = wr * wc;
    const int lane = tid & 63;

    int t = blockIdx.x;
    if (a.xcd_chunk > 0) t = (t & 7) * a.xcd_chunk + (t >> 3);
    if (t >= a.n_tiles) return;
    const int tile_r = t / a.tiles_c, tile_c = t - tile_r * a.tiles_c;
    const int rows = a.rows, cols = a.cols, pitch = a.pitch, nq = pitch / CC;
    const int th = wr * CR, tw = wc * CC;
    const int r0 = tile_r * th, c0 = tile_c * tw;
    const int row_first = r0 - depth, col_first = c0 - HC;
    const int ER = min(th, rows - r0) + 2 * depth;   // staged rows in use

    stage_tile<Op, B, CC>(src, a.plane, pitch, a.in, rows, cols, row_first, col_first, ER, cols + HC, a.pad,
                          a.vec_ok, a.stage_magic, tid, nthreads);
    __syncthreads();

    // does the staged tile reach outside the matrix?  (same answer for the whole workgroup)
    const bool at_border = row_first < 0 || row_first + ER > rows || col_first < 0 || col_first + pitch > cols;
    // items of a time step: groups of R rows x vectors of a row, walked linearly by work-item id;
    // the next item sits in the next lane unless this is the wavefront's or the workgroup's last
    const bool next_in_lane = lane < 63 && tid + 1 < nthreads;
    const int dg = (int)__umulhi((unsigned)nthreads, a.stage_magic), dq = nthreads - dg * nq;

    for (int k = 1; k < depth; ++k) {
        // application k on tile rows [k, ER - k): everything that can still be right
        const int n_groups = (ER - 2 * k + R - 1) / R;
        int g = (int)__umulhi((unsigned)tid, a.stage_magic);
        int q = tid - g * nq;
        int off = (k + g * R) * pitch + q * CC;   // walks with (g, q)
        while (g < n_groups) {
            const int i0 = k + g * R;
            const float *rp = src + off;
            QuadRow up = load_quad_row(rp - pitch, lane > 0, next_in_lane);
            QuadRow mid = load_quad_row(rp, lane > 0, next_in_lane);
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const int i = i0 + rr;
                if (i >= ER - k) break;
                const QuadRow dn = load_quad_row(rp + (rr + 1) * pitch, lane > 0, next_in_lane);
                T res[CC];
                temporal_quad<Op>(res, up, mid, dn, a.w, a.scalar0);
                if (B == kConstant && at_border) {
                    const int gr = row_first + i;
#pragma unroll
                    for (int cc = 0; cc < CC; ++cc) {
                        const int gc = col_first + q * CC + cc;
                        if ((unsigned)gr >= (unsigned)rows || (unsigned)gc >= (unsigned)cols) res[cc] = a.pad;
                    }
                }
                store_vec(dst + off + rr * pitch, res);
                up = mid;
                mid = dn;
            }
            g += dg;
            q += dq;
            off += dg * R * pitch + dq * CC;
            if (q >= nq) {   // (g, q) -> (g + 1, q - nq)
                q -= nq;
                ++g;
                off += (R - 1) * pitch;
            }
        }
        __syncthreads();
        if (B == kClamp && at_border) {
            // clamped positions take the new value of the nearest in-matrix cell
            for (int idx = tid; idx < (ER - 2 * k) * pitch; idx += nthreads) {
                const int i2 = k + idx / pitch, j2 = idx % pitch;
                const int gr = row_first + i2, gc = col_first + j2;
                if ((unsigned)gr >= (unsigned)rows || (unsigned)gc >= (unsigned)cols) {
                    const int ci = min(max(gr, 0), rows - 1) - row_first, cj = min(max(gc, 0), cols - 1) - col_first;
                    // the nearest cell lies inside the staged tile whenever this position can
                    // still influence the tile's own cells; stale rim positions may skip it
                    if (ci >= k && ci < ER - k && cj >= 0 && cj < pitch) dst[i2 * pitch + j2] = dst[ci * pitch + cj];
                }
            }
            __syncthreads();
        }
        float *tmp = src;
        src = dst;
        dst = tmp;
    }

    // last application: the tile's own cells, straight to global memory.  Work-item (ty, tx) owns
    // rows ty*CR.. and vector 1 + tx; its row neighbours are the adjacent lanes except at the two
    // ends of the workgroup's row.
    const int c = c0 + tx * CC;
    const bool west_in_lane = lane > 0 && tx > 0, east_in_lane = lane < 63 && tx + 1 < wc;
    const float *rp = src + (depth + ty * CR) * pitch + (1 + tx) * CC;
    QuadRow up = load_quad_row(rp - pitch, west_in_lane, east_in_lane);
    QuadRow mid = load_quad_row(rp, west_in_lane, east_in_lane);
#pragma unroll
    for (int cr = 0; cr < CR; ++cr) {
        const int r = r0 + ty * CR + cr;
        // (every lane keeps loading, so that lanes still at work find their neighbours' values)
        const QuadRow dn = load_quad_row(rp + (cr + 1) * pitch, west_in_lane, east_in_lane);
        if (r < rows && c < cols) {
            T res[CC];
            temporal_quad<Op>(res, up, mid, dn, a.w, a.scalar0);
            T *out = a.out + (size_t)r * cols + c;
            if (a.vec_ok && c + CC <= cols) {
                store_out_vec(out, res, a.nt_store != 0);
            } else {
#pragma unroll
                for (int cc = 0; cc < CC; ++cc)
                    if (c + cc < cols) out[cc] = res[cc];
            }
        }
        up = mid;
        mid = dn;
    }
}

// ---- Game of Life, several generations per launch ------------------------------------------
// Same scheme on packed bytes: 16 cells per vector, a rim of `depth` rows and one vector.

// The 16 cells at `p` (a 16-byte aligned position in an LDS buffer) as a LifeRow; the cells west
// and east of them come from the adjacent lanes, or from the adjoining LDS words where those
// lanes do not hold them (see load_quad_row).
__device__ __forceinline__ LifeRow life_lds_row(const uint8_t *p, bool west_in_lane, bool east_in_lane) {
    LifeRow x;
    const uint4 v = *reinterpret_cast<const uint4 *>(p);
    x.w[0] = v.x; x.w[1] = v.y; x.w[2] = v.z; x.w[3] = v.w;
    x.l = from_lane_below(x.w[3]) >> 24;
    x.r = from_lane_above(x.w[0]) & 0xffu;
    if (!west_in_lane) x.l = *reinterpret_cast<const uint32_t *>(p - 4) >> 24;
    if (!east_in_lane) x.r = *reinterpret_cast<const uint32_t *>(p + 16) & 0xffu;
    return x;
}

template <int B, int CR, int MAXT>
__global__ __launch_bounds__(MAXT) void life_temporal_kernel(const TileArgs<OpLife, HaloC<1, 1, 1, 1>> a,
                                                             const int depth) {
    constexpr int CC = 16, HC = 16;
    constexpr int R = kTemporalRows;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint8_t *src = lds_raw + CC;   // one spare vector before and after the two buffers
    uint8_t *dst = src + a.plane;

    const int wr = blockDim.y, wc = blockDim.x;
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int tid = ty * wc + tx, nthreads = wr * wc;
    const int lane = tid & 63;

    int t = blockIdx.x;
    if (a.xcd_chunk > 0) t = (t & 7) * a.xcd_chunk + (t >> 3);
    if (t >= a.n_tiles) return;
    const int tile_r = t / a.tiles_c, tile_c = t - tile_r * a.tiles_c;
    const int rows = a.rows, cols = a.cols, pitch = a.pitch, nq = pitch / CC;
    const int th = wr * CR, tw = wc * CC;
    const int r0 = tile_r * th, c0 = tile_c * tw;
    const int row_first = r0 - depth, col_first = c0 - HC;
    const int ER = min(th, rows - r0) + 2 * depth;

    stage_tile<OpLife, B, CC>(src, a.plane, pitch, a.in, rows, cols, row_first, col_first, ER, cols + HC, a.pad,
                              a.vec_ok, a.stage_magic, tid, nthreads);
    __syncthreads();

    const bool at_border = row_first < 0 || row_first + ER > rows || col_first < 0 || col_first + pitch > cols;
    const bool next_in_lane = lane < 63 && tid + 1 < nthreads;
    const int dg = (int)__umulhi((unsigned)nthreads, a.stage_magic), dq = nthreads - dg * nq;

    for (int k = 1; k < depth; ++k) {
        const int n_groups = (ER - 2 * k + R - 1) / R;
        int g = (int)__umulhi((unsigned)tid, a.stage_magic);
        int q = tid - g * nq;
        int off = (k + g * R) * pitch + q * CC;
        while (g < n_groups) {
            const int i0 = k + g * R;
            const uint8_t *rp = src + off;
            LifeRow up = life_lds_row(rp - pitch, lane > 0, next_in_lane);
            LifeRow mid = life_lds_row(rp, lane > 0, next_in_lane);
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const int i = i0 + rr;
                if (i >= ER - k) break;
                const LifeRow dn = life_lds_row(rp + (rr + 1) * pitch, lane > 0, next_in_lane);
                uint32_t o[4];
                life_rule(o, up, mid, dn);
                if (B == kConstant && at_border) {
                    const int gr = row_first + i;
#pragma unroll
                    for (int b = 0; b < CC; ++b) {
                        const int gc = col_first + q * CC + b;
                        if ((unsigned)gr >= (unsigned)rows || (unsigned)gc >= (unsigned)cols)
                            o[b >> 2] = (o[b >> 2] & ~(0xffu << (8 * (b & 3)))) | ((uint32_t)a.pad << (8 * (b & 3)));
                    }
                }
                *reinterpret_cast<uint4 *>(dst + off + rr * pitch) = make_uint4(o[0], o[1], o[2], o[3]);
                up = mid;
                mid = dn;
            }
            g += dg;
            q += dq;
            off += dg * R * pitch + dq * CC;
            if (q >= nq) {
                q -= nq;
                ++g;
                off += (R - 1) * pitch;
            }
        }
        __syncthreads();
        if (B == kClamp && at_border) {
            for (int idx = tid; idx < (ER - 2 * k) * pitch; idx += nthreads) {
                const int i2 = k + idx / pitch, j2 = idx % pitch;
                const int gr = row_first + i2, gc = col_first + j2;
                if ((unsigned)gr >= (unsigned)rows || (unsigned)gc >= (unsigned)cols) {
                    const int ci = min(max(gr, 0), rows - 1) - row_first, cj = min(max(gc, 0), cols - 1) - col_first;
                    if (ci >= k && ci < ER - k && cj >= 0 && cj < pitch) dst[i2 * pitch + j2] = dst[ci * pitch + cj];
                }
            }
            __syncthreads();
        }
        uint8_t *tmp = src;
        src = dst;
        dst = tmp;
    }

    const int c = c0 + tx * CC;
    const bool west_in_lane = lane > 0 && tx > 0, east_in_lane = lane < 63 && tx + 1 < wc;
    const uint8_t *rp = src + (depth + ty * CR) * pitch + (1 + tx) * CC;
    LifeRow up = life_lds_row(rp - pitch, west_in_lane, east_in_lane);
    LifeRow mid = life_lds_row(rp, west_in_lane, east_in_lane);
#pragma unroll
    for (int cr = 0; cr < CR; ++cr) {
        const int r = r0 + ty * CR + cr;
        const LifeRow dn = life_lds_row(rp + (cr + 1) * pitch, west_in_lane, east_in_lane);
        if (r < rows && c < cols) {
            uint32_t o[4];
            life_rule(o, up, mid, dn);
            uint8_t *out = a.out + (size_t)r * cols + c;
            if (a.vec_ok && c + CC <= cols) {
                store_word4(out, make_uint4(o[0], o[1], o[2], o[3]), a.nt_store != 0);
            } else {
#pragma unroll
                for (int b = 0; b < CC; ++b)
                    if (c + b < cols) out[b] = (uint8_t)(o[b >> 2] >> (8 * (b & 3)));
            }
        }
        up = mid;
        mid = dn;
    }
}

}  // namespace sk
