// The marching kernel of march_kernel.h for border regions that are only known at launch.
//
// A wavefront that marches down the matrix keeps one partial result per output row in flight, in
// registers, so the number of rows in flight has to be a compile-time number.  This kernel is
// compiled for a largest region NM / SM / EM / WM and serves every region within it.  Partial
// results sit in a chain: link k holds the output row that has received its region rows 0 .. k-1;
// an arriving input row is region row k of link k, whose sum then moves on to link k+1 (the links
// are taken from the last to the first) or, from the region's last row, to the output matrix.
// The code of a step therefore does not depend on which step it is, and the loop over the steps
// is unrolled only as far as rows are requested ahead.  Links the actual region does not have,
// or whose output row belongs to another wavefront, are skipped by one wavefront-uniform bit test
// each.  A lane's row neighbours cannot come from
// cross-lane moves here (their distances are compile-time numbers): the wavefront writes the row
// to local memory and every lane reads the window that starts at its region's west edge, so the
// taps of a region row are the window's first E + W + 1 positions: the kernel is compiled once
// for every such number of columns WC, and only how they divide into east and west is left to the
// launch.  The weights come from a copy of the table in local memory as well, one copy per
// wavefront (no barrier anywhere), a region row's weights requested two rows ahead of their use.  A cell sees exactly the taps of its region, north to south and west to east: the fold,
// and the output bits, of every other mapping.  For customising functions that fold tap by tap
// (the weighted sums).
#pragma once
#include "march_kernel.h"

namespace sk {

// Largest region of a masked kernel (N, S, E, W) plus the actual one.
template <int NM, int SM, int EM, int WM>
struct HaloM {
    static constexpr bool kStatic = false;
    static constexpr bool kMasked = true;
    static constexpr int N = NM, S = SM, E = EM, W = WM;
    int n_, s_, e_, w_;
    __host__ __device__ int n() const { return n_; }
    __host__ __device__ int s() const { return s_; }
    __host__ __device__ int e() const { return e_; }
    __host__ __device__ int w() const { return w_; }
};

template <class Op, int B, class Halo, int WC, bool FAST, int MAXT>
__device__ __forceinline__ void march_masked_body(const TileArgs<Op, Halo> &a, const int H) {
    using T = typename Op::T;
    using L = typename Op::L;
    static_assert(!Op::kRowFold && Op::kPlanes == 1, "functions that fold tap by tap");
    static_assert(sizeof(T) == 4 && sizeof(L) == 4, "32-bit elements");
    constexpr int CC = 4;
    constexpr int EM = Halo::E, WM = Halo::W;
    // The row in local memory: cell j of lane l at j * kPlane + kPadLanes + l, so that the lanes' reads of one
    // window position fall on consecutive banks (a cell's own position in the row, 4 l + j, would put them four
    // banks apart: four lanes per bank).
    constexpr int kPadLanes = 2, kPlane = 64 + 2 * kPadLanes;
    static_assert(EM <= kPadLanes * CC && WM <= kPadLanes * CC, "a lane's window stays within the row and its pads");
    constexpr int RM = Halo::N + Halo::S + 1;     // links of the chain
    static_assert(WC >= 1 && WC <= EM + WM + 1, "columns of a region within the largest one");
    static_assert(RM < 32, "one bit per link");
    constexpr int kTable = (RM * WC + 63) / 64 * 64;
    constexpr int kWindow = WC + CC - 1;
    constexpr int P = 4;                          // input rows requested ahead

    // the actual region: the same in every lane
    const int n = a.halo.n(), e = a.halo.e(), w = a.halo.w();
    const int r = n + a.halo.s() + 1;             // its rows
    const int rim_w = march_rim(w), vectors = march_vectors(w, e);

    const int tid = (int)threadIdx.y * (int)blockDim.x + (int)threadIdx.x;
    const int lane = tid & 63;
    const int waves_per_block = ((int)blockDim.x * (int)blockDim.y) >> 6;
    int b = (int)blockIdx.x;
    if (a.xcd_chunk > 0) b = (b & 7) * a.xcd_chunk + (b >> 3);
    const int wave = __builtin_amdgcn_readfirstlane(b * waves_per_block + (tid >> 6));
    if (wave >= a.n_tiles) return;

    // this wavefront's copy of the weights (entry k * WC + i: region row k, i-th column from the west) and its row
    __shared__ float tables[MAXT / 64][kTable];
    __shared__ L row_buffers[MAXT / 64][CC * kPlane];
    const int wave_in_block = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *const table = tables[wave_in_block];
    L *const row_buffer = row_buffers[wave_in_block];
#pragma unroll
    for (int base = 0; base < kTable; base += 64) {
        const int idx = base + lane;
        table[idx] = idx < r * WC ? a.w[idx] : 0.0f;
    }
    L *const own = row_buffer + kPadLanes + lane;             // this lane's four cells: own[j * kPlane]
    // the window from the west edge of the first cell's region: position i is the row's cell 4 lane + i - w, and
    // positions four apart are neighbours in local memory
    const L *window[CC];
#pragma unroll
    for (int i = 0; i < CC; ++i) {
        const int j = (i - w) & (CC - 1), q = (i - w - j) >> 2;
        window[i] = own + j * kPlane + q;
    }

    const int seg = wave / a.tiles_c, strip = wave - seg * a.tiles_c;
    const int rows = a.rows, cols = a.cols;
    const int r0 = seg * H;
    const int gc0 = (strip * vectors - rim_w + lane) * CC;    // first of this lane's four columns
    const bool writes = lane >= rim_w && lane < rim_w + vectors && gc0 < cols;

    const bool outside = (unsigned)gc0 >= (unsigned)cols;
    int vcol = gc0;
    if (outside) vcol = B == kWrap ? resolve<B>(gc0, cols) : (gc0 < 0 ? 0 : cols - CC);
    const bool edge_wave = __any(outside) != 0;
    const unsigned in_off = (unsigned)vcol * (unsigned)sizeof(T);
    const unsigned out_off = (unsigned)gc0 * (unsigned)sizeof(T);
    int col[CC];
#pragma unroll
    for (int j = 0; j < CC; ++j) col[j] = resolve<B>(gc0 + j, cols);
    const bool wanted = gc0 < cols + e;

    // input row r0 - n + t arrives at step t
    const int kSteps = H + r - 1;

    auto load_row = [&](int t, T (&v)[CC]) {
        const int tt = t < kSteps ? t : kSteps - 1;
        const int gr = resolve<B>(r0 - n + tt, rows);
        if (FAST) {
            const char *rowp = reinterpret_cast<const char *>(a.in + (size_t)(gr < 0 ? 0 : gr) * cols);
            load_vec(v, reinterpret_cast<const T *>(rowp + in_off));
        } else {
#pragma unroll
            for (int j = 0; j < CC; ++j)
                v[j] = (gr >= 0 && wanted && col[j] >= 0) ? a.in[(size_t)gr * cols + col[j]] : a.pad;
        }
    };
    auto fix_row = [&](int t, T (&v)[CC]) {
        const bool row_outside = B == kConstant && (unsigned)(r0 - n + t) >= (unsigned)rows;
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
    // what one lane wrote to local memory, the others of its wavefront may read after this
    auto wave_sync = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    T pf[P][CC];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        load_row(p, pf[p]);
        __builtin_amdgcn_sched_barrier(0);      // in consumption order (see march_kernel.h)
    }
    typename Op::State link[RM + 1][CC];        // link[0] is never read: a sum starts from Op::init
#pragma unroll
    for (int k = 0; k <= RM; ++k)
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) Op::init(link[k][cc]);

    // steps beyond kSteps (the last pass of the unrolled part) find no output row of the segment
    for (int t0 = 0; t0 < kSteps; t0 += P) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int t = t0 + p;
            fix_row(t, pf[p]);
            L sv[1][CC];
            Op::template stage_vec<CC>(pf[p], sv);
            load_row(t + P, pf[p]);
            // the row as this lane's cells see it: window[i + cc] is cell cc's i-th neighbour from the west
            wave_sync();                        // the last step's reads come first
#pragma unroll
            for (int j = 0; j < CC; ++j) own[j * kPlane] = sv[0][j];
            wave_sync();
            L win[kWindow];
#pragma unroll
            for (int i = 0; i < kWindow; ++i) win[i] = window[i % CC][i / CC];
            // This input row is region row k (0 = northernmost) of output row t - k of the segment.  The links
            // that have something to fold at this step, one bit each: k < r and 0 <= t - k < H.  (Made anew at
            // every step from the region's numbers: compared once for all steps, the outcomes would be kept as
            // lane masks in more scalar registers than there are.)
            int rk = r;
            asm volatile("" : "+s"(rk));
            const int k_end = t + 1 < rk ? t + 1 : rk, k_begin = t - H + 1 > 0 ? t - H + 1 : 0;
            const uint32_t links = k_begin < k_end ? ((~0u >> (32 - (k_end - k_begin))) << k_begin) : 0u;
            // a row's weights are requested kAhead rows ahead, whether the region has those rows or not
            constexpr int kAhead = 2;
            float wk[kAhead + 1][WC];
#pragma unroll
            for (int k = RM - 1; k > RM - 1 - kAhead && k >= 0; --k)
#pragma unroll
                for (int i = 0; i < WC; ++i) wk[k % (kAhead + 1)][i] = table[k * WC + i];
#pragma unroll
            for (int k = RM - 1; k >= 0; --k) {
                if (k >= kAhead) {
#pragma unroll
                    for (int i = 0; i < WC; ++i) wk[(k - kAhead) % (kAhead + 1)][i] = table[(k - kAhead) * WC + i];
                }
                // the region has no such row, or the output row is another wavefront's
                if (!((links >> k) & 1u)) continue;
                typename Op::State(&sum)[CC] = link[k + 1];         // the row's taps carry the sum to the next link
#pragma unroll
                for (int cc = 0; cc < CC; ++cc) {
                    if (k == 0)
                        Op::init(sum[cc]);
                    else
                        sum[cc] = link[k][cc];
                }
#pragma unroll
                for (int i = 0; i < WC; ++i) {
#pragma unroll
                    for (int cc = 0; cc < CC; ++cc) {
                        const L parts[1] = {win[i + cc]};
                        Op::visit(sum[cc], k - n, i - w, wk[k % (kAhead + 1)][i], Op::combine(parts));
                    }
                }
                if (k == rk - 1) {
                    const int gr = r0 + t - k;                      // the output row that is complete now
                    if (gr < rows && writes) {
                        T res[CC];
#pragma unroll
                        for (int cc = 0; cc < CC; ++cc) res[cc] = Op::finish(sum[cc], a.scalar0);
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

template <class Op, int B, class Halo, int WC, bool FAST, int MAXT>
__global__ __launch_bounds__(MAXT) void march_masked_kernel(const TileArgs<Op, Halo> a, const int H) {
    march_masked_body<Op, B, Halo, WC, FAST, MAXT>(a, H);
}

}  // namespace sk
