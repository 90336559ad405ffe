// Game of Life, several generations per launch, with every time level in registers: the packed-
// byte arithmetic of the direct Life kernel on the marching order of the streaming fp32 kernel.
//
// A lane holds WORDS 32-bit words (4 * WORDS cells) of a row; a wavefront's 64 lanes make a strip
// and walk down H + 2 * DEPTH rows.  For each generation k the last three rows of generation
// k - 1 are kept; their byte-wise column sums need only one byte from each neighbouring lane
// (one cross-lane move per side and generation), and the 3x3 block sums, the neighbour counts and
// the rule follow as in the direct kernel.  What a generation computes within k cells of a
// strip's edge is stale after k generations: the outermost ceil(DEPTH / (4 * WORDS)) lanes of
// each side are rim lanes and are not written.  WRAP and CONSTANT borders, as for the fp32 kernel.
#pragma once
#include "tile_kernel.h"

namespace sk {

constexpr int kLifeStreamMaxDepth = 8;
__host__ __device__ constexpr int life_stream_rim(int depth, int words) { return (depth + 4 * words - 1) / (4 * words); }
__host__ __device__ constexpr int life_stream_cols(int depth, int words) {
    return (64 - 2 * life_stream_rim(depth, words)) * 4 * words;
}

template <int WORDS>
__device__ __forceinline__ void load_words(uint32_t (&v)[WORDS], const void *src) {
    if constexpr (WORDS == 1) {
        v[0] = *reinterpret_cast<const uint32_t *>(src);
    } else if constexpr (WORDS == 2) {
        const uint2 t = *reinterpret_cast<const uint2 *>(src);
        v[0] = t.x, v[1] = t.y;
    } else {
        static_assert(WORDS == 4, "1, 2 or 4 words per lane");
        const uint4 t = *reinterpret_cast<const uint4 *>(src);
        v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
    }
}
// (the 16-byte stores can be non-temporal, as in the other kernels; the narrower ones are plain)
template <int WORDS>
__device__ __forceinline__ void store_words(void *dst, const uint32_t (&v)[WORDS], bool nt) {
    if constexpr (WORDS == 1) {
        *reinterpret_cast<uint32_t *>(dst) = v[0];
    } else if constexpr (WORDS == 2) {
        *reinterpret_cast<uint2 *>(dst) = make_uint2(v[0], v[1]);
    } else {
        store_word4(dst, make_uint4(v[0], v[1], v[2], v[3]), nt);
    }
}

// FAST: rows are whole aligned 16-byte vectors, so a lane's cells lie either all inside the matrix
// or all outside it and a row is one load at a per-lane column plus a wavefront-uniform row
// address, issued without a branch.  Otherwise cells are loaded and stored one by one.
template <int B, int DEPTH, int WORDS, bool FAST>
__device__ __forceinline__ void life_stream_body(const TileArgs<OpLife, HaloC<1, 1, 1, 1>> &a, const int H) {
    static_assert(B == kWrap || B == kConstant, "wrap and constant borders only");
    static_assert(DEPTH >= 1 && DEPTH <= kLifeStreamMaxDepth, "generations per launch");
    constexpr int CC = 4 * WORDS;                   // cells per lane
    constexpr int R = 3;                            // rows of a generation kept
    constexpr int PF = 6;                           // input rows in flight = steps per round (a multiple of R)
    constexpr int kRim = life_stream_rim(DEPTH, WORDS);
    constexpr int kCols = life_stream_cols(DEPTH, WORDS);

    const int tid = (int)threadIdx.y * (int)blockDim.x + (int)threadIdx.x;
    const int lane = tid & 63;
    const int waves_per_block = ((int)blockDim.x * (int)blockDim.y) >> 6;
    // a wavefront's index is the same in all its lanes: keep it, and all that follows from it, scalar
    const int wave = __builtin_amdgcn_readfirstlane((int)blockIdx.x * waves_per_block + (tid >> 6));
    if (wave >= a.n_tiles) return;
    const int seg = wave / a.tiles_c, strip = wave - seg * a.tiles_c;
    const int rows = a.rows, cols = a.cols;
    const int r0 = seg * H;
    const int gc0 = strip * kCols - kRim * CC + lane * CC;     // first of this lane's cells
    const bool writes = lane >= kRim && lane < 64 - kRim && gc0 < cols;
    const uint32_t pad_word = (uint32_t)a.pad * 0x01010101u;

    // FAST: the column the lane's load starts at (wrapped, or any valid one for padding)
    const bool outside = (unsigned)gc0 >= (unsigned)cols;
    const int vcol = !outside ? gc0 : (B == kWrap ? resolve<B>(gc0, cols) : 0);
    const bool edge_wave = __any(outside) != 0;     // the same for the whole wavefront
    // otherwise: per cell, the column after border resolution, and which bytes are matrix cells
    uint32_t inside_mask[WORDS];
#pragma unroll
    for (int w = 0; w < WORDS; ++w) {
        inside_mask[w] = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b)
            if ((unsigned)(gc0 + 4 * w + b) < (unsigned)cols) inside_mask[w] |= 0xffu << (8 * b);
    }

    const int kSteps = H + 2 * DEPTH;               // input rows a segment consumes
    const int kRounds = (kSteps + PF - 1) / PF;     // whole rounds; steps past kSteps store nothing

    // issue the loads of input row r0 - DEPTH + t
    auto load_row = [&](int t, uint32_t (&v)[WORDS]) {
        const int tt = t < kSteps ? t : kSteps - 1;
        const int gr = resolve<B>(r0 - DEPTH + tt, rows);      // the same for the whole wavefront
        if (FAST) {
            load_words<WORDS>(v, a.in + (size_t)(gr < 0 ? 0 : gr) * cols + (unsigned)vcol);
        } else {
#pragma unroll
            for (int w = 0; w < WORDS; ++w) {
                uint32_t word = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int gc = resolve<B>(gc0 + 4 * w + b, cols);
                    const uint32_t cell = (gr < 0 || gc < 0) ? a.pad : a.in[(size_t)gr * cols + gc];
                    word |= cell << (8 * b);
                }
                v[w] = word;
            }
        }
    };
    // CONSTANT: cells of matrix row gr (any generation) that are not matrix cells hold the padding
    auto pad_outside = [&](int gr, uint32_t (&v)[WORDS]) {
        if (B != kConstant) return;
        const bool outside_r = (unsigned)gr >= (unsigned)rows;
        if (FAST) {
            if (outside_r || edge_wave) {
#pragma unroll
                for (int w = 0; w < WORDS; ++w) v[w] = (outside_r || outside) ? pad_word : v[w];
            }
        } else {
#pragma unroll
            for (int w = 0; w < WORDS; ++w) {
                const uint32_t keep = outside_r ? 0u : inside_mask[w];
                v[w] = (v[w] & keep) | (pad_word & ~keep);
            }
        }
    };

    // lv[k][s]: generation k's row that was produced at a time step with t % 3 == s (0 = input)
    uint32_t lv[DEPTH][R][WORDS];
#pragma unroll
    for (int k = 0; k < DEPTH; ++k)
#pragma unroll
        for (int s = 0; s < R; ++s)
#pragma unroll
            for (int w = 0; w < WORDS; ++w) lv[k][s][w] = 0;
    uint32_t pf[PF][WORDS];   // rows on their way from memory, PF time steps ahead
#pragma unroll
    for (int s = 0; s < PF; ++s) {
        load_row(s, pf[s]);
        // in the order the march consumes them: were the scheduler to issue the first-needed row
        // last, every round of the loop would begin by waiting for all loads in flight
        __builtin_amdgcn_sched_barrier(0);
    }

    for (int round = 0; round < kRounds; ++round) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int t = round * PF + p;
            const int u = p % R;                    // = t % R
#pragma unroll
            for (int w = 0; w < WORDS; ++w) lv[0][u][w] = pf[p][w];
            pad_outside(r0 - DEPTH + t, lv[0][u]);
            load_row(t + PF, pf[p]);
#pragma unroll
            for (int k = 1; k <= DEPTH; ++k) {
                // generation k's first row that anything depends on is due at step 2k
                if (t < 2 * k) continue;
                // generation k's row r0 - DEPTH + t - k from generation k-1's three newest rows
                const uint32_t(&up)[WORDS] = lv[k - 1][(u + 1) % R];
                const uint32_t(&mid)[WORDS] = lv[k - 1][(u + 2) % R];
                const uint32_t(&dn)[WORDS] = lv[k - 1][u];
                uint32_t v[WORDS];                  // byte-wise column sums, <= 3
#pragma unroll
                for (int w = 0; w < WORDS; ++w) v[w] = up[w] + mid[w] + dn[w];
                const uint32_t from_w = from_lane_below(v[WORDS - 1]);   // its top byte: the column west of ours
                const uint32_t from_e = from_lane_above(v[0]);           // its low byte: the column east of ours
                uint32_t res[WORDS];
#pragma unroll
                for (int w = 0; w < WORDS; ++w) {
                    const uint32_t prev = w == 0 ? from_w : v[w - 1], next = w == WORDS - 1 ? from_e : v[w + 1];
                    const uint32_t west = (v[w] << 8) | (prev >> 24);
                    const uint32_t east = (v[w] >> 8) | (next << 24);
                    const uint32_t s = v[w] + west + east;         // 3x3 block sums, <= 9 per byte
                    const uint32_t n = s - mid[w];                 // neighbours only
                    res[w] = zero_bytes((n | mid[w]) ^ 0x03030303u);   // zero byte <=> alive next (B3/S23)
                }
                const int gr = r0 - DEPTH + t - k;      // the matrix row just produced
                if (k < DEPTH) {
                    pad_outside(gr, res);
#pragma unroll
                    for (int w = 0; w < WORDS; ++w) lv[k][u][w] = res[w];
                } else if (t >= 2 * DEPTH && t < kSteps && gr < rows && writes) {
                    uint8_t *dst = a.out + (size_t)gr * cols + (unsigned)gc0;
                    if (FAST) {
                        store_words<WORDS>(dst, res, a.nt_store != 0);
                    } else {
#pragma unroll
                        for (int c = 0; c < CC; ++c)
                            if (gc0 + c < cols) dst[c] = (uint8_t)(res[c >> 2] >> (8 * (c & 3)));
                    }
                }
            }
        }
    }
}

template <int B, int DEPTH, int WORDS, bool FAST, int MAXT>
__global__ __launch_bounds__(MAXT) void life_stream_kernel(const TileArgs<OpLife, HaloC<1, 1, 1, 1>> a, const int H) {
    life_stream_body<B, DEPTH, WORDS, FAST>(a, H);
}

}  // namespace sk
