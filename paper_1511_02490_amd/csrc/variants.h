// Shared between the translation units of libstencil: tile geometry, kernel arguments, the launchers
// of every kernel family and the templates that register their variants (the scenario handle and
// the registry entry of a compiled kernel variant: scenario.h).  Each variants_*.hip instantiates one group of
// kernels and exports a register function; libstencil.hip assembles the registry and holds the
// C ABI.  (Everything here has internal linkage: each unit gets its own small copy.)
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <type_traits>
#include <vector>

#include "direct_kernel.h"
#include "stream_kernel.h"
#include "temporal_kernel.h"
#include "tile_kernel.h"
#include "march_kernel.h"
#include "march_masked_kernel.h"
#include "life_stream_kernel.h"
#include "pointwise_kernel.h"

#include "scenario.h"

// Local memory a workgroup may allocate: the device's own figure once a GPU has been used, the
// header's constant before that (defined in libstencil.hip).
int64_t stencil_local_memory_limit();

namespace {

// the registry key of a scenario's kernel
int variant_kernel(const stencil *s) {
    if (s->kernel == STENCIL_WEIGHTED_SUM && s->dtype == STENCIL_F64) return STENCIL_WEIGHTED_SUM_F64;
    if (s->kernel == STENCIL_WEIGHTED_SUM && s->dtype == STENCIL_I32) return STENCIL_WEIGHTED_SUM_I32;
    if (s->kernel == STENCIL_WEIGHTED_SUM && s->dtype == STENCIL_U8) return STENCIL_WEIGHTED_SUM_U8;
    return s->kernel;
}

struct TileGeom {
    int th, tw;        // elements covered by one workgroup
    int pitch;         // LDS pitch in staged elements
    int plane;         // staged elements per LDS plane
    int64_t lds_bytes;
    int tiles_r, tiles_c;
};

TileGeom tile_geom(const stencil *s, const Variant &v, int wr, int wc) {
    TileGeom g;
    g.th = wr * v.cr;
    g.tw = wc * v.cc;
    const int hwa = v.cc == 1 ? s->hw : sk::round_up(s->hw, v.cc);
    const int hea = v.cc == 1 ? s->he : sk::round_up(s->he, v.cc);
    g.pitch = hwa + g.tw + hea;
    g.plane = (g.th + s->hn + s->hs) * g.pitch;
    g.lds_bytes = (int64_t)g.plane * v.staged_bytes;
    if (v.staging == STENCIL_STAGING_DIRECT) {
        g.plane = 0;
        g.lds_bytes = 0;
    } else if (v.staging == STENCIL_STAGING_STREAM) {
        // one wavefront per tile: s->cr rows of a strip of 62..64 vectors; no local memory
        g.th = s->cr;
        g.tw = !v.fuses ? sk::march_vectors(s->hw, s->he) * 4
               : s->kernel == STENCIL_LIFE ? sk::life_stream_cols(s->temporal_depth, v.cc / 4)
                                           : sk::stream_cols(s->temporal_depth);
        g.pitch = 4;
        g.plane = 0;
        g.lds_bytes = 0;
    } else if (v.staging == STENCIL_STAGING_TEMPORAL) {
        // tile + `depth` rows above and below, one vector left and right; two buffers
        g.pitch = g.tw + 2 * v.cc;
        g.plane = (g.th + 2 * s->temporal_depth) * g.pitch;
        g.lds_bytes = 2 * (int64_t)g.plane * v.staged_bytes + 32;   // + one spare vector at each end
    }
    g.tiles_r = (int)((s->rows + g.th - 1) / g.th);
    g.tiles_c = (int)((s->cols + g.tw - 1) / g.tw);
    return g;
}

// Kernel arguments and grid for one launch; `blocks` is the grid size.
template <class Op, class Halo, int CR, int CC>
sk::TileArgs<Op, Halo> make_args(const stencil *s, int staging, const void *in, void *out, int wr, int wc,
                                 unsigned *blocks, size_t *lds_bytes) {
    using T = typename Op::T;
    Variant v{};
    v.staging = staging;
    v.cr = CR;
    v.cc = CC;
    v.staged_bytes = (int)sizeof(typename Op::L) * Op::kPlanes;
    const TileGeom g = tile_geom(s, v, wr, wc);
    sk::TileArgs<Op, Halo> a;
    a.in = static_cast<const T *>(in);
    a.out = static_cast<typename sk::out_type_of<Op>::type *>(out);
    a.rows = (int)s->rows;
    a.cols = (int)s->cols;
    a.tiles_c = g.tiles_c;
    a.n_tiles = g.tiles_r * g.tiles_c;
    a.pitch = g.pitch;
    a.plane = g.plane;
    {
        // vectors (elements when CC = 1) per staged row; kernels that stage nothing have none
        const unsigned items = std::max(1u, (unsigned)(g.pitch / CC));
        a.stage_magic = (unsigned)((0x100000000ull + items - 1) / items);
    }
    // a work-item moves CC cells at a time: rows of both matrices must start at multiples of that
    // (16 bytes, except 4 where four byte cells are loaded)
    using O = typename sk::out_type_of<Op>::type;
    constexpr size_t in_vec = CC * sizeof(T), out_vec = CC * sizeof(O);
    a.vec_ok = (CC > 1 && ((size_t)s->cols * sizeof(T)) % in_vec == 0 && (uintptr_t)in % in_vec == 0 &&
                ((size_t)s->cols * sizeof(O)) % out_vec == 0 && (uintptr_t)out % out_vec == 0) ? 1 : 0;
    a.nt_store = s->nt_store;
    a.pad = (T)s->pad;
    a.scalar0 = s->scalar0;
    if constexpr (Halo::kStatic) {
        if constexpr (Op::kWeights)
            for (int k = 0; k < (int)(sizeof(a.w.v) / sizeof(a.w.v[0])); ++k) a.w.v[k] = s->weights[k];
        else
            a.w.v[0] = 0.0f;
    } else {
        a.halo.n_ = s->hn;
        a.halo.s_ = s->hs;
        a.halo.e_ = s->he;
        a.halo.w_ = s->hw;
        a.w.v = s->table_in_use;
    }
    *blocks = (unsigned)a.n_tiles;
    a.xcd_chunk = 0;
    if (s->xcd_remap && a.n_tiles >= 64) {
        a.xcd_chunk = (a.n_tiles + 7) / 8;
        *blocks = (unsigned)a.xcd_chunk * 8u;
    }
    *lds_bytes = (size_t)g.lds_bytes;
    return a;
}

// Tiles above 64 KiB need the kernel's dynamic local-memory limit raised, once per kernel and
// device; `raised_on` remembers the device it was last done on.
hipError_t allow_large_tiles(const void *kernel, size_t lds, int *raised_on) {
    if (lds <= 65536) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (*raised_on != dev) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)stencil_local_memory_limit());
        if (e != hipSuccess) return e;
        *raised_on = dev;
    }
    return hipSuccess;
}

template <class Op, int B, int CR, int MAXT>
hipError_t launch_temporal(const stencil *s, const void *in, void *out, int wr, int wc, int depth,
                           hipStream_t stream) {
    using Halo = sk::HaloC<1, 1, 1, 1>;
    unsigned blocks;
    size_t lds;
    const auto a = make_args<Op, Halo, CR, 4>(s, STENCIL_STAGING_TEMPORAL, in, out, wr, wc, &blocks, &lds);
    static thread_local int raised_on = -1;
    hipError_t e = allow_large_tiles(reinterpret_cast<const void *>(&sk::temporal_kernel<Op, B, CR, MAXT>), lds,
                                     &raised_on);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((sk::temporal_kernel<Op, B, CR, MAXT>), dim3(blocks), dim3(wc, wr), lds, stream, a, depth);
    return hipGetLastError();
}

template <class Op, int B>
hipError_t launch_stream(const stencil *s, const void *in, void *out, int wr, int wc, int depth, hipStream_t stream) {
    using Halo = sk::HaloC<1, 1, 1, 1>;
    constexpr int kMaxT = 256;
    if (depth < 1 || depth > sk::kStreamMaxDepth) return hipErrorInvalidValue;
    const int CR = s->cr;   // rows per segment
    unsigned blocks;
    size_t lds;
    auto a = make_args<Op, Halo, 0, 4>(s, STENCIL_STAGING_STREAM, in, out, wr, wc, &blocks, &lds);
    // a tile is one wavefront's segment: CR rows of a strip whose width follows from the number of
    // applications this launch fuses (the last launch of a run may fuse fewer)
    const int strip_cols = sk::stream_cols(depth);
    a.tiles_c = (int)((s->cols + strip_cols - 1) / strip_cols);
    a.n_tiles = (int)((s->rows + CR - 1) / CR) * a.tiles_c;
    a.xcd_chunk = 0;
    const unsigned waves_per_block = (unsigned)(wr * wc) / 64u;
    blocks = ((unsigned)a.n_tiles + waves_per_block - 1) / waves_per_block;
    const dim3 grid(blocks), block(wc, wr);
#define STREAM_LAUNCH(D)                                                                                       \
    if (a.vec_ok)                                                                                              \
        hipLaunchKernelGGL((sk::stream_kernel<Op, B, D, true, kMaxT>), grid, block, 0, stream, a, CR);         \
    else                                                                                                       \
        hipLaunchKernelGGL((sk::stream_kernel<Op, B, D, false, kMaxT>), grid, block, 0, stream, a, CR);        \
    break
    switch (depth) {
    case 1: STREAM_LAUNCH(1);
    case 2: STREAM_LAUNCH(2);
    case 3: STREAM_LAUNCH(3);
    case 4: STREAM_LAUNCH(4);
    case 5: STREAM_LAUNCH(5);
    case 6: STREAM_LAUNCH(6);
    case 7: STREAM_LAUNCH(7);
    case 8: STREAM_LAUNCH(8);
    default: return hipErrorInvalidValue;
    }
#undef STREAM_LAUNCH
    return hipGetLastError();
}

// Game of Life, `depth` generations per launch in registers (life_stream_kernel.h).
template <int B, int WORDS>
hipError_t launch_life_stream(const stencil *s, const void *in, void *out, int wr, int wc, int depth,
                              hipStream_t stream) {
    using Halo = sk::HaloC<1, 1, 1, 1>;
    constexpr int kMaxT = 256;
    if (depth < 1 || depth > sk::kLifeStreamMaxDepth) return hipErrorInvalidValue;
    const int CR = s->cr;   // rows per segment
    unsigned blocks;
    size_t lds;
    auto a = make_args<sk::OpLife, Halo, 0, 16>(s, STENCIL_STAGING_STREAM, in, out, wr, wc, &blocks, &lds);
    const int strip_cols = sk::life_stream_cols(depth, WORDS);
    a.tiles_c = (int)((s->cols + strip_cols - 1) / strip_cols);
    a.n_tiles = (int)((s->rows + CR - 1) / CR) * a.tiles_c;
    a.xcd_chunk = 0;
    const unsigned waves_per_block = (unsigned)(wr * wc) / 64u;
    blocks = ((unsigned)a.n_tiles + waves_per_block - 1) / waves_per_block;
    const dim3 grid(blocks), block(wc, wr);
#define LIFE_STREAM_LAUNCH(D)                                                                                  \
    if (a.vec_ok)                                                                                              \
        hipLaunchKernelGGL((sk::life_stream_kernel<B, D, WORDS, true, kMaxT>), grid, block, 0, stream, a, CR); \
    else                                                                                                       \
        hipLaunchKernelGGL((sk::life_stream_kernel<B, D, WORDS, false, kMaxT>), grid, block, 0, stream, a, CR);\
    break
    switch (depth) {
    case 1: LIFE_STREAM_LAUNCH(1);
    case 2: LIFE_STREAM_LAUNCH(2);
    case 3: LIFE_STREAM_LAUNCH(3);
    case 4: LIFE_STREAM_LAUNCH(4);
    case 5: LIFE_STREAM_LAUNCH(5);
    case 6: LIFE_STREAM_LAUNCH(6);
    case 7: LIFE_STREAM_LAUNCH(7);
    case 8: LIFE_STREAM_LAUNCH(8);
    default: return hipErrorInvalidValue;
    }
#undef LIFE_STREAM_LAUNCH
    return hipGetLastError();
}

// The threshold stencil: float in, bytes out, no border region (pointwise_kernel.h).
template <int CR, int CC>
hipError_t launch_threshold(const stencil *s, const void *in, void *out, int wr, int wc, int, hipStream_t stream) {
    sk::ThresholdArgs a;
    a.in = static_cast<const float *>(in);
    a.out = static_cast<uint8_t *>(out);
    a.rows = (int)s->rows;
    a.cols = (int)s->cols;
    const int th = wr * CR, tw = wc * CC;
    a.tiles_c = (a.cols + tw - 1) / tw;
    a.n_tiles = ((a.rows + th - 1) / th) * a.tiles_c;
    a.vec_ok = (CC == 4 && s->cols % 4 == 0 && (uintptr_t)in % 16 == 0 && (uintptr_t)out % 4 == 0) ? 1 : 0;
    a.level = s->scalar0;
    unsigned blocks = (unsigned)a.n_tiles;
    a.xcd_chunk = 0;
    if (s->xcd_remap && a.n_tiles >= 64) {
        a.xcd_chunk = (a.n_tiles + 7) / 8;
        blocks = (unsigned)a.xcd_chunk * 8u;
    }
    hipLaunchKernelGGL((sk::threshold_kernel<CR, CC, STENCIL_MAX_WG_SIZE>), dim3(blocks), dim3(wc, wr), 0, stream, a);
    return hipGetLastError();
}

// One application, marched down the matrix in registers (march_kernel.h).
template <class Op, int B, class Halo>
hipError_t launch_march(const stencil *s, const void *in, void *out, int wr, int wc, int, hipStream_t stream) {
    constexpr int kMaxT = 256;
    unsigned blocks;
    size_t lds;
    auto a = make_args<Op, Halo, 0, 4>(s, STENCIL_STAGING_STREAM, in, out, wr, wc, &blocks, &lds);
    // a tile is a wavefront's segment; workgroups only group wavefronts
    const unsigned waves_per_block = (unsigned)(wr * wc) / 64u;
    blocks = ((unsigned)a.n_tiles + waves_per_block - 1) / waves_per_block;
    a.xcd_chunk = 0;
    if (s->xcd_remap && blocks >= 64) {
        a.xcd_chunk = (int)((blocks + 7) / 8);
        blocks = (unsigned)a.xcd_chunk * 8u;
    }
    // whole aligned vectors per row, or the element-by-element body
    if (a.vec_ok)
        hipLaunchKernelGGL((sk::march_kernel<Op, B, Halo, true, kMaxT>), dim3(blocks), dim3(wc, wr), 0, stream, a,
                           s->cr);
    else
        hipLaunchKernelGGL((sk::march_kernel<Op, B, Halo, false, kMaxT>), dim3(blocks), dim3(wc, wr), 0, stream, a,
                           s->cr);
    return hipGetLastError();
}

// The same for any region within the kernel's largest one (march_masked_kernel.h): the kernel compiled for the
// region's number of columns.
template <class Op, int B, class Halo, int WC = 1>
hipError_t launch_march_masked(const stencil *s, const void *in, void *out, int wr, int wc, int, hipStream_t stream) {
    constexpr int kMaxT = 256;
    if constexpr (WC > Halo::E + Halo::W + 1) {
        return hipErrorInvalidValue;
    } else {
        if (s->he + s->hw + 1 != WC) return launch_march_masked<Op, B, Halo, WC + 1>(s, in, out, wr, wc, 0, stream);
        if (s->hn > Halo::N || s->hs > Halo::S || s->he > Halo::E || s->hw > Halo::W) return hipErrorInvalidValue;
        unsigned blocks;
        size_t lds;
        auto a = make_args<Op, Halo, 0, 4>(s, STENCIL_STAGING_STREAM, in, out, wr, wc, &blocks, &lds);
        const unsigned waves_per_block = (unsigned)(wr * wc) / 64u;
        blocks = ((unsigned)a.n_tiles + waves_per_block - 1) / waves_per_block;
        a.xcd_chunk = 0;
        if (s->xcd_remap && blocks >= 64) {
            a.xcd_chunk = (int)((blocks + 7) / 8);
            blocks = (unsigned)a.xcd_chunk * 8u;
        }
        if (a.vec_ok)
            hipLaunchKernelGGL((sk::march_masked_kernel<Op, B, Halo, WC, true, kMaxT>), dim3(blocks), dim3(wc, wr), 0,
                               stream, a, s->cr);
        else
            hipLaunchKernelGGL((sk::march_masked_kernel<Op, B, Halo, WC, false, kMaxT>), dim3(blocks), dim3(wc, wr), 0,
                               stream, a, s->cr);
        return hipGetLastError();
    }
}

template <int B, int CR, int MAXT>
hipError_t launch_life_temporal(const stencil *s, const void *in, void *out, int wr, int wc, int depth,
                                hipStream_t stream) {
    unsigned blocks;
    size_t lds;
    const auto a = make_args<sk::OpLife, sk::HaloC<1, 1, 1, 1>, CR, 16>(s, STENCIL_STAGING_TEMPORAL, in, out, wr, wc,
                                                                        &blocks, &lds);
    static thread_local int raised_on = -1;
    hipError_t e = allow_large_tiles(reinterpret_cast<const void *>(&sk::life_temporal_kernel<B, CR, MAXT>), lds,
                                     &raised_on);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((sk::life_temporal_kernel<B, CR, MAXT>), dim3(blocks), dim3(wc, wr), lds, stream, a, depth);
    return hipGetLastError();
}

template <class Op, int B, class Halo, int CR, int CC, int MAXT>
hipError_t launch_tile(const stencil *s, const void *in, void *out, int wr, int wc, int, hipStream_t stream) {
    unsigned blocks;
    size_t lds;
    const auto a = make_args<Op, Halo, CR, CC>(s, STENCIL_STAGING_LOCAL, in, out, wr, wc, &blocks, &lds);
    static thread_local int raised_on = -1;
    hipError_t e = allow_large_tiles(reinterpret_cast<const void *>(&sk::tile_kernel<Op, B, Halo, CR, CC, MAXT>),
                                     lds, &raised_on);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((sk::tile_kernel<Op, B, Halo, CR, CC, MAXT>), dim3(blocks), dim3(wc, wr), lds, stream, a);
    return hipGetLastError();
}

template <class Op, int B, class Halo, int CR, int CC, int MAXT>
hipError_t launch_direct(const stencil *s, const void *in, void *out, int wr, int wc, int, hipStream_t stream) {
    unsigned blocks;
    size_t lds;
    const auto a = make_args<Op, Halo, CR, CC>(s, STENCIL_STAGING_DIRECT, in, out, wr, wc, &blocks, &lds);
    hipLaunchKernelGGL((sk::direct_kernel<Op, B, Halo, CR, CC, MAXT>), dim3(blocks), dim3(wc, wr), 0, stream, a);
    return hipGetLastError();
}

template <int B, int CR, int MAXT>
hipError_t launch_life_direct(const stencil *s, const void *in, void *out, int wr, int wc, int, hipStream_t stream) {
    unsigned blocks;
    size_t lds;
    const auto a = make_args<sk::OpLife, sk::HaloC<1, 1, 1, 1>, CR, 16>(s, STENCIL_STAGING_DIRECT, in, out, wr, wc,
                                                                        &blocks, &lds);
    hipLaunchKernelGGL((sk::life_direct_kernel<B, CR, MAXT>), dim3(blocks), dim3(wc, wr), 0, stream, a);
    return hipGetLastError();
}


// The kernel behind each launcher (the variant with whole aligned vectors where there are two).
template <class Op, int B, class Halo, int CR, int CC, int MAXT>
const void *kernel_tile(const stencil *) { return reinterpret_cast<const void *>(&sk::tile_kernel<Op, B, Halo, CR, CC, MAXT>); }
template <class Op, int B, class Halo, int CR, int CC, int MAXT>
const void *kernel_direct(const stencil *) { return reinterpret_cast<const void *>(&sk::direct_kernel<Op, B, Halo, CR, CC, MAXT>); }
template <int B, int CR, int MAXT>
const void *kernel_life_direct(const stencil *) { return reinterpret_cast<const void *>(&sk::life_direct_kernel<B, CR, MAXT>); }
template <class Op, int B, int CR, int MAXT>
const void *kernel_temporal(const stencil *) { return reinterpret_cast<const void *>(&sk::temporal_kernel<Op, B, CR, MAXT>); }
template <int B, int CR, int MAXT>
const void *kernel_life_temporal(const stencil *) { return reinterpret_cast<const void *>(&sk::life_temporal_kernel<B, CR, MAXT>); }
template <int CR, int CC>
const void *kernel_threshold(const stencil *) { return reinterpret_cast<const void *>(&sk::threshold_kernel<CR, CC, STENCIL_MAX_WG_SIZE>); }
template <class Op, int B, class Halo>
const void *kernel_march(const stencil *) { return reinterpret_cast<const void *>(&sk::march_kernel<Op, B, Halo, true, 256>); }
template <class Op, int B, class Halo, int WC = 1>
const void *kernel_march_masked(const stencil *s) {
    if constexpr (WC > Halo::E + Halo::W + 1)
        return nullptr;
    else if (s->he + s->hw + 1 != WC)
        return kernel_march_masked<Op, B, Halo, WC + 1>(s);
    else
        return reinterpret_cast<const void *>(&sk::march_masked_kernel<Op, B, Halo, WC, true, 256>);
}
template <class Op, int B>
const void *kernel_stream(const stencil *s) {
    switch (s->temporal_depth) {
    case 1: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 1, true, 256>);
    case 2: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 2, true, 256>);
    case 3: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 3, true, 256>);
    case 4: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 4, true, 256>);
    case 5: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 5, true, 256>);
    case 6: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 6, true, 256>);
    case 7: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 7, true, 256>);
    case 8: return reinterpret_cast<const void *>(&sk::stream_kernel<Op, B, 8, true, 256>);
    default: return nullptr;
    }
}
template <int B, int WORDS>
const void *kernel_life_stream(const stencil *s) {
    switch (s->temporal_depth) {
    case 1: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 1, WORDS, true, 256>);
    case 2: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 2, WORDS, true, 256>);
    case 3: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 3, WORDS, true, 256>);
    case 4: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 4, WORDS, true, 256>);
    case 5: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 5, WORDS, true, 256>);
    case 6: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 6, WORDS, true, 256>);
    case 7: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 7, WORDS, true, 256>);
    case 8: return reinterpret_cast<const void *>(&sk::life_stream_kernel<B, 8, WORDS, true, 256>);
    default: return nullptr;
    }
}

// Per-kernel workgroup-size limit (Section 3.1: the registers a kernel needs bound its
// maximum workgroup size).  The heavily blocked variants are compiled for 256 work-items so
// that their register windows stay out of scratch memory.
template <class Op, int CR, int CC>
constexpr int variant_max_threads() {
    if (std::is_same<Op, sk::OpSinCos>::value && CR * CC >= 32) return 256;
    if (std::is_same<Op, sk::OpLife>::value && CR * CC >= 64) return 256;
    if (std::is_same<Op, sk::OpWeightedSumU8>::value && CR * CC >= 32) return 256;
    return STENCIL_MAX_WG_SIZE;
}

template <class Op, int KID, int B, class Halo, int CR, int CC>
void reg_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_LOCAL;
    v.kernel = KID;
    v.border = B;
    if (Halo::kStatic) {
        v.hn = Halo::N; v.hs = Halo::S; v.he = Halo::E; v.hw = Halo::W;
    } else {
        v.hn = v.hs = v.he = v.hw = -1;
    }
    v.cr = CR;
    v.cc = CC;
    constexpr int kMaxT = variant_max_threads<Op, CR, CC>();
    v.max_threads = kMaxT;
    v.staged_bytes = (int)sizeof(typename Op::L) * Op::kPlanes;
    v.launch = &launch_tile<Op, B, Halo, CR, CC, kMaxT>;
    v.kernel_of = &kernel_tile<Op, B, Halo, CR, CC, kMaxT>;
    r.push_back(v);
}

template <class Op, int KID, int B, class Halo, int CR, int CC>
void reg_direct_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_DIRECT;
    v.kernel = KID;
    v.border = B;
    v.hn = Halo::N; v.hs = Halo::S; v.he = Halo::E; v.hw = Halo::W;
    v.cr = CR;
    v.cc = CC;
    v.max_threads = STENCIL_MAX_WG_SIZE;
    v.staged_bytes = 0;
    v.launch = &launch_direct<Op, B, Halo, CR, CC, STENCIL_MAX_WG_SIZE>;
    v.kernel_of = &kernel_direct<Op, B, Halo, CR, CC, STENCIL_MAX_WG_SIZE>;
    r.push_back(v);
}

template <class Op, int KID, class Halo, int CC>
void reg_direct(std::vector<Variant> &r) {
    reg_direct_one<Op, KID, sk::kClamp, Halo, 1, CC>(r);
    reg_direct_one<Op, KID, sk::kWrap, Halo, 1, CC>(r);
    reg_direct_one<Op, KID, sk::kConstant, Halo, 1, CC>(r);
    reg_direct_one<Op, KID, sk::kClamp, Halo, 2, CC>(r);
    reg_direct_one<Op, KID, sk::kWrap, Halo, 2, CC>(r);
    reg_direct_one<Op, KID, sk::kConstant, Halo, 2, CC>(r);
    reg_direct_one<Op, KID, sk::kClamp, Halo, 4, CC>(r);
    reg_direct_one<Op, KID, sk::kWrap, Halo, 4, CC>(r);
    reg_direct_one<Op, KID, sk::kConstant, Halo, 4, CC>(r);
}

template <class Op, int KID, int B, int CR>
void reg_temporal_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_TEMPORAL;
    v.kernel = KID;
    v.border = B;
    v.hn = v.hs = v.he = v.hw = 1;
    v.cr = CR;
    v.cc = 4;
    v.max_threads = STENCIL_MAX_WG_SIZE;
    v.staged_bytes = 4;
    v.fuses = true;
    v.launch = &launch_temporal<Op, B, CR, STENCIL_MAX_WG_SIZE>;
    v.kernel_of = &kernel_temporal<Op, B, CR, STENCIL_MAX_WG_SIZE>;
    r.push_back(v);
}

template <class Op, int KID, int CR>
void reg_temporal(std::vector<Variant> &r) {
    reg_temporal_one<Op, KID, sk::kClamp, CR>(r);
    reg_temporal_one<Op, KID, sk::kWrap, CR>(r);
    reg_temporal_one<Op, KID, sk::kConstant, CR>(r);
}

template <class Op, int KID, int B>
void reg_stream_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_STREAM;
    v.kernel = KID;
    v.border = B;
    v.hn = v.hs = v.he = v.hw = 1;
    v.cr = 0;
    v.cc = 4;
    v.max_threads = 256;
    v.staged_bytes = 0;
    v.fuses = true;
    v.launch = &launch_stream<Op, B>;
    v.kernel_of = &kernel_stream<Op, B>;
    r.push_back(v);
}

template <class Op, int KID>
void reg_stream(std::vector<Variant> &r) {
    reg_stream_one<Op, KID, sk::kWrap>(r);
    reg_stream_one<Op, KID, sk::kConstant>(r);
}

template <int B, int WORDS>
void reg_life_stream_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_STREAM;
    v.kernel = STENCIL_LIFE;
    v.border = B;
    v.hn = v.hs = v.he = v.hw = 1;
    v.cr = 0;
    v.cc = 4 * WORDS;
    v.max_threads = 256;
    v.staged_bytes = 0;
    v.fuses = true;
    v.launch = &launch_life_stream<B, WORDS>;
    v.kernel_of = &kernel_life_stream<B, WORDS>;
    r.push_back(v);
}

template <int WORDS>
void reg_life_stream(std::vector<Variant> &r) {
    reg_life_stream_one<sk::kWrap, WORDS>(r);
    reg_life_stream_one<sk::kConstant, WORDS>(r);
}

template <int B, int CR, int CC>
void reg_threshold_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_LOCAL;     // the paper's mapping; with no border region there is no tile to stage
    v.kernel = STENCIL_THRESHOLD;
    v.border = B;
    v.hn = v.hs = v.he = v.hw = 0;
    v.cr = CR;
    v.cc = CC;
    v.max_threads = STENCIL_MAX_WG_SIZE;
    v.staged_bytes = 0;
    v.launch = &launch_threshold<CR, CC>;
    v.kernel_of = &kernel_threshold<CR, CC>;
    r.push_back(v);
}

template <int CR, int CC>
void reg_threshold(std::vector<Variant> &r) {
    reg_threshold_one<sk::kClamp, CR, CC>(r);
    reg_threshold_one<sk::kWrap, CR, CC>(r);
    reg_threshold_one<sk::kConstant, CR, CC>(r);
}

template <class Op, int KID, int B, class Halo>
void reg_march_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_STREAM;
    v.kernel = KID;
    v.border = B;
    v.hn = Halo::N;
    v.hs = Halo::S;
    v.he = Halo::E;
    v.hw = Halo::W;
    v.cr = 0;
    v.cc = 4;
    v.max_threads = 256;
    v.staged_bytes = 0;
    v.fuses = false;
    v.launch = &launch_march<Op, B, Halo>;
    v.kernel_of = &kernel_march<Op, B, Halo>;
    r.push_back(v);
}

template <class Op, int KID, class Halo>
void reg_march(std::vector<Variant> &r) {
    reg_march_one<Op, KID, sk::kClamp, Halo>(r);
    reg_march_one<Op, KID, sk::kWrap, Halo>(r);
    reg_march_one<Op, KID, sk::kConstant, Halo>(r);
}

template <class Op, int KID, int B, class Halo>
void reg_march_masked_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_STREAM;
    v.kernel = KID;
    v.border = B;
    v.hn = v.hs = v.he = v.hw = -2;
    v.mn = Halo::N;
    v.ms = Halo::S;
    v.me = Halo::E;
    v.mw = Halo::W;
    v.cr = 0;
    v.cc = 4;
    v.max_threads = 256;
    v.staged_bytes = 0;
    v.fuses = false;
    v.launch = &launch_march_masked<Op, B, Halo>;
    v.kernel_of = &kernel_march_masked<Op, B, Halo>;
    r.push_back(v);
}

template <class Op, int KID, class Halo>
void reg_march_masked(std::vector<Variant> &r) {
    reg_march_masked_one<Op, KID, sk::kClamp, Halo>(r);
    reg_march_masked_one<Op, KID, sk::kWrap, Halo>(r);
    reg_march_masked_one<Op, KID, sk::kConstant, Halo>(r);
}

template <int B, int CR>
void reg_life_temporal_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_TEMPORAL;
    v.kernel = STENCIL_LIFE;
    v.border = B;
    v.hn = v.hs = v.he = v.hw = 1;
    v.cr = CR;
    v.cc = 16;
    v.max_threads = STENCIL_MAX_WG_SIZE;
    v.staged_bytes = 1;
    v.fuses = true;
    v.launch = &launch_life_temporal<B, CR, STENCIL_MAX_WG_SIZE>;
    v.kernel_of = &kernel_life_temporal<B, CR, STENCIL_MAX_WG_SIZE>;
    r.push_back(v);
}

template <int CR>
void reg_life_temporal(std::vector<Variant> &r) {
    reg_life_temporal_one<sk::kClamp, CR>(r);
    reg_life_temporal_one<sk::kWrap, CR>(r);
    reg_life_temporal_one<sk::kConstant, CR>(r);
}

template <int B, int CR>
void reg_life_direct_one(std::vector<Variant> &r) {
    Variant v;
    v.staging = STENCIL_STAGING_DIRECT;
    v.kernel = STENCIL_LIFE;
    v.border = B;
    v.hn = v.hs = v.he = v.hw = 1;
    v.cr = CR;
    v.cc = 16;
    v.max_threads = STENCIL_MAX_WG_SIZE;
    v.staged_bytes = 0;
    v.launch = &launch_life_direct<B, CR, STENCIL_MAX_WG_SIZE>;
    v.kernel_of = &kernel_life_direct<B, CR, STENCIL_MAX_WG_SIZE>;
    r.push_back(v);
}

template <int CR>
void reg_life_direct(std::vector<Variant> &r) {
    reg_life_direct_one<sk::kClamp, CR>(r);
    reg_life_direct_one<sk::kWrap, CR>(r);
    reg_life_direct_one<sk::kConstant, CR>(r);
}

template <class Op, int KID, class Halo, int CR, int CC>
void reg_borders(std::vector<Variant> &r) {
    reg_one<Op, KID, sk::kClamp, Halo, CR, CC>(r);
    reg_one<Op, KID, sk::kWrap, Halo, CR, CC>(r);
    reg_one<Op, KID, sk::kConstant, Halo, CR, CC>(r);
}

template <class Op, int KID, class Halo, int CCV>
void reg_blockings(std::vector<Variant> &r) {
    reg_borders<Op, KID, Halo, 1, 1>(r);
    reg_borders<Op, KID, Halo, 2, 1>(r);
    reg_borders<Op, KID, Halo, 4, 1>(r);
    reg_borders<Op, KID, Halo, 8, 1>(r);
    reg_borders<Op, KID, Halo, 1, CCV>(r);
    reg_borders<Op, KID, Halo, 2, CCV>(r);
    reg_borders<Op, KID, Halo, 4, CCV>(r);
    reg_borders<Op, KID, Halo, 8, CCV>(r);
}

}  // namespace

// The groups of variants, one translation unit each.
void register_weighted_sum_tiles(std::vector<Variant> &r);
void register_sincos(std::vector<Variant> &r);
void register_unit_region_tiles(std::vector<Variant> &r);
void register_direct_and_temporal(std::vector<Variant> &r);
void register_streams(std::vector<Variant> &r);
void register_life_streams(std::vector<Variant> &r);
void register_wide_regions(std::vector<Variant> &r);
void register_runtime_march(std::vector<Variant> &r);
