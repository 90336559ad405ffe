// The scenario handle behind the C ABI's stencil_t - host-side state only - and the registry entry of
// a compiled kernel variant.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <utility>
#include <vector>

#include "../../include/libstencil.h"

// ---- scenario handle ---------------------------------------------------------------------

// (scenario, in, out, wg_rows, wg_cols, applications fused into this launch, stream)
using LaunchFn = hipError_t (*)(const stencil *, const void *, void *, int, int, int, hipStream_t);

struct Variant {
    int staging;          // STENCIL_STAGING_LOCAL, _DIRECT, _TEMPORAL or _STREAM
    int kernel, border;
    int hn, hs, he, hw;   // -1: run-time border region; -2: any region within the largest one (mn, ms, me, mw)
    int mn = 0, ms = 0, me = 0, mw = 0;
    int cr, cc;           // cr = 0 (register-streaming kernels): any segment height up to kMaxSegmentRows
    int max_threads;      // per-kernel workgroup-size limit (Section 3.1)
    int staged_bytes;     // bytes per staged element in LDS
    bool fuses = false;   // a launch makes `temporal_depth` applications instead of one
    LaunchFn launch;
    // the compiled kernel a launch of this scenario would start (what hipFuncGetAttributes is asked about)
    const void *(*kernel_of)(const stencil *) = nullptr;
};
constexpr int kMaxSegmentRows = 4096;
inline bool rows_match(const Variant &v, int cr) { return v.cr == cr || (v.cr == 0 && cr >= 1 && cr <= kMaxSegmentRows); }

struct stencil {
    int64_t rows = 0, cols = 0;
    int dtype = STENCIL_F32;
    int hn = 0, hs = 0, he = 0, hw = 0;
    int border = STENCIL_CLAMP;
    double pad = 0.0;
    int kernel = STENCIL_WEIGHTED_SUM;
    std::vector<float> weights;
    float scalar0 = 0.0f;
    int staging = STENCIL_STAGING_LOCAL;
    int cr = 1, cc = 1;
    int xcd_remap = 1;
    int nt_store = 0;         // output vectors are written with non-temporal stores
    int temporal_depth = 2;   // applications per launch under STENCIL_STAGING_TEMPORAL
    int sweep_cutoff_pct = 0; // > 0: sizes slower than this percentage of the best so far are cut short
    int best_rows = 0, best_cols = 0;
    int fail_rows = 0, fail_cols = 0;   // testing aid: launches of this workgroup size fail (-1: every launch)
    // the classifier stencil_run(0, 0) asks when no sweep has been made (not owned), and its fallback handler
    const stencil_predictor_t *predictor = nullptr;
    int predictor_handler = 0;
    // device-side state, created on first use
    void *scratch = nullptr;
    float *d_tables[2] = {nullptr, nullptr};   // weight tables of a run-time region; a replaced table goes into the other one
    float *d_weights = nullptr;                // the current one of the two
    const float *table_in_use = nullptr;       // what the launchers hand to the kernels
    bool weights_uploaded = false;
    std::vector<hipEvent_t> events;
    // matrix pairs the sweeps' applications go round (stencil_set_sweep_rotation); empty: the caller's pair
    std::vector<std::pair<const void *, void *>> rotation;
    size_t rotation_at = 0;
    size_t elem() const { return dtype == STENCIL_U8 ? 1 : (dtype == STENCIL_F64 ? 8 : 4); }
    size_t bytes() const { return (size_t)rows * (size_t)cols * elem(); }
    // the output matrix: the input's element type, except for the threshold stencil (floats in,
    // bytes out) and the weighted sum of a byte matrix (bytes in, floats out)
    int out_dtype() const {
        if (kernel == STENCIL_THRESHOLD) return STENCIL_U8;
        if (kernel == STENCIL_WEIGHTED_SUM && dtype == STENCIL_U8) return STENCIL_F32;
        return dtype;
    }
    size_t out_elem() const { return out_dtype() == STENCIL_U8 ? 1 : (out_dtype() == STENCIL_F64 ? 8 : 4); }
    size_t out_bytes() const { return (size_t)rows * (size_t)cols * out_elem(); }
};

// Variant keys of WEIGHTED_SUM on the other element types (internal: the public kernel id is
// STENCIL_WEIGHTED_SUM, the matrix dtype selects the variant).
enum { STENCIL_WEIGHTED_SUM_F64 = 100, STENCIL_WEIGHTED_SUM_I32 = 101, STENCIL_WEIGHTED_SUM_U8 = 102 };

