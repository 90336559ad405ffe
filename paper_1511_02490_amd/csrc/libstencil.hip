// libstencil: C-ABI front end, scenario handle, legality, launch and the timed
// workgroup-size sweep.  The interface is documented in include/libstencil.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>
#include <mutex>
#include <new>
#include <type_traits>
#include <unordered_map>
#include <vector>

#include "host_tuning.h"
#include "variants.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int fail_hip(hipError_t e, const char *what) {
    return fail(STENCIL_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

// Section 3.1 takes W_max(s) from the device and the compiled kernel, Section 3.2 takes the
// device's features from the OpenCL device API.  Here: hipGetDeviceProperties at the first call
// that uses the GPU (of the device current then), hipFuncGetAttributes per kernel after that.
// Before any GPU use - and on a machine without one - the header's constants stand in.
struct DeviceLimits {
    int compute_units = 256;
    int64_t local_memory = STENCIL_LOCAL_MEM_BYTES;
    int max_wg = STENCIL_MAX_WG_SIZE;
    bool queried = false;
};
DeviceLimits g_limits;
std::mutex g_limits_mutex;
std::unordered_map<const void *, int> g_kernel_max_threads;

void query_device_limits() {
    std::lock_guard<std::mutex> lock(g_limits_mutex);
    if (g_limits.queried) return;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return;                       // keep the constants; a launch will report what is wrong
    }
    if (prop.multiProcessorCount > 0) g_limits.compute_units = prop.multiProcessorCount;
    if (prop.maxThreadsPerBlock > 0) g_limits.max_wg = prop.maxThreadsPerBlock;
    // what one workgroup can be given once a kernel's dynamic limit is raised: all of a compute unit's
    const int64_t lds = std::max<int64_t>((int64_t)prop.maxSharedMemoryPerMultiProcessor, (int64_t)prop.sharedMemPerBlock);
    if (lds > 0) g_limits.local_memory = lds;
    g_limits.queried = true;
}

}  // namespace

int64_t stencil_local_memory_limit() { return g_limits.local_memory; }

namespace {

// Plain copy: one 16-byte vector per work-item (tail bytes one by one).  The achievable
// read+write bandwidth the stencil kernels are compared with, and the known-size kernel that
// hardware traffic counters are calibrated against.
__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ in, uint4 *__restrict__ out,
                                                   size_t n_vec, size_t n_bytes) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_vec) out[i] = in[i];
    const size_t tail = n_vec * 16 + i;
    if (i < 16 && tail < n_bytes)
        reinterpret_cast<unsigned char *>(out)[tail] = reinterpret_cast<const unsigned char *>(in)[tail];
}

// A weight table travels to the device inside kernel arguments, 512 floats per launch: ordered on
// the caller's stream like the stencil launches that read it, no staging buffer, no allocation.
struct TableChunk { float v[512]; };
__global__ __launch_bounds__(512) void table_upload_kernel(float *dst, const TableChunk c, int offset, int n) {
    const int i = (int)threadIdx.x;
    if (i < n) dst[offset + i] = c.v[i];
}

hipError_t upload_table(float *dst, const std::vector<float> &w, hipStream_t stream) {
    for (size_t at = 0; at < w.size(); at += 512) {
        TableChunk c;
        const int n = (int)std::min<size_t>(512, w.size() - at);
        std::memcpy(c.v, w.data() + at, (size_t)n * sizeof(float));
        hipLaunchKernelGGL(table_upload_kernel, dim3(1), dim3(512), 0, stream, dst, c, (int)at, n);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- the buffer of stencil_run_static ---------------------------------------------------------
// Device memory the library needs beyond `in` and `out` - the run-time region's weight table and
// the matrix that iterated runs ping-pong through - for callers that must not allocate: one array
// per GPU, part of the code object, held until the process ends.  Host code never passes the
// array's name to the device (on the host it is only a stand-in for the symbol): the address is
// asked for once per device and kept.
constexpr size_t kStaticTableBytes = 32768;                       // 8192 weights (the largest region has 65 x 65)
constexpr size_t kStaticMatrixBytes = STENCIL_STATIC_MATRIX_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticTableBytes + kStaticMatrixBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

// The calling thread's current device's copy of `scratch` (each GPU holds its own, at its own address).
int static_scratch(unsigned char **ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(STENCIL_E_INVALID, "device index %d beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail_hip(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return STENCIL_OK;
}


const std::vector<Variant> &registry() {
    static const std::vector<Variant> reg = [] {
        std::vector<Variant> r;
        register_weighted_sum_tiles(r);
        register_sincos(r);
        register_unit_region_tiles(r);
        register_direct_and_temporal(r);
        register_streams(r);
        register_life_streams(r);
        register_wide_regions(r);
        register_runtime_march(r);
        return r;
    }();
    return reg;
}

// whether a variant compiled for any region within a largest one covers the scenario's region
bool within(const Variant &v, const stencil *s) {
    return v.hn == -2 && s->hn <= v.mn && s->hs <= v.ms && s->he <= v.me && s->hw <= v.mw;
}

// The variant that serves a scenario: a compile-time border region if one matches, else a kernel
// compiled for a largest region that holds it, else the run-time one.
const Variant *find_variant(const stencil *s) {
    const Variant *dyn = nullptr, *masked = nullptr;
    for (const Variant &v : registry()) {
        if (v.kernel != variant_kernel(s) || v.border != s->border || !rows_match(v, s->cr) || v.cc != s->cc ||
            v.staging != s->staging)
            continue;
        if (v.hn == s->hn && v.hs == s->hs && v.he == s->he && v.hw == s->hw) return &v;
        // among the masked variants the one with the smallest largest region
        if (within(v, s) && (!masked || v.mn + v.ms < masked->mn + masked->ms)) masked = &v;
        if (v.hn == -1) dyn = &v;
    }
    return masked ? masked : dyn;
}

bool mapping_supported(const stencil *s, int staging, int cr, int cc) {
    // the register-streaming kernels address a row's cells by 32-bit byte offsets
    if (staging == STENCIL_STAGING_STREAM && (uint64_t)s->cols * s->elem() >= (1ull << 32)) return false;
    for (const Variant &v : registry())
        if (v.kernel == variant_kernel(s) && v.border == s->border && v.staging == staging && rows_match(v, cr) && v.cc == cc &&
            (v.hn == -1 || within(v, s) || (v.hn == s->hn && v.hs == s->hs && v.he == s->he && v.hw == s->hw)))
            return true;
    return false;
}

// W_max(s): the kernel's own limit (its launch bounds; once the GPU is in use, what the runtime
// reports for the compiled kernel) within the device's.
int kernel_max_threads(const stencil *s, const Variant *v) {
    int lim = std::min(v->max_threads, g_limits.max_wg);
    if (!g_limits.queried || !v->kernel_of) return lim;
    const void *k = v->kernel_of(s);
    if (!k) return lim;
    std::lock_guard<std::mutex> lock(g_limits_mutex);
    auto it = g_kernel_max_threads.find(k);
    if (it == g_kernel_max_threads.end()) {
        hipFuncAttributes attr;
        int reported = lim;
        if (hipFuncGetAttributes(&attr, k) == hipSuccess && attr.maxThreadsPerBlock > 0)
            reported = attr.maxThreadsPerBlock;
        else
            (void)hipGetLastError();
        it = g_kernel_max_threads.emplace(k, reported).first;
    }
    return std::min(lim, it->second);
}

int check_legal(const stencil *s, const Variant *v, int wr, int wc) {
    if (!v) return fail(STENCIL_E_INVALID, "no kernel variant for this scenario");
    if (wr < 1 || wc < 1)
        return fail(STENCIL_E_REFUSED, "workgroup size %dx%d: dimensions must be >= 1", wr, wc);
    const int w_max = kernel_max_threads(s, v);
    if ((int64_t)wr * wc > w_max)
        return fail(STENCIL_E_REFUSED, "workgroup size %dx%d exceeds W_max = %d work-items", wr, wc, w_max);
    if (v->staging == STENCIL_STAGING_TEMPORAL && s->temporal_depth > STENCIL_MAX_TEMPORAL_DEPTH)
        return fail(STENCIL_E_INVALID, "the local-memory temporal kernels fuse at most %d applications (depth is %d)",
                    STENCIL_MAX_TEMPORAL_DEPTH, s->temporal_depth);
    if (v->staging == STENCIL_STAGING_STREAM && (wr * wc) % 64 != 0)
        return fail(STENCIL_E_REFUSED, "workgroup size %dx%d refused: this mapping gives each wavefront a strip, the "
                                       "workgroup must be whole wavefronts of 64 work-items", wr, wc);
    const TileGeom g = tile_geom(s, *v, wr, wc);
    if (g.lds_bytes > g_limits.local_memory)
        return fail(STENCIL_E_REFUSED, "workgroup size %dx%d refused: tile needs %lld bytes of local memory (limit %lld)",
                    wr, wc, (long long)g.lds_bytes, (long long)g_limits.local_memory);
    return STENCIL_OK;
}

int ensure_device_state(stencil *s, const Variant *v, bool need_scratch, hipStream_t stream) {
    query_device_limits();
    if (v->hn < 0 && !s->weights_uploaded) {
        // A replaced table goes into the other of two device tables, by launches ordered on this
        // run's stream: earlier launches (on any stream) keep reading the table they were given.
        const int slot = s->d_weights == s->d_tables[0] && s->d_tables[0] ? 1 : 0;
        if (!s->d_tables[slot]) {
            hipError_t e = hipMalloc((void **)&s->d_tables[slot], kStaticTableBytes);
            if (e != hipSuccess) return fail(STENCIL_E_RESOURCES, "hipMalloc(weights): %s", hipGetErrorString(e));
        }
        hipError_t e = upload_table(s->d_tables[slot], s->weights, stream);
        if (e != hipSuccess) return fail_hip(e, "weight table upload");
        s->d_weights = s->d_tables[slot];
        s->weights_uploaded = true;
    }
    s->table_in_use = s->d_weights;
    if (need_scratch && !s->scratch) {
        hipError_t e = hipMalloc(&s->scratch, s->bytes());
        if (e != hipSuccess) {
            s->scratch = nullptr;
            return fail(STENCIL_E_RESOURCES, "hipMalloc(scratch matrix, %zu bytes): %s", s->bytes(),
                        hipGetErrorString(e));
        }
    }
    return STENCIL_OK;
}

// Launches a run of `iters` applications takes: the fusing kernels make `temporal_depth` per launch.
int launches_of(const stencil *s, const Variant *v, int iters) {
    const int per = v->fuses ? s->temporal_depth : 1;
    return (iters + per - 1) / per;
}

// A launch the runtime turned down.  Section 3.1: some sizes within W_max are refused all the same
// and "can only be discovered emergently", by the launch failing; the caller takes another size
// (Section 4.2).  The errors that mean "not this configuration" - resources, configuration,
// argument - become STENCIL_E_REFUSED with the runtime's text; anything else is a runtime error.
int launch_failure(hipError_t e, int wr, int wc) {
    switch (e) {
    case hipErrorLaunchOutOfResources:
    case hipErrorInvalidConfiguration:
    case hipErrorInvalidValue:
    case hipErrorOutOfMemory:
    case hipErrorSharedObjectInitFailed:
        return fail(STENCIL_E_REFUSED, "workgroup size %dx%d refused at launch: %s", wr, wc, hipGetErrorString(e));
    default:
        return fail_hip(e, "kernel launch");
    }
}

// `iters` out-of-place applications ending in `out`, never writing `in`.
int run_checked(stencil *s, const Variant *v, const void *in, void *out, void *pingpong, int iters, int wr, int wc,
                hipStream_t stream) {
    if (s->out_dtype() != s->dtype && iters != 1)
        return fail(STENCIL_E_INVALID, "the output is of another element type than the input: exactly one application");
    if (iters == 0) {
        hipError_t e = hipMemcpyAsync(out, in, s->bytes(), hipMemcpyDeviceToDevice, stream);
        return e == hipSuccess ? STENCIL_OK : fail_hip(e, "hipMemcpyAsync");
    }
    // `per` applications per launch; the launches alternate between `out` and the scratch
    // matrix so that the last one lands in `out`
    const int per = v->fuses ? s->temporal_depth : 1;
    const int launches = launches_of(s, v, iters);
    const void *src = in;
    void *dst = (launches % 2 == 1) ? out : pingpong;
    for (int done = 0; done < iters;) {
        const int now = std::min(per, iters - done);
        const bool injected = s->fail_rows == -1 || (s->fail_rows == wr && s->fail_cols == wc);
        hipError_t e = injected ? hipErrorLaunchOutOfResources : v->launch(s, src, dst, wr, wc, now, stream);
        if (e != hipSuccess) return launch_failure(e, wr, wc);
        done += now;
        src = dst;
        dst = (dst == out) ? pingpong : out;
    }
    return STENCIL_OK;
}

int validate_buffers(const stencil *s, const void *in, const void *out) {
    if (!in || !out) return fail(STENCIL_E_INVALID, "in/out must not be NULL");
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out, n = s->bytes(), m = s->out_bytes();
    if (a < b + m && b < a + n) return fail(STENCIL_E_INVALID, "in and out overlap");
    if (a % s->elem() || b % s->out_elem()) return fail(STENCIL_E_INVALID, "in/out are not element-aligned");
    return STENCIL_OK;
}

// f(s) (Section 3.2): dataset, kernel and device features.
void scenario_features(const stencil *s, double *f) {
    const double taps = (double)(s->hn + s->hs + 1) * (s->he + s->hw + 1);
    f[0] = (double)s->rows;
    f[1] = (double)s->cols;
    f[2] = (double)s->elem();
    f[3] = s->hn;
    f[4] = s->hs;
    f[5] = s->he;
    f[6] = s->hw;
    f[7] = taps;
    f[8] = s->kernel == STENCIL_SINCOS ? 1.0 : 0.0;
    f[9] = (double)g_limits.compute_units;
    f[10] = (double)g_limits.local_memory;
    f[11] = (double)g_limits.max_wg;
    f[12] = (double)s->out_elem();
    // The paper counts a kernel's instructions in its compiled form; here the operations each
    // customising function states per cell, filled in by hand: arithmetic and comparisons ...
    double ops = 0.0, special = 0.0;
    switch (s->kernel) {
    case STENCIL_WEIGHTED_SUM: ops = 2.0 * taps - 1.0; break;           // a product per tap, the sum
    case STENCIL_LIFE: ops = 11.0; break;                               // 7 adds for 8 neighbours, two compares, and, or
    case STENCIL_HEAT: ops = 7.0; break;                                // three adds, 4u, the difference, alpha t, the sum
    case STENCIL_SINCOS: ops = 3.0 * taps + 1.0; special = 2.0; break;  // w sin + cos and the sums; one sine, one cosine
    case STENCIL_SOBEL: ops = 17.0; special = 1.0; break;               // 8 differences / sums, 2 fma, 2 squares, a sum; a root
    case STENCIL_NMS: ops = 8.0; break;                                 // four compares, two ands, an or, the selection
    case STENCIL_THRESHOLD: ops = 1.0; break;
    default: break;
    }
    f[13] = ops;
    f[14] = special;                                                    // ... of which on the transcendental unit
    f[15] = (double)s->border;
}

int classify_and_repair(const stencil *s, const Variant *v, const host_tuning::Classifier *c, const int *cand_rows,
                        const int *cand_cols, int n_cand, int handler, int baseline_rows, int baseline_cols,
                        uint64_t random, int *wg_rows, int *wg_cols) {
    double f[STENCIL_N_FEATURES];
    scenario_features(s, f);
    int wr = 0, wc = 0;
    if (!c->classify(f, STENCIL_N_FEATURES, &wr, &wc))
        return fail(STENCIL_E_INVALID, "classifier has no training pairs, or feature count differs");
    // Algorithm 1: a legal prediction is kept; otherwise the handler chooses
    if (check_legal(s, v, wr, wc) != STENCIL_OK) {
        if (handler == STENCIL_FALLBACK_BASELINE) {
            if (check_legal(s, v, baseline_rows, baseline_cols) != STENCIL_OK)
                return fail(STENCIL_E_REFUSED, "the baseline size %dx%d is not legal for this scenario", baseline_rows,
                            baseline_cols);
            wr = baseline_rows;
            wc = baseline_cols;
        } else {
            std::vector<int> legal;
            for (int k = 0; k < n_cand; ++k)
                if (check_legal(s, v, cand_rows[k], cand_cols[k]) == STENCIL_OK) legal.push_back(k);
            if (legal.empty()) return fail(STENCIL_E_REFUSED, "no legal candidate workgroup size");
            int pick = legal[0];
            if (handler == STENCIL_FALLBACK_RANDOM) {
                pick = legal[(size_t)(random % legal.size())];
            } else {
                double d_min = std::numeric_limits<double>::infinity();
                for (int k : legal) {
                    const double dr = cand_rows[k] - wr, dc = cand_cols[k] - wc;
                    const double d = std::sqrt(dr * dr + dc * dc);
                    if (d < d_min) {
                        d_min = d;
                        pick = k;
                    }
                }
            }
            wr = cand_rows[pick];
            wc = cand_cols[pick];
        }
    }
    *wg_rows = wr;
    *wg_cols = wc;
    return STENCIL_OK;
}

// The size stencil_run(0, 0) takes (Section 2: choosing it is the implementation's job): the best
// of the handle's last sweep; else what the attached classifier predicts for the scenario
// (Algorithm 1 over the power-of-two sizes); else a wave64-shaped default.
void default_wg(const stencil *s, const Variant *v, int *wr, int *wc) {
    if (s->best_rows > 0 && check_legal(s, v, s->best_rows, s->best_cols) == STENCIL_OK) {
        *wr = s->best_rows;
        *wc = s->best_cols;
        return;
    }
    // one wavefront wide, a few rows tall; shrink until the tile fits local memory
    int r = 4, c = 64;
    while (check_legal(s, v, r, c) != STENCIL_OK && (r > 1 || c > 1)) {
        if (r > 1) r /= 2; else c /= 2;
    }
    if (s->predictor) {
        std::vector<int> vals, cr, cc;
        host_tuning::size_values(STENCIL_ENUM_POW2, STENCIL_MAX_WG_SIZE, vals);
        for (int a : vals)
            for (int b : vals)
                if ((int64_t)a * b <= STENCIL_MAX_WG_SIZE) {
                    cr.push_back(a);
                    cc.push_back(b);
                }
        int pr = 0, pc = 0;
        if (classify_and_repair(s, v, reinterpret_cast<const host_tuning::Classifier *>(s->predictor), cr.data(), cc.data(),
                                (int)cr.size(), s->predictor_handler, r, c, 0, &pr, &pc) == STENCIL_OK) {
            r = pr;
            c = pc;
        }
    }
    *wr = r;
    *wc = c;
}

}  // namespace

constexpr int kWarmup = 3;   // untimed launches before the samples of a size (Section 5)

// ---- C ABI -----------------------------------------------------------------------------------

extern "C" {

const char *stencil_last_error(void) { return g_err; }

int stencil_create(stencil_t **out, int64_t rows, int64_t cols, int dtype, int halo_n, int halo_s,
                   int halo_e, int halo_w, int border_mode) {
    if (!out) return fail(STENCIL_E_INVALID, "out handle pointer is NULL");
    *out = nullptr;
    if (rows < 1 || cols < 1) return fail(STENCIL_E_INVALID, "rows and cols must be >= 1 (got %lld x %lld)",
                                          (long long)rows, (long long)cols);
    if (rows > INT32_MAX || cols > INT32_MAX || rows * cols > (int64_t)INT32_MAX)
        return fail(STENCIL_E_INVALID, "matrix too large: rows*cols must be < 2^31");
    if (dtype < STENCIL_F32 || dtype > STENCIL_F64) return fail(STENCIL_E_INVALID, "unknown dtype %d", dtype);
    const int h[4] = {halo_n, halo_s, halo_e, halo_w};
    for (int k = 0; k < 4; ++k)
        if (h[k] < 0 || h[k] > STENCIL_MAX_HALO)
            return fail(STENCIL_E_INVALID, "border region extents must be in [0, %d]", STENCIL_MAX_HALO);
    if (border_mode < STENCIL_CLAMP || border_mode > STENCIL_CONSTANT)
        return fail(STENCIL_E_INVALID, "unknown border mode %d", border_mode);
    stencil *s = new (std::nothrow) stencil;
    if (!s) return fail(STENCIL_E_RESOURCES, "out of host memory");
    s->rows = rows;
    s->cols = cols;
    s->dtype = dtype;
    s->hn = halo_n; s->hs = halo_s; s->he = halo_e; s->hw = halo_w;
    s->border = border_mode;
    if (dtype != STENCIL_U8) {
        s->kernel = STENCIL_WEIGHTED_SUM;
        s->weights.assign((size_t)(halo_n + halo_s + 1) * (halo_e + halo_w + 1), 0.0f);
    } else {
        s->kernel = -1;   // a U8 matrix has no default customising function
    }
    *out = s;
    return STENCIL_OK;
}

void stencil_destroy(stencil_t *s) {
    if (!s) return;
    for (hipEvent_t e : s->events) (void)hipEventDestroy(e);
    if (s->scratch) (void)hipFree(s->scratch);
    for (float *t : s->d_tables)
        if (t) (void)hipFree(t);
    delete s;
}

int stencil_set_kernel(stencil_t *s, int kernel_id, const float *weights, int n_weights,
                       const float *scalars, int n_scalars) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    const int cells = (s->hn + s->hs + 1) * (s->he + s->hw + 1);
    const bool unit_region = s->hn == 1 && s->hs == 1 && s->he == 1 && s->hw == 1;
    switch (kernel_id) {
    case STENCIL_WEIGHTED_SUM:
    case STENCIL_SINCOS:
        if (kernel_id == STENCIL_SINCOS && s->dtype != STENCIL_F32)
            return fail(STENCIL_E_INVALID, "this kernel is not available for the matrix's element type");
        if (!weights || n_weights != cells)
            return fail(STENCIL_E_INVALID, "weights must hold (N+S+1)*(E+W+1) = %d floats (got %d)", cells, n_weights);
        if (s->dtype == STENCIL_I32)
            for (int k = 0; k < cells; ++k)
                if (weights[k] != std::rint(weights[k]) || std::fabs(weights[k]) > 16777216.0f)
                    return fail(STENCIL_E_INVALID, "an I32 matrix needs integer weights (weights[%d] = %g)", k, weights[k]);
        s->weights.assign(weights, weights + cells);
        break;
    case STENCIL_LIFE:
        if (s->dtype != STENCIL_U8) return fail(STENCIL_E_INVALID, "LIFE needs a U8 matrix");
        if (!unit_region) return fail(STENCIL_E_INVALID, "LIFE needs border region 1/1/1/1");
        // the packed-byte kernels add cells without carries between bytes: every cell, the padding
        // value included, must be 0 or 1
        if (s->pad != 0.0 && s->pad != 1.0)
            return fail(STENCIL_E_INVALID, "LIFE needs a padding value of 0 or 1 (it is %g)", s->pad);
        s->weights.clear();
        break;
    case STENCIL_HEAT:
        if (s->dtype != STENCIL_F32) return fail(STENCIL_E_INVALID, "HEAT needs an F32 matrix");
        if (!unit_region) return fail(STENCIL_E_INVALID, "HEAT needs border region 1/1/1/1");
        if (!scalars || n_scalars < 1) return fail(STENCIL_E_INVALID, "HEAT needs scalars[0] = alpha");
        s->scalar0 = scalars[0];
        s->weights.clear();
        break;
    case STENCIL_SOBEL:
    case STENCIL_NMS:
        if (s->dtype != STENCIL_F32) return fail(STENCIL_E_INVALID, "SOBEL and NMS need an F32 matrix");
        if (!unit_region) return fail(STENCIL_E_INVALID, "SOBEL and NMS need border region 1/1/1/1");
        s->weights.clear();
        break;
    case STENCIL_THRESHOLD:
        if (s->dtype != STENCIL_F32) return fail(STENCIL_E_INVALID, "THRESHOLD needs an F32 matrix");
        if (s->hn || s->hs || s->he || s->hw) return fail(STENCIL_E_INVALID, "THRESHOLD has no border region (0/0/0/0)");
        if (!scalars || n_scalars < 1) return fail(STENCIL_E_INVALID, "THRESHOLD needs scalars[0] = level");
        s->scalar0 = scalars[0];
        s->weights.clear();
        break;
    default:
        return fail(STENCIL_E_INVALID, "unknown kernel id %d", kernel_id);
    }
    s->kernel = kernel_id;
    s->weights_uploaded = false;
    if (!mapping_supported(s, s->staging, s->cr, s->cc)) {
        s->staging = STENCIL_STAGING_LOCAL;
        s->cr = 1;
        s->cc = 1;
    }
    s->best_rows = s->best_cols = 0;
    return STENCIL_OK;
}

int stencil_set_border_value(stencil_t *s, double value) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (s->dtype == STENCIL_I32 && !(value == std::floor(value) && std::fabs(value) <= 2147483647.0))
        return fail(STENCIL_E_INVALID, "padding value of an I32 matrix must be an integer that fits");
    if (s->dtype == STENCIL_U8 && (value < 0 || value > 255 || value != std::floor(value)))
        return fail(STENCIL_E_INVALID, "padding value of a U8 matrix must be an integer in [0, 255]");
    if (s->kernel == STENCIL_LIFE && value > 1)
        return fail(STENCIL_E_INVALID, "LIFE cells are 0 or 1: the padding value must be too");
    s->pad = value;
    return STENCIL_OK;
}

int stencil_set_mapping(stencil_t *s, int staging, int cells_rows, int cells_cols) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (s->kernel < 0) return fail(STENCIL_E_INVALID, "select a kernel first");
    if (!mapping_supported(s, staging, cells_rows, cells_cols))
        return fail(STENCIL_E_INVALID, "mapping (staging %d, %dx%d cells per work-item) is not available for this scenario",
                    staging, cells_rows, cells_cols);
    s->staging = staging;
    s->cr = cells_rows;
    s->cc = cells_cols;
    s->best_rows = s->best_cols = 0;
    return STENCIL_OK;
}

int stencil_output_dtype(const stencil_t *s) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    return s->out_dtype();
}

int stencil_get_mapping(const stencil_t *s, int *staging, int *cells_rows, int *cells_cols) {
    if (!s || !staging || !cells_rows || !cells_cols) return fail(STENCIL_E_INVALID, "NULL argument");
    *staging = s->staging;
    *cells_rows = s->cr;
    *cells_cols = s->cc;
    return STENCIL_OK;
}

int stencil_stream_segment_rows(const stencil_t *s, int wavefronts_per_simd, int *cells_rows) {
    if (!s || !cells_rows) return fail(STENCIL_E_INVALID, "NULL argument");
    if (wavefronts_per_simd < 1) return fail(STENCIL_E_INVALID, "wavefronts per SIMD must be >= 1");
    const Variant *v = find_variant(s);
    if (s->staging != STENCIL_STAGING_STREAM || !v)
        return fail(STENCIL_E_INVALID, "the scenario is not on the register-streaming mapping");
    const int64_t strip_cols = tile_geom(s, *v, 1, 64).tw;
    const int64_t strips = (s->cols + strip_cols - 1) / strip_cols;
    const int64_t slots = (int64_t)g_limits.compute_units * 4 * wavefronts_per_simd;
    // as many segments per strip as the slots allow, at least one; then the shortest height that needs no more
    const int64_t segments = std::max<int64_t>(1, std::min<int64_t>(slots / strips, s->rows));
    const int64_t h = (s->rows + segments - 1) / segments;
    if (h > kMaxSegmentRows)
        return fail(STENCIL_E_REFUSED, "segments of %lld rows are beyond the kernels' %d", (long long)h, kMaxSegmentRows);
    *cells_rows = (int)h;
    return STENCIL_OK;
}

int stencil_set_option(stencil_t *s, int option, int value) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    switch (option) {
    case STENCIL_OPT_XCD_REMAP:
        s->xcd_remap = value ? 1 : 0;
        return STENCIL_OK;
    case STENCIL_OPT_NT_STORE:
        s->nt_store = value ? 1 : 0;
        return STENCIL_OK;
    case STENCIL_OPT_SWEEP_CUTOFF:
        if (value < 0 || (value > 0 && value < 100))
            return fail(STENCIL_E_INVALID, "sweep cutoff is a percentage >= 100, or 0 to sample every size fully");
        s->sweep_cutoff_pct = value;
        return STENCIL_OK;
    case STENCIL_OPT_TEMPORAL_DEPTH:
        if (value < 1 || value > STENCIL_MAX_STREAM_DEPTH)
            return fail(STENCIL_E_INVALID, "temporal depth must be in [1, %d]", STENCIL_MAX_STREAM_DEPTH);
        if (value > STENCIL_MAX_TEMPORAL_DEPTH && s->staging == STENCIL_STAGING_TEMPORAL)
            return fail(STENCIL_E_INVALID, "the local-memory temporal kernels fuse at most %d applications",
                        STENCIL_MAX_TEMPORAL_DEPTH);
        s->temporal_depth = value;
        s->best_rows = s->best_cols = 0;
        return STENCIL_OK;
    case STENCIL_OPT_FAIL_LAUNCH:
        if (value == 0) {
            s->fail_rows = s->fail_cols = 0;
        } else if (value == -1) {
            s->fail_rows = s->fail_cols = -1;
        } else {
            if (value < 0 || (value >> 16) < 1 || (value & 0xffff) < 1)
                return fail(STENCIL_E_INVALID, "STENCIL_OPT_FAIL_LAUNCH takes (w_r << 16) | w_c, -1 or 0");
            s->fail_rows = value >> 16;
            s->fail_cols = value & 0xffff;
        }
        return STENCIL_OK;
    default:
        return fail(STENCIL_E_INVALID, "unknown option %d", option);
    }
}

int stencil_max_wg_size(const stencil_t *s) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    const Variant *v = find_variant(s);
    if (!v) return fail(STENCIL_E_INVALID, "no kernel variant for this scenario");
    return kernel_max_threads(s, v);
}

int64_t stencil_tile_bytes(const stencil_t *s, int wg_rows, int wg_cols) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    const Variant *v = find_variant(s);
    if (!v || wg_rows < 1 || wg_cols < 1) return fail(STENCIL_E_INVALID, "bad scenario or workgroup size");
    return tile_geom(s, *v, wg_rows, wg_cols).lds_bytes;
}

int stencil_is_legal(const stencil_t *s, int wg_rows, int wg_cols) {
    if (!s) return 0;
    return check_legal(s, find_variant(s), wg_rows, wg_cols) == STENCIL_OK ? 1 : 0;
}

int stencil_enumerate_wg(int mode, int max_threads, int *rows, int *cols, int cap) {
    if (max_threads < 1 || cap < 0 || (cap > 0 && (!rows || !cols)))
        return fail(STENCIL_E_INVALID, "bad arguments to stencil_enumerate_wg");
    std::vector<int> vals;
    if (!host_tuning::size_values(mode, max_threads, vals)) return fail(STENCIL_E_INVALID, "unknown enumeration mode %d", mode);
    int n = 0;
    for (int r : vals)
        for (int c : vals)
            if ((int64_t)r * c <= max_threads) {
                if (n < cap) {
                    rows[n] = r;
                    cols[n] = c;
                }
                ++n;
            }
    return n;
}

int stencil_run(stencil_t *s, const void *in, void *out, int iters, int wg_rows, int wg_cols, void *stream) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (iters < 0) return fail(STENCIL_E_INVALID, "iters must be >= 0");
    int rc = validate_buffers(s, in, out);
    if (rc != STENCIL_OK) return rc;
    const Variant *v = find_variant(s);
    if (!v) return fail(STENCIL_E_INVALID, "no kernel selected for this scenario");
    query_device_limits();
    if (wg_rows == 0 && wg_cols == 0) default_wg(s, v, &wg_rows, &wg_cols);
    rc = check_legal(s, v, wg_rows, wg_cols);
    if (rc != STENCIL_OK) return rc;
    rc = ensure_device_state(s, v, launches_of(s, v, iters) > 1, (hipStream_t)stream);
    if (rc != STENCIL_OK) return rc;
    rc = run_checked(s, v, in, out, s->scratch, iters, wg_rows, wg_cols, (hipStream_t)stream);
    if (rc == STENCIL_OK) g_err[0] = '\0';
    return rc;
}

int stencil_run_static(stencil_t *s, const void *in, void *out, int iters, int wg_rows, int wg_cols, void *stream_) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (iters < 0) return fail(STENCIL_E_INVALID, "iters must be >= 0");
    int rc = validate_buffers(s, in, out);
    if (rc != STENCIL_OK) return rc;
    const Variant *v = find_variant(s);
    if (!v) return fail(STENCIL_E_INVALID, "no kernel selected for this scenario");
    query_device_limits();
    if (wg_rows == 0 && wg_cols == 0) default_wg(s, v, &wg_rows, &wg_cols);
    rc = check_legal(s, v, wg_rows, wg_cols);
    if (rc != STENCIL_OK) return rc;
    // what this run needs beyond in / out must fit the fixed buffer
    const bool needs_matrix = launches_of(s, v, iters) > 1;
    if (needs_matrix && s->bytes() > kStaticMatrixBytes)
        return fail(STENCIL_E_INVALID, "stencil_run_static: a run of %d launches ping-pongs through a matrix of %zu bytes, "
                                       "the fixed buffer holds %zu", launches_of(s, v, iters), s->bytes(), kStaticMatrixBytes);
    const bool needs_table = v->hn < 0;
    if (needs_table && s->weights.size() * sizeof(float) > kStaticTableBytes)
        return fail(STENCIL_E_INVALID, "stencil_run_static: weight table of %zu bytes, the fixed buffer holds %zu",
                    s->weights.size() * sizeof(float), kStaticTableBytes);
    unsigned char *buf = nullptr;
    rc = static_scratch(&buf);
    if (rc != STENCIL_OK) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    float *table = reinterpret_cast<float *>(buf);
    void *matrix = buf + kStaticTableBytes;
    if (needs_table) {
        // the buffer keeps whatever the last call (of any handle) left: this run's table goes in
        // first, ordered on the stream before the launches that read it
        hipError_t e = upload_table(table, s->weights, stream);
        if (e != hipSuccess) return fail_hip(e, "weight table upload");
    }
    // every launch writes its whole destination matrix before the next reads it: nothing to clear
    s->table_in_use = table;
    rc = run_checked(s, v, in, out, matrix, iters, wg_rows, wg_cols, stream);
    s->table_in_use = s->d_weights;
    if (rc == STENCIL_OK) g_err[0] = '\0';
    return rc;
}

int stencil_set_sweep_rotation(stencil_t *s, const void *const *ins, void *const *outs, int n) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (n < 0 || n > STENCIL_MAX_ROTATION || (n > 0 && (!ins || !outs)))
        return fail(STENCIL_E_INVALID, "a rotation has 0..%d matrix pairs", STENCIL_MAX_ROTATION);
    std::vector<std::pair<const void *, void *>> pairs;
    for (int k = 0; k < n; ++k) {
        int rc = validate_buffers(s, ins[k], outs[k]);
        if (rc != STENCIL_OK) return rc;
        // an output that another pair reads or writes would make the applications depend on each other
        const uintptr_t o = (uintptr_t)outs[k], m = s->out_bytes();
        for (int j = 0; j < n; ++j) {
            if (j == k) continue;
            const uintptr_t a = (uintptr_t)ins[j], b = (uintptr_t)outs[j];
            if ((o < a + s->bytes() && a < o + m) || (o < b + m && b < o + m))
                return fail(STENCIL_E_INVALID, "output %d overlaps a matrix of pair %d", k, j);
        }
        pairs.emplace_back(ins[k], outs[k]);
    }
    s->rotation.swap(pairs);
    s->rotation_at = 0;
    return STENCIL_OK;
}

int stencil_sweep_wg(stencil_t *s, const void *in, void *out, int iters, const int *wg_rows_list,
                     const int *wg_cols_list, int n, int fixed_rows, int fixed_cols, int reps,
                     double *mean_ms, double *min_ms, double *median_ms, double *stddev_ms, int *status,
                     int *best_index, double *speedup_over_fixed, void *stream_) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (n < 0 || (n > 0 && (!wg_rows_list || !wg_cols_list))) return fail(STENCIL_E_INVALID, "bad size list");
    if (iters < 1) return fail(STENCIL_E_INVALID, "a sweep needs iters >= 1");
    int rc = validate_buffers(s, in, out);
    if (rc != STENCIL_OK) return rc;
    const Variant *v = find_variant(s);
    if (!v) return fail(STENCIL_E_INVALID, "no kernel selected for this scenario");
    if (reps <= 0) reps = 30;
    hipStream_t stream = (hipStream_t)stream_;
    // (single applications on a rotation of pairs need no ping-pong matrix)
    rc = ensure_device_state(s, v, s->rotation.empty() && launches_of(s, v, iters) > 1, stream);
    if (rc != STENCIL_OK) return rc;
    // event pairs for the samples, made when the first size is actually timed
    auto need_events = [&]() -> int {
        while ((int)s->events.size() < 2 * reps) {
            hipEvent_t e;
            hipError_t he = hipEventCreate(&e);
            if (he != hipSuccess) return fail_hip(he, "hipEventCreate");
            s->events.push_back(e);
        }
        return STENCIL_OK;
    };
    const double nan = std::numeric_limits<double>::quiet_NaN();
    std::vector<double> samples((size_t)reps);
    // The applications of one sample: a chain in -> out of `iters` applications, or, with a rotation of
    // matrix pairs set, `iters` independent single applications, each on the pair whose turn it is.
    auto run_sample = [&](int wr, int wc) -> int {
        if (s->rotation.empty()) return run_checked(s, v, in, out, s->scratch, iters, wr, wc, stream);
        for (int i = 0; i < iters; ++i) {
            const auto &pair = s->rotation[s->rotation_at++ % s->rotation.size()];
            int r = run_checked(s, v, pair.first, pair.second, s->scratch, 1, wr, wc, stream);
            if (r != STENCIL_OK) return r;
        }
        return STENCIL_OK;
    };

    std::vector<double> means((size_t)n + 1, nan);
    std::vector<int> stat((size_t)n + 1, STENCIL_E_REFUSED);

    // times one size into slot k; returns STENCIL_OK also when the size is refused
    // probe_only: one warm-up and two samples instead of three warm-ups and `reps` samples
    auto time_size = [&](int wr, int wc, int k, bool probe_only) -> int {
        // a size that is not legal, or that the runtime refuses when it is launched (Section 3.1's
        // refused parameters show only then): recorded, and the sweep goes on
        auto refused = [&]() -> int {
            stat[k] = STENCIL_E_REFUSED;
            means[k] = nan;
            if (k < n) {
                if (min_ms) min_ms[k] = nan;
                if (median_ms) median_ms[k] = nan;
                if (stddev_ms) stddev_ms[k] = nan;
            }
            return STENCIL_OK;
        };
        if (check_legal(s, v, wr, wc) != STENCIL_OK) return refused();
        // samples [from, to) into the event pairs, then wait for them and read the times
        auto take = [&](int from, int to) -> int {
            for (int i = from; i < to; ++i) {
                hipError_t e = hipEventRecord(s->events[2 * i], stream);
                if (e != hipSuccess) return fail_hip(e, "hipEventRecord");
                int r = run_sample(wr, wc);
                if (r != STENCIL_OK) return r;
                e = hipEventRecord(s->events[2 * i + 1], stream);
                if (e != hipSuccess) return fail_hip(e, "hipEventRecord");
            }
            if (to > from) {
                hipError_t e = hipEventSynchronize(s->events[2 * to - 1]);
                if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize");
            }
            for (int i = from; i < to; ++i) {
                float ms = 0.0f;
                hipError_t e = hipEventElapsedTime(&ms, s->events[2 * i], s->events[2 * i + 1]);
                if (e != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
                samples[i] = ms;
            }
            return STENCIL_OK;
        };
        const int taken = probe_only ? std::min(2, reps) : reps;
        for (int w = 0; w < (probe_only ? 1 : kWarmup); ++w) {
            int r = run_sample(wr, wc);
            if (r == STENCIL_E_REFUSED) return refused();
            if (r != STENCIL_OK) return r;
        }
        {
            int r = need_events();
            if (r == STENCIL_OK) r = take(0, taken);
            if (r == STENCIL_E_REFUSED) return refused();
            if (r != STENCIL_OK) return r;
        }
        samples.resize((size_t)taken);
        host_tuning::SampleStats st = host_tuning::summarise(samples);
        samples.resize((size_t)reps);
        means[k] = st.mean;
        stat[k] = STENCIL_OK;

        if (k < n) {
            if (min_ms) min_ms[k] = st.min;
            if (median_ms) median_ms[k] = st.median;
            if (stddev_ms) stddev_ms[k] = st.stddev;
        }
        return STENCIL_OK;
    };

    if (s->sweep_cutoff_pct > 0 && reps > 2) {
        // adaptive sampling: probe every size, then sample fully only those within reach of the best
        double best_probe = std::numeric_limits<double>::infinity();
        for (int k = 0; k < n; ++k) {
            rc = time_size(wg_rows_list[k], wg_cols_list[k], k, true);
            if (rc != STENCIL_OK) return rc;
            if (stat[k] == STENCIL_OK) best_probe = std::min(best_probe, means[k]);
        }
        for (int k = 0; k < n; ++k) {
            if (stat[k] != STENCIL_OK || means[k] * 100.0 > best_probe * s->sweep_cutoff_pct) continue;
            rc = time_size(wg_rows_list[k], wg_cols_list[k], k, false);
            if (rc != STENCIL_OK) return rc;
        }
    } else {
        for (int k = 0; k < n; ++k) {
            rc = time_size(wg_rows_list[k], wg_cols_list[k], k, false);
            if (rc != STENCIL_OK) return rc;
        }
    }
    double fixed_ms = nan;
    if (fixed_rows > 0 && fixed_cols > 0) {
        int at = -1;
        for (int k = 0; k < n; ++k)
            if (wg_rows_list[k] == fixed_rows && wg_cols_list[k] == fixed_cols) { at = k; break; }
        if (at < 0) {
            rc = time_size(fixed_rows, fixed_cols, n, false);
            if (rc != STENCIL_OK) return rc;
            at = n;
        }
        if (stat[at] == STENCIL_OK) fixed_ms = means[at];
    }
    int best = -1;
    double speedup = nan;
    host_tuning::reduce(wg_rows_list, wg_cols_list, n, means.data(), stat.data(), fixed_ms, &best, nullptr, &speedup);
    for (int k = 0; k < n; ++k) {
        if (mean_ms) mean_ms[k] = means[k];
        if (status) status[k] = stat[k];
    }
    if (best_index) *best_index = best;
    if (speedup_over_fixed) *speedup_over_fixed = speedup;
    if (best >= 0) {
        s->best_rows = wg_rows_list[best];
        s->best_cols = wg_cols_list[best];
    }
    return STENCIL_OK;
}

int stencil_sweep_configs(stencil_t *s, const void *in, void *out, int iters, const stencil_config_t *configs, int n,
                          int reps, double *mean_ms, int *status, int *best_index, void *stream) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (n < 0 || (n > 0 && !configs) || !mean_ms || !status) return fail(STENCIL_E_INVALID, "bad configuration list");
    if (iters < 1) return fail(STENCIL_E_INVALID, "a sweep needs iters >= 1");
    int rc = validate_buffers(s, in, out);
    if (rc != STENCIL_OK) return rc;
    const double nan = std::numeric_limits<double>::quiet_NaN();
    const int staging0 = s->staging, cr0 = s->cr, cc0 = s->cc, depth0 = s->temporal_depth, remap0 = s->xcd_remap;
    const int nt0 = s->nt_store;
    int best = -1;
    for (int k = 0; k < n; ++k) {
        const stencil_config_t &c = configs[k];
        mean_ms[k] = nan;
        status[k] = STENCIL_E_INVALID;
        // a mapping the scenario does not have, or a depth the mapping does not have: skipped
        s->temporal_depth = depth0;       // "as is" means as it was when the sweep began
        s->xcd_remap = c.xcd_remap < 0 ? remap0 : (c.xcd_remap ? 1 : 0);
        s->nt_store = c.nt_store < 0 ? nt0 : (c.nt_store ? 1 : 0);
        if (stencil_set_mapping(s, c.staging, c.cells_rows, c.cells_cols) != STENCIL_OK) continue;
        if (c.depth != 0 && stencil_set_option(s, STENCIL_OPT_TEMPORAL_DEPTH, c.depth) != STENCIL_OK) continue;
        const Variant *v = find_variant(s);
        if (v && check_legal(s, v, c.wg_rows, c.wg_cols) == STENCIL_E_INVALID) continue;
        int st = STENCIL_E_REFUSED, b = -1;
        rc = stencil_sweep_wg(s, in, out, iters, &c.wg_rows, &c.wg_cols, 1, 0, 0, reps, &mean_ms[k], nullptr, nullptr,
                              nullptr, &st, &b, nullptr, stream);
        if (rc != STENCIL_OK) break;      // a runtime error ends the sweep
        status[k] = st;
        if (st == STENCIL_OK && (best < 0 || mean_ms[k] < mean_ms[best])) best = k;
    }
    if (rc == STENCIL_OK && best >= 0) {
        // leave the scenario on the fastest configuration, remembered for stencil_run(0, 0)
        const stencil_config_t &c = configs[best];
        s->temporal_depth = depth0;
        s->xcd_remap = c.xcd_remap < 0 ? remap0 : (c.xcd_remap ? 1 : 0);
        s->nt_store = c.nt_store < 0 ? nt0 : (c.nt_store ? 1 : 0);
        (void)stencil_set_mapping(s, c.staging, c.cells_rows, c.cells_cols);
        if (c.depth != 0) (void)stencil_set_option(s, STENCIL_OPT_TEMPORAL_DEPTH, c.depth);
        s->best_rows = c.wg_rows;
        s->best_cols = c.wg_cols;
    } else {
        s->staging = staging0;
        s->cr = cr0;
        s->cc = cc0;
        s->temporal_depth = depth0;
        s->xcd_remap = remap0;
        s->nt_store = nt0;
        s->best_rows = s->best_cols = 0;
    }
    if (best_index) *best_index = best;
    if (rc == STENCIL_OK) g_err[0] = '\0';
    return rc;
}

int stencil_device_copy(const void *in, void *out, int64_t bytes, void *stream) {
    if (!in || !out || bytes < 0) return fail(STENCIL_E_INVALID, "bad arguments to stencil_device_copy");
    if ((uintptr_t)in % 16 || (uintptr_t)out % 16) return fail(STENCIL_E_INVALID, "buffers must be 16-byte aligned");
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if (a < b + (uintptr_t)bytes && b < a + (uintptr_t)bytes) return fail(STENCIL_E_INVALID, "in and out overlap");
    if (bytes == 0) return STENCIL_OK;
    const size_t n_vec = (size_t)bytes / 16;
    const size_t threads = std::max<size_t>(n_vec, 16);
    const size_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffull) return fail(STENCIL_E_INVALID, "copy too large for one launch");
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       static_cast<const uint4 *>(in), static_cast<uint4 *>(out), n_vec, (size_t)bytes);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? STENCIL_OK : fail_hip(e, "copy kernel launch");
}

int stencil_time_copy(const void *in, void *out, int64_t bytes, int burst, int reps, double *mean_ms,
                      double *min_ms, void *stream_) {
    if (burst < 1 || reps < 1 || !mean_ms) return fail(STENCIL_E_INVALID, "bad arguments to stencil_time_copy");
    hipStream_t stream = (hipStream_t)stream_;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return fail_hip(e, "hipEventCreate");
    }
    int rc = STENCIL_OK;
    double sum = 0.0, lo = 0.0;
    // the sweep's protocol: warm-up launches, then `reps` samples, a sample being a burst of launches
    for (int i = -kWarmup; i < reps && rc == STENCIL_OK; ++i) {
        if ((e = hipEventRecord(e0, stream)) != hipSuccess) { rc = fail_hip(e, "hipEventRecord"); break; }
        for (int b = 0; b < burst && rc == STENCIL_OK; ++b) rc = stencil_device_copy(in, out, bytes, stream_);
        if (rc != STENCIL_OK) break;
        if ((e = hipEventRecord(e1, stream)) != hipSuccess) { rc = fail_hip(e, "hipEventRecord"); break; }
        if ((e = hipEventSynchronize(e1)) != hipSuccess) { rc = fail_hip(e, "hipEventSynchronize"); break; }
        float ms = 0.0f;
        if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) { rc = fail_hip(e, "hipEventElapsedTime"); break; }
        if (i < 0) continue;
        const double per = (double)ms / burst;
        sum += per;
        lo = (i == 0 || per < lo) ? per : lo;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != STENCIL_OK) return rc;
    *mean_ms = sum / reps;
    if (min_ms) *min_ms = lo;
    return STENCIL_OK;
}

int stencil_sweep_reduce(const int *wg_rows_list, const int *wg_cols_list, int n, const double *mean_ms,
                         const int *status, double fixed_ms, int *best_index, double *performance,
                         double *speedup_over_fixed) {
    if (n < 0 || (n > 0 && (!wg_rows_list || !wg_cols_list || !mean_ms || !status)))
        return fail(STENCIL_E_INVALID, "bad arguments to stencil_sweep_reduce");
    host_tuning::reduce(wg_rows_list, wg_cols_list, n, mean_ms, status, fixed_ms, best_index, performance,
                        speedup_over_fixed);
    return STENCIL_OK;
}

int stencil_baseline_wg(const double *performance, int n_scenarios, int n_sizes, int *best_index) {
    if (!performance || !best_index || n_scenarios < 1 || n_sizes < 1)
        return fail(STENCIL_E_INVALID, "bad arguments to stencil_baseline_wg");
    *best_index = host_tuning::baseline_index(performance, n_scenarios, n_sizes);
    return STENCIL_OK;
}

int stencil_features(const stencil_t *s, double *f) {
    if (!s || !f) return fail(STENCIL_E_INVALID, "NULL argument");
    scenario_features(s, f);
    return STENCIL_OK;
}

int stencil_predictor_create(stencil_predictor_t **out, int classifier) {
    if (!out) return fail(STENCIL_E_INVALID, "NULL argument");
    *out = nullptr;
    if (classifier < STENCIL_CLASSIFIER_NEAREST || classifier > STENCIL_CLASSIFIER_ZEROR)
        return fail(STENCIL_E_INVALID, "unknown classifier %d", classifier);
    *out = reinterpret_cast<stencil_predictor_t *>(new (std::nothrow) host_tuning::Classifier(classifier));
    return *out ? STENCIL_OK : fail(STENCIL_E_RESOURCES, "out of host memory");
}

void stencil_predictor_destroy(stencil_predictor_t *p) {
    delete reinterpret_cast<host_tuning::Classifier *>(p);
}

int stencil_predictor_add(stencil_predictor_t *p, const double *features, int n_features, int wg_rows, int wg_cols) {
    if (!p || !features || n_features < 1 || wg_rows < 1 || wg_cols < 1) return fail(STENCIL_E_INVALID, "bad arguments");
    auto *c = reinterpret_cast<host_tuning::Classifier *>(p);
    if (!c->add(features, n_features, wg_rows, wg_cols))
        return fail(STENCIL_E_INVALID, "feature count %d differs from earlier training pairs", n_features);
    return STENCIL_OK;
}

int stencil_predictor_classify(const stencil_predictor_t *p, const double *features, int n_features,
                               int *wg_rows, int *wg_cols) {
    if (!p || !features || !wg_rows || !wg_cols) return fail(STENCIL_E_INVALID, "NULL argument");
    auto *c = reinterpret_cast<const host_tuning::Classifier *>(p);
    if (!c->classify(features, n_features, wg_rows, wg_cols))
        return fail(STENCIL_E_INVALID, "classifier has no training pairs, or feature count differs");
    return STENCIL_OK;
}

int stencil_predict_wg(const stencil_t *s, const stencil_predictor_t *p, const int *cand_rows, const int *cand_cols,
                       int n_cand, int handler, int baseline_rows, int baseline_cols, uint64_t random,
                       int *wg_rows, int *wg_cols) {
    if (!s || !p || !wg_rows || !wg_cols || n_cand < 0 || (n_cand > 0 && (!cand_rows || !cand_cols)))
        return fail(STENCIL_E_INVALID, "bad arguments");
    if (handler < STENCIL_FALLBACK_NEAREST || handler > STENCIL_FALLBACK_RANDOM)
        return fail(STENCIL_E_INVALID, "unknown fallback handler %d", handler);
    const Variant *v = find_variant(s);
    int wr = 0, wc = 0;
    int rc = classify_and_repair(s, v, reinterpret_cast<const host_tuning::Classifier *>(p), cand_rows, cand_cols, n_cand,
                                 handler, baseline_rows, baseline_cols, random, &wr, &wc);
    if (rc != STENCIL_OK) return rc;
    g_err[0] = '\0';
    *wg_rows = wr;
    *wg_cols = wc;
    return STENCIL_OK;
}

int stencil_attach_predictor(stencil_t *s, const stencil_predictor_t *p, int handler) {
    if (!s) return fail(STENCIL_E_INVALID, "handle is NULL");
    if (handler < STENCIL_FALLBACK_NEAREST || handler > STENCIL_FALLBACK_RANDOM)
        return fail(STENCIL_E_INVALID, "unknown fallback handler %d", handler);
    s->predictor = p;
    s->predictor_handler = handler;
    return STENCIL_OK;
}

int stencil_default_wg(const stencil_t *s, int *wg_rows, int *wg_cols) {
    if (!s || !wg_rows || !wg_cols) return fail(STENCIL_E_INVALID, "NULL argument");
    const Variant *v = find_variant(s);
    if (!v) return fail(STENCIL_E_INVALID, "no kernel selected for this scenario");
    default_wg(s, v, wg_rows, wg_cols);
    return STENCIL_OK;
}

int stencil_predictor_load(stencil_predictor_t **out, const char *path, int classifier) {
    if (!out || !path) return fail(STENCIL_E_INVALID, "NULL argument");
    *out = nullptr;
    FILE *fh = std::fopen(path, "r");
    if (!fh) return fail(STENCIL_E_INVALID, "cannot open %s", path);
    stencil_predictor_t *p = nullptr;
    int rc = stencil_predictor_create(&p, classifier);
    int n_features = 0, line_no = 0, pairs = 0;
    char line[8192];
    while (rc == STENCIL_OK && std::fgets(line, sizeof(line), fh)) {
        ++line_no;
        char *at = line;
        while (*at == ' ' || *at == '\t') ++at;
        if (*at == '#' || *at == '\n' || *at == '\r' || *at == '\0') continue;
        if (n_features == 0) {
            if (std::sscanf(at, "features %d", &n_features) != 1 || n_features < 1 || n_features > 256)
                rc = fail(STENCIL_E_INVALID, "%s:%d: expected \"features <count>\"", path, line_no);
            continue;
        }
        std::vector<double> row;
        char *end = at;
        for (;;) {
            const double x = std::strtod(at, &end);
            if (end == at) break;
            row.push_back(x);
            at = end;
        }
        if ((int)row.size() != n_features + 2 || row[(size_t)n_features] < 1 || row[(size_t)n_features + 1] < 1)
            rc = fail(STENCIL_E_INVALID, "%s:%d: expected %d features and a workgroup size", path, line_no, n_features);
        else
            rc = stencil_predictor_add(p, row.data(), n_features, (int)row[(size_t)n_features], (int)row[(size_t)n_features + 1]);
        ++pairs;
    }
    std::fclose(fh);
    if (rc == STENCIL_OK && pairs == 0) rc = fail(STENCIL_E_INVALID, "%s holds no training pairs", path);
    if (rc != STENCIL_OK) {
        stencil_predictor_destroy(p);
        return rc;
    }
    *out = p;
    return STENCIL_OK;
}

int stencil_regressor_create(stencil_regressor_t **out) {
    if (!out) return fail(STENCIL_E_INVALID, "NULL argument");
    *out = reinterpret_cast<stencil_regressor_t *>(new (std::nothrow) host_tuning::Regressor);
    return *out ? STENCIL_OK : fail(STENCIL_E_RESOURCES, "out of host memory");
}

void stencil_regressor_destroy(stencil_regressor_t *r) { delete reinterpret_cast<host_tuning::Regressor *>(r); }

int stencil_regressor_add(stencil_regressor_t *r, const double *features, int n_features, int wg_rows, int wg_cols,
                          double value) {
    if (!r || !features || n_features < 1 || wg_rows < 1 || wg_cols < 1 || std::isnan(value))
        return fail(STENCIL_E_INVALID, "bad arguments");
    if (!reinterpret_cast<host_tuning::Regressor *>(r)->add(features, n_features, wg_rows, wg_cols, value))
        return fail(STENCIL_E_INVALID, "feature count %d differs from earlier tuples", n_features);
    return STENCIL_OK;
}

int stencil_regressor_predict(const stencil_regressor_t *r, const double *features, int n_features, int wg_rows,
                              int wg_cols, double *value) {
    if (!r || !features || !value) return fail(STENCIL_E_INVALID, "NULL argument");
    auto *reg = reinterpret_cast<const host_tuning::Regressor *>(r);
    if (reg->n_features() != n_features) return fail(STENCIL_E_INVALID, "regressor is empty, or feature count differs");
    *value = reg->predict(features, wg_rows, wg_cols);
    return STENCIL_OK;
}

int stencil_regressor_fit_forest(stencil_regressor_t *r, int n_trees, int n_rows, const int *bootstrap,
                                 const unsigned char *masks, int min_leaf, int max_depth) {
    if (!r) return fail(STENCIL_E_INVALID, "NULL argument");
    auto *reg = reinterpret_cast<host_tuning::Regressor *>(r);
    if (reg->n_tuples() == 0) return fail(STENCIL_E_INVALID, "the regressor holds no tuples");
    if (!reg->fit_forest(n_trees, n_rows, bootstrap, masks, min_leaf, max_depth))
        return fail(STENCIL_E_INVALID, "bad forest description (tree count, bootstrap index, input mask or limits)");
    return STENCIL_OK;
}

int stencil_predict_wg_regression(const stencil_t *s, const stencil_regressor_t *r, const int *cand_rows,
                                  const int *cand_cols, int n_cand, int fitness, int *wg_rows, int *wg_cols,
                                  int *n_refused) {
    if (!s || !r || !wg_rows || !wg_cols || n_cand < 0 || (n_cand > 0 && (!cand_rows || !cand_cols)))
        return fail(STENCIL_E_INVALID, "bad arguments");
    if (fitness != STENCIL_FITNESS_RECIPROCAL && fitness != STENCIL_FITNESS_IDENTITY)
        return fail(STENCIL_E_INVALID, "unknown fitness function %d", fitness);
    auto *reg = reinterpret_cast<const host_tuning::Regressor *>(r);
    double f[STENCIL_N_FEATURES];
    int rc = stencil_features(s, f);
    if (rc != STENCIL_OK) return rc;
    if (reg->n_features() != STENCIL_N_FEATURES) return fail(STENCIL_E_INVALID, "regressor is empty, or feature count differs");
    const Variant *v = find_variant(s);
    if (!v) return fail(STENCIL_E_INVALID, "no kernel variant for this scenario");
    // Algorithm 2: candidates within W_max; best by fitness of the prediction; a refused
    // parameter is struck from the pool and the next best taken
    std::vector<int> pool;
    std::vector<double> fit;
    for (int k = 0; k < n_cand; ++k) {
        if (cand_rows[k] < 1 || cand_cols[k] < 1 || (int64_t)cand_rows[k] * cand_cols[k] > kernel_max_threads(s, v)) continue;
        const double y = reg->predict(f, cand_rows[k], cand_cols[k]);
        if (std::isnan(y)) continue;
        pool.push_back(k);
        fit.push_back(fitness == STENCIL_FITNESS_RECIPROCAL ? 1.0 / y : y);
    }
    int refused = 0;
    while (!pool.empty()) {
        size_t best = 0;
        for (size_t i = 1; i < pool.size(); ++i)
            if (fit[i] > fit[best]) best = i;
        const int k = pool[best];
        if (check_legal(s, v, cand_rows[k], cand_cols[k]) == STENCIL_OK) {
            g_err[0] = '\0';
            *wg_rows = cand_rows[k];
            *wg_cols = cand_cols[k];
            if (n_refused) *n_refused = refused;
            return STENCIL_OK;
        }
        ++refused;
        pool.erase(pool.begin() + (long)best);
        fit.erase(fit.begin() + (long)best);
    }
    return fail(STENCIL_E_REFUSED, "no legal candidate workgroup size");
}

}  // extern "C"
