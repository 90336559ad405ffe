/*
 * libstencil - 2D stencil skeleton with a tunable workgroup size, for AMD MI355X (gfx950).
 *
 * The operation is the stencil pattern of Section 2 of "Autotuning OpenCL Workgroup Size
 * for Stencil Patterns" (arXiv 1511.02490): a customising function is applied to every
 * element of a 2D matrix; it sees the element and a rectangular border region of
 * `north`, `south`, `east`, `west` cells around it; neighbours outside the matrix are
 * substituted by the nearest in-matrix cell or by a padding constant (periodic wrap is
 * provided in addition).  The matrix is decomposed into workgroups of w_r x w_c work-items
 * (Figure 1), each staging a tile plus perimeter border region in local memory; the
 * workgroup size is the tunable parameter, and the sweep of Section 5 times every size.
 *
 * Conventions: matrices are contiguous row-major a[r][c]; north = smaller r, south = larger
 * r, west = smaller c, east = larger c; the region includes the centre.  Weight tables are
 * (north+south+1) x (east+west+1), row-major, applied as a correlation:
 *   out[r][c] = sum_{dr=-north..south} sum_{dc=-west..east} w[dr+north][dc+west] * V(r+dr, c+dc)
 * where V substitutes out-of-matrix positions according to the border mode.
 *
 * Pointers named `in` / `out` are DEVICE pointers owned by the caller.  Every other pointer
 * is a HOST pointer.  All functions return STENCIL_OK (0) or a negative stencil_status and
 * never abort or throw; `stencil_last_error()` gives the text of the calling thread's last
 * failure.  Functions that take no `in`/`out` make no GPU call and work on a machine
 * without a GPU.
 *
 * Ownership and concurrency: a handle (stencil_t, predictor, regressor) belongs to its
 * creator until the matching destroy call; different handles may be used from different
 * threads at once, one handle from one thread at a time.  A stencil_t owns device memory on
 * the device that was current when it first ran (a scratch matrix for iterated runs, the
 * weight table of a run-time region): use it with that device current, and do not overlap
 * iterated runs of one handle on different streams - they share the scratch matrix.
 */
#ifndef LIBSTENCIL_H
#define LIBSTENCIL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct stencil stencil_t;
typedef struct stencil_predictor stencil_predictor_t;
typedef struct stencil_regressor stencil_regressor_t;

enum stencil_status {
    STENCIL_OK = 0,
    STENCIL_E_INVALID = -1,   /* bad argument: null, out of range, aliasing buffers        */
    STENCIL_E_REFUSED = -2,   /* workgroup size not legal for this scenario (Section 3.1:
                                 over W_max, or a "refused parameter": tile exceeds local
                                 memory)                                                  */
    STENCIL_E_RESOURCES = -3, /* allocation failed                                         */
    STENCIL_E_HIP = -4        /* HIP runtime error; text in stencil_last_error()           */
};

/* Element types (Section 3.3: integers, single or double precision; U8 for cellular automata). */
enum stencil_dtype { STENCIL_F32 = 0, STENCIL_U8 = 1, STENCIL_I32 = 2, STENCIL_F64 = 3 };

/* Border substitution (Section 2): CLAMP = value of the nearest cell within the matrix,
 * CONSTANT = predefined padding value, WRAP = periodic (true modulo). */
enum stencil_border { STENCIL_CLAMP = 0, STENCIL_WRAP = 1, STENCIL_CONSTANT = 2 };

/* Customising functions (Table 2 names the paper's kernels; it does not print them).
 *   WEIGHTED_SUM: sum of w * V over the region - "gaussian" - in (dr, dc) row-major order.
 *                 F32: fp32 fma chain.  F64: fp64 fma chain (weights widened).  I32: 32-bit
 *                 wrap-around arithmetic; the weights must be integers.  F64 / I32 run with
 *                 the local-memory tile, cells per work-item (1,1), (1,2), (2,2), (4,2) / (1,1),
 *                 (1,4), (2,4), (4,4), and with regions 1/1/1/1 and 2/2/2/2 also DIRECT, cells_rows
 *                 in {1,2,4}, cells_cols = 2 / 4 (a 16-byte vector of the element type).
 *                 U8: a byte matrix in, an F32 matrix out (input and output types differ,
 *                 Section 3.3) - an 8-bit image blurred into floats; cells are converted
 *                 exactly, then the fp32 fma chain; the padding value is a byte.  Exactly one
 *                 application per stencil_run / sweep sample; local-memory tile only, cells
 *                 per work-item (1,1), (4,1), (1,4), (2,4), (4,4), (1,16) or (2,16).
 *   LIFE (u8):    Conway B3/S23 on cells 0/1, region 1/1/1/1 - "gol".  Precondition: every cell
 *                 is 0 or 1 (the kernels add packed bytes); a padding value above 1 is rejected.
 *   HEAT (f32):   u + alpha * (((n + s) + (e + w)) - 4u), region 1/1/1/1, every operation
 *                 rounded to fp32 in this order - "he".  scalars[0] = alpha.
 *   SINCOS (f32): sum over the region of w * sin(V) + cos(V) - a compute-intensive
 *                 synthetic stencil (Section 3.3).  sin/cos are evaluated in fp32.
 * The three stencils of the Canny edge detector (Section 5, Table 2: "sobel", "nms", "threshold";
 * the formulas are this library's, every operation rounded to fp32 in the order written):
 *   SOBEL (f32):  region 1/1/1/1; gx = ((ne - nw) + 2 (e - w)) + (se - sw),
 *                 gy = ((sw - nw) + 2 (s - n)) + (se - ne), out = sqrt(gx gx + gy gy).
 *   NMS (f32):    region 1/1/1/1; a cell keeps its value if it is no smaller than both its west
 *                 and east neighbours, or than both its north and south neighbours; else 0.
 *   THRESHOLD:    no border region (0/0/0/0); F32 matrix in, U8 matrix out (the kernel whose
 *                 output type differs from its input type, Section 3.3): 1 where the value is
 *                 >= scalars[0], else 0.  Exactly one application per stencil_run / sweep sample.
 */
enum stencil_kernel {
    STENCIL_WEIGHTED_SUM = 0,
    STENCIL_LIFE = 1,
    STENCIL_HEAT = 2,
    STENCIL_SINCOS = 3,
    STENCIL_SOBEL = 4,
    STENCIL_NMS = 5,
    STENCIL_THRESHOLD = 6
};

enum stencil_enum_mode {
    STENCIL_ENUM_POW2 = 0, /* w_r, w_c in {1,2,4,...}              */
    STENCIL_ENUM_EVEN = 1  /* w_r, w_c in {2,4,...,64} (Section 5) */
};

#define STENCIL_MAX_HALO 32            /* Table 2's border sizes go up to 30 */
/* The device's limits as far as they are known without asking it (an MI355X's).  The first call
 * that uses the GPU asks the device (work-items per workgroup, local memory, compute units) and,
 * per compiled kernel, the runtime (Section 3.1: W_max(s) depends on device and kernel); from then
 * on legality and f(s) use those answers. */
#define STENCIL_MAX_WG_SIZE 1024       /* work-items per workgroup */
#define STENCIL_LOCAL_MEM_BYTES 163840 /* local memory one workgroup may allocate (160 KiB) */

/* ---- scenario ---------------------------------------------------------------------- */

/* Section 2: the user defines size, type and border region of the matrix.  Creates a
 * handle (owned by the library, release with stencil_destroy); makes no GPU call.
 * rows, cols >= 1 and rows*cols < 2^31; halos in [0, STENCIL_MAX_HALO].  The customising
 * function defaults to WEIGHTED_SUM with all-zero weights until stencil_set_kernel. */
int stencil_create(stencil_t **out, int64_t rows, int64_t cols, int dtype,
                   int halo_n, int halo_s, int halo_e, int halo_w, int border_mode);

/* Frees the handle, its scratch matrix and its events.  NULL is accepted. */
void stencil_destroy(stencil_t *st);

/* Selects the customising function (Section 2).  `weights` (host, copied) must hold
 * (north+south+1)*(east+west+1) floats for WEIGHTED_SUM / SINCOS and is ignored otherwise;
 * `scalars` (host, copied): HEAT takes alpha.  LIFE and HEAT require region 1/1/1/1;
 * LIFE requires dtype U8, HEAT and SINCOS F32, WEIGHTED_SUM F32, F64 or I32. */
int stencil_set_kernel(stencil_t *st, int kernel_id, const float *weights, int n_weights,
                       const float *scalars, int n_scalars);

/* Padding value for STENCIL_CONSTANT (Section 2); default 0.  For a U8 matrix it must be an
 * integer in [0, 255] (0 or 1 for LIFE). */
int stencil_set_border_value(stencil_t *st, double value);

/* How elements map to work-items and where the window is staged.
 *   staging: STENCIL_STAGING_LOCAL  - the paper's scheme (Section 2): the workgroup's tile plus
 *            perimeter border region is staged in local memory, then every work-item reads
 *            its window from there.  Available for every scenario; the default.
 *            STENCIL_STAGING_DIRECT - nothing is staged: work-items read their windows from
 *            global memory as 16-byte vectors and rely on the L1/L2 caches for the overlap.
 *            Available for WEIGHTED_SUM with regions 1/1/1/1 and 2/2/2/2, HEAT, SOBEL, NMS and LIFE;
 *            needs no local memory, so no size is refused for its tile.
 *            STENCIL_STAGING_TEMPORAL - temporal blocking for iterated runs: one launch stages
 *            the tile plus a border region STENCIL_OPT_TEMPORAL_DEPTH cells deep in local
 *            memory and advances it by that many applications before writing it back, so a
 *            stencil_run of `iters` applications takes ceil(iters / depth) launches.
 *            Available for HEAT and WEIGHTED_SUM with region 1/1/1/1 (cells_cols = 4) and
 *            for LIFE (cells_cols = 16); cells_rows in {1,2,4,8}.
 *   cells_rows x cells_cols: block of adjacent cells one work-item computes (register
 *            blocking); a workgroup of w_r x w_c work-items covers (w_r*cells_rows) x
 *            (w_c*cells_cols) elements.  (1,1) is the paper's one element per work-item.
 *            LOCAL: cells_rows in {1,2,4,8}, cells_cols in {1,4} (F32) or {1,16} (U8); THRESHOLD:
 *            (1,1), (2,1), (1,4), (2,4), (4,4), and nothing is staged for want of a border region;
 *            DIRECT: cells_rows in {1,2,4} (LIFE also 8), cells_cols = 4 (F32) or 16 (U8).
 *            STENCIL_STAGING_STREAM - register streaming, no tile in local memory: each wavefront walks
 *            down a strip of 60 to 64 four-cell vectors (the outermost lanes at a side that has
 *            a border region only feed their neighbours), cells_rows (1..4096) rows at a time,
 *            taking row neighbours from adjacent lanes; cells_cols = 4.  Two kernels:
 *            HEAT and WEIGHTED_SUM with region 1/1/1/1, WRAP and CONSTANT borders: temporal
 *            blocking, the last three rows of every time level stay in registers,
 *            STENCIL_OPT_TEMPORAL_DEPTH applications per launch (up to
 *            STENCIL_MAX_STREAM_DEPTH; one rim lane per side up to 4, two beyond);
 *            SINCOS with region N1 S5 E3 W0 and WEIGHTED_SUM (F32), any border mode: one
 *            application per launch, each input row is loaded and pre-processed once and folded
 *            into the N+S+1 output rows it belongs to.  WEIGHTED_SUM regions 2/2/2/2 .. 5/5/5/5
 *            have kernels of their own; any other region with N, S <= 5 and E, W <= 4 runs a
 *            kernel compiled for its number of columns E+W+1 and for at most 5 (N, S <= 2) or 11
 *            rows, which hands row neighbours through local memory (a few KiB per workgroup,
 *            never a reason for refusal).  Larger regions: not available (the local-memory
 *            tile is as fast there: its fold is bound by arithmetic).
 *            The workgroup only groups wavefronts: w_r*w_c must be a multiple of 64 (other
 *            sizes are refused) and at most 256.  Not available for a matrix whose rows are 4 GiB
 *            or longer (cells within a row are addressed by 32-bit byte offsets).
 * Output values never depend on the mapping.  Heavily blocked variants have a lower per-kernel
 * W_max (Section 3.1), see stencil_max_wg_size. */
enum stencil_staging {
    STENCIL_STAGING_LOCAL = 0,
    STENCIL_STAGING_DIRECT = 1,
    STENCIL_STAGING_TEMPORAL = 2,
    STENCIL_STAGING_STREAM = 3
};
int stencil_set_mapping(stencil_t *st, int staging, int cells_rows, int cells_cols);

/* Element type (enum stencil_dtype) of the matrix `out` must be: the scenario's own, except
 * STENCIL_U8 once STENCIL_THRESHOLD is selected and STENCIL_F32 for STENCIL_WEIGHTED_SUM on a
 * U8 matrix.  `out` always holds rows*cols elements of it. */
int stencil_output_dtype(const stencil_t *st);
int stencil_get_mapping(const stencil_t *st, int *staging, int *cells_rows, int *cells_cols);

/* Segment heights worth trying under STENCIL_STAGING_STREAM.  There a wavefront is the unit of work
 * (one strip of columns x cells_rows rows), a SIMD holds a few of them at a time, and a launch is
 * fastest when its wavefronts fill a whole number of such slots on every SIMD: one wavefront more
 * and a last, nearly empty round is added.  For a scenario already on the mapping this returns in
 * *cells_rows the smallest height at which strips x segments <= 4 x compute units x
 * wavefronts_per_simd (the compute units: the device's, 256 until a GPU has been used); taller
 * segments repeat fewer run-in rows, shorter ones hide more latency - 2 to 6 per SIMD are the
 * values to sweep (stencil_sweep_configs).  STENCIL_E_INVALID on another mapping,
 * STENCIL_E_REFUSED if the height would exceed the kernels' 4096. */
int stencil_stream_segment_rows(const stencil_t *st, int wavefronts_per_simd, int *cells_rows);

/* Launch options.  STENCIL_OPT_XCD_REMAP (default 1): workgroups are numbered so that each of
 * the eight XCDs (each with its own L2) works on one contiguous band of tiles.
 * STENCIL_OPT_TEMPORAL_DEPTH (default 2): applications fused into one launch, 1..
 * STENCIL_MAX_TEMPORAL_DEPTH under STENCIL_STAGING_TEMPORAL, 1..STENCIL_MAX_STREAM_DEPTH under
 * STENCIL_STAGING_STREAM (a depth above 4 makes every size illegal under the former).
 * STENCIL_OPT_SWEEP_CUTOFF (default 0 = off; otherwise a percentage >= 100): adaptive sampling
 * for stencil_sweep_wg, after the paper's closing remarks on minimising the observations needed
 * to tell bad sizes from good ones: every size first gets one warm-up and two samples; only the
 * sizes whose two-sample mean is within cutoff/100 times the best one are then sampled in full
 * (3 warm-ups + `reps` samples); the others keep their two-sample statistics.
 * STENCIL_OPT_NT_STORE (default 0): the kernels' 16-byte stores of output cells are issued as
 * non-temporal stores (the output is not read again by the launch that writes it); narrower
 * stores (unaligned rows, one cell per work-item, the threshold stencil) stay plain.  Same
 * results, different cache behaviour: it pays on matrices beyond the caches and costs where
 * the next application would have found its input in a cache.
 * STENCIL_OPT_FAIL_LAUNCH (default 0 = off) is a testing aid for the handling of refused parameters
 * that only show when a launch fails (Section 3.1): with value (w_r << 16) | w_c every launch with
 * that workgroup size - with -1 every launch - is not made and reports the runtime's
 * out-of-resources error instead, which stencil_run returns as STENCIL_E_REFUSED and the sweeps
 * record as a refused size. */
#define STENCIL_MAX_TEMPORAL_DEPTH 4   /* STENCIL_STAGING_TEMPORAL */
#define STENCIL_MAX_STREAM_DEPTH 8     /* STENCIL_STAGING_STREAM */
enum stencil_option { STENCIL_OPT_XCD_REMAP = 0, STENCIL_OPT_TEMPORAL_DEPTH = 1, STENCIL_OPT_SWEEP_CUTOFF = 2,
                      STENCIL_OPT_NT_STORE = 3, STENCIL_OPT_FAIL_LAUNCH = 4 };
int stencil_set_option(stencil_t *st, int option, int value);

/* ---- legality (Section 3.1) ---------------------------------------------------------- */

/* W_max(s): the largest number of work-items a workgroup of this scenario may have. */
int stencil_max_wg_size(const stencil_t *st);

/* Bytes of local memory the tile of Section 2 (workgroup plus perimeter border region)
 * needs for this scenario and workgroup size, as laid out by the kernels. */
int64_t stencil_tile_bytes(const stencil_t *st, int wg_rows, int wg_cols);

/* Eq. 1: 1 if (wg_rows, wg_cols) is legal for this scenario (w_r*w_c <= W_max(s) and not a
 * refused parameter, i.e. its tile fits local memory), else 0.  What can be decided before a
 * launch; a size may still be refused by the launch itself (stencil_run then returns
 * STENCIL_E_REFUSED with the runtime's text, the sweeps record the size as refused and go on). */
int stencil_is_legal(const stencil_t *st, int wg_rows, int wg_cols);

/* Section 5's enumeration.  Writes up to `cap` pairs to rows[]/cols[] (may be NULL when
 * cap = 0) in row-major order of (w_r, w_c) and returns the total number of pairs with
 * w_r*w_c <= max_threads (or a negative status). */
int stencil_enumerate_wg(int mode, int max_threads, int *rows, int *cols, int cap);

/* ---- execution ------------------------------------------------------------------------ */

/* Applies the stencil `iters` times (out-of-place steps; the input of step k+1 is the
 * output of step k) with workgroups of wg_rows x wg_cols work-items.  `in` and `out` are
 * device buffers of rows*cols elements, contiguous row-major, non-overlapping; `in` is
 * never written; the final matrix is always in `out`; iters = 0 copies.  A scratch matrix
 * for the intermediate steps is allocated by the first run that takes more than one launch
 * and kept until destroy.  Asynchronous on `stream` (a hipStream_t; NULL = default stream),
 * no host synchronisation: the weight table of a run-time region travels to the device in small
 * launches ordered on `stream` ahead of the stencil's, and a table that stencil_set_kernel
 * replaced goes into the other of two device tables, so launches already queued keep theirs
 * (with launches of more than one earlier table still in flight on other streams, order them
 * yourself).  Calls that allocate nothing (a second run of the same
 * kind on the same handle) can be captured into a HIP graph; make that first run outside
 * the capture.
 * wg_rows = wg_cols = 0 lets the library choose (Section 2: selecting the size is the
 * implementation's responsibility): the best size of the handle's last sweep; else the
 * prediction of the classifier given to stencil_attach_predictor (Algorithm 1 over the
 * power-of-two sizes); else a built-in default.  Illegal sizes return STENCIL_E_REFUSED without
 * launching; so does a size that the runtime refuses at launch. */
int stencil_run(stencil_t *st, const void *in, void *out, int iters,
                int wg_rows, int wg_cols, void *stream);

/* stencil_run for callers that cannot allocate device memory - code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: the same kernels, but the device memory a run
 * needs beyond `in` and `out` (the weight table of a run-time border region; the matrix that a run
 * of more than one launch ping-pongs through) lies in one fixed buffer that is part of the
 * library's code object, STENCIL_STATIC_MATRIX_BYTES (+ 32 KiB for the table) per GPU, held from
 * the library's load until the process ends.  Calls no hipMalloc / hipFree and no allocating
 * routine; the first call on a device looks up the buffer's address (make it outside a capture).
 * STENCIL_E_INVALID, with nothing launched, if the run needs more than the buffer holds: a
 * matrix above STENCIL_STATIC_MATRIX_BYTES with more than one launch (one launch never needs
 * the matrix), or a weight table above 8192 entries.  Everything else as for stencil_run
 * (arguments, legality, asynchronous on `stream`); the handle's own scratch matrix and tables are
 * neither used nor created.  All handles and all calls on one GPU share the buffer, which keeps
 * the last call's contents: each call uploads its table and overwrites the matrix before reading
 * it, and calls that overlap on one GPU (different streams or threads) race - serialise them. */
#define STENCIL_STATIC_MATRIX_BYTES (16 << 20)
int stencil_run_static(stencil_t *st, const void *in, void *out, int iters,
                       int wg_rows, int wg_cols, void *stream);

/* Matrix pairs for the sweeps to go round.  A sweep's sample is otherwise a chain of `iters`
 * applications on the caller's one pair (in -> out), and on a device with a large last-level cache
 * every sample then finds in it what the sample before read or wrote: on MI355X (256 MB, on the
 * memory side) a single application to a 256 MiB matrix runs up to 25 % faster on a pair it has just
 * been applied to than on matrices fresh from HBM, and the size that wins is not always the same.
 * With n >= 1 pairs set, a sample of stencil_sweep_wg / stencil_sweep_configs is `iters` independent
 * single applications, ins[k] -> outs[k], on the pairs in turn (the sweeps' own in / out arguments
 * are still validated, and still receive nothing they would not have received).  Device pointers,
 * each a whole matrix of the scenario's input / output type, kept by reference: they must stay
 * valid until the rotation is replaced or cleared (n = 0) or the handle destroyed; no output may
 * overlap any other matrix of the rotation (inputs may be shared).  Enough pairs that their total
 * size is a few times the cache make every application a cold one.  STENCIL_E_INVALID on a bad
 * pointer, an overlap, or n outside 0..STENCIL_MAX_ROTATION. */
#define STENCIL_MAX_ROTATION 64
int stencil_set_sweep_rotation(stencil_t *st, const void *const *ins, void *const *outs, int n);

/* Section 5's measurement: for each of the n sizes, 3 untimed runs and then `reps` timed
 * samples (reps <= 0 means 30), each sample one stencil_run(iters) bracketed by events on
 * `stream`.  Outputs (host arrays of n, each may be NULL): mean / min / median / sample
 * standard deviation in milliseconds per sample, and status (STENCIL_OK or
 * STENCIL_E_REFUSED; refused sizes get NaN times and the sweep continues, Section 4.2).
 * best_index = argmin of the mean over legal sizes (Eq. 3; ties: fewer work-items, then
 * smaller w_r), -1 if none.  speedup_over_fixed = mean(fixed) / mean(best) (Section 7's
 * speedup metric; the fixed size is timed additionally if it is not in the list; NaN if it
 * is refused); pass fixed_rows = 0 to skip.  Synchronous: returns after the last sample.
 * Remembers the best size for stencil_run(0, 0). */
int stencil_sweep_wg(stencil_t *st, const void *in, void *out, int iters,
                     const int *wg_rows_list, const int *wg_cols_list, int n,
                     int fixed_rows, int fixed_cols, int reps,
                     double *mean_ms, double *min_ms, double *median_ms, double *stddev_ms,
                     int *status, int *best_index, double *speedup_over_fixed, void *stream);

/* The sweep over more than the workgroup size (the paper's closing section names further
 * optimisation parameters as the next step): each configuration fixes the mapping
 * (stencil_set_mapping's three arguments), the number of applications fused per launch (depth; 0
 * keeps the current STENCIL_OPT_TEMPORAL_DEPTH), the numbering of workgroups (xcd_remap; -1 keeps
 * the current STENCIL_OPT_XCD_REMAP), the kind of output stores (nt_store; -1 keeps the current
 * STENCIL_OPT_NT_STORE) and a workgroup size, and is timed by
 * stencil_sweep_wg's protocol.  mean_ms[k] = mean milliseconds per sample (`iters` applications),
 * NaN unless status[k] == STENCIL_OK; status[k] = STENCIL_E_INVALID for a mapping or depth the
 * scenario does not offer, STENCIL_E_REFUSED for an illegal workgroup size; best_index (may be
 * NULL) = fastest configuration or -1.  Afterwards the scenario is left on the fastest
 * configuration (mapping, depth, numbering, stores, and its size for stencil_run(0, 0)); on error, or if none ran, on
 * the one it had.  configs, mean_ms, status: host arrays of n.  Synchronous. */
typedef struct stencil_config {
    int staging, cells_rows, cells_cols;   /* as for stencil_set_mapping */
    int depth;                             /* applications per launch, 0 = leave as is */
    int xcd_remap;                         /* STENCIL_OPT_XCD_REMAP: 0 or 1, -1 = leave as is */
    int nt_store;                          /* STENCIL_OPT_NT_STORE: 0 or 1, -1 = leave as is */
    int wg_rows, wg_cols;
} stencil_config_t;
int stencil_sweep_configs(stencil_t *st, const void *in, void *out, int iters,
                          const stencil_config_t *configs, int n, int reps,
                          double *mean_ms, int *status, int *best_index, void *stream);

/* Reference for the bandwidth a stencil can hope for: a plain device-to-device copy kernel
 * (one 16-byte vector per work-item) of `bytes` bytes from `in` to `out` (device pointers,
 * 16-byte aligned, non-overlapping), asynchronous on `stream`.  Not part of the paper's
 * method; used to express achieved bandwidth relative to a copy and to calibrate hardware
 * traffic counters against a kernel of known size. */
int stencil_device_copy(const void *in, void *out, int64_t bytes, void *stream);

/* The same copy timed by the sweep's protocol (Section 5: warm-up, then `reps` samples by
 * events on `stream`, a sample being `burst` launches back to back): mean_ms and, if not NULL,
 * min_ms (host pointers) receive milliseconds per launch.  Synchronous.  burst, reps >= 1. */
int stencil_time_copy(const void *in, void *out, int64_t bytes, int burst, int reps, double *mean_ms,
                      double *min_ms, void *stream);

/* The reductions of a sweep on their own (Eq. 3; Section 7's performance and speedup), on
 * host arrays: best_index as above; performance[i] = mean_ms[best] / mean_ms[i] (NaN where
 * status[i] != STENCIL_OK; may be NULL); speedup = fixed_ms / mean_ms[best]. */
int stencil_sweep_reduce(const int *wg_rows_list, const int *wg_cols_list, int n,
                         const double *mean_ms, const int *status, double fixed_ms,
                         int *best_index, double *performance, double *speedup_over_fixed);

/* Algorithm 1's Baseline handler (also the "best fixed workgroup size" the paper's speedups
 * are quoted against): `performance` is n_scenarios x n_sizes, row-major, p(s, w) as returned by
 * stencil_sweep_reduce with NaN where w is not legal for s.  best_index = the size that is legal
 * for every scenario (W_safe, Eq. 2) with the highest geometric mean of p, or -1 if none is. */
int stencil_baseline_wg(const double *performance, int n_scenarios, int n_sizes, int *best_index);

/* ---- prediction (Section 3.2, Section 4.1, Algorithm 1) ---------------------------------- */

#define STENCIL_N_FEATURES 16

/* f(s): dataset, kernel and device features of the scenario, STENCIL_N_FEATURES doubles:
 * rows, cols, input element bytes, north, south, east, west, region cells, compute-intensive
 * flag, compute units, local memory bytes, max workgroup size, output element bytes
 * (Section 3.2: "the input and output data types"), operations per cell that the customising
 * function states (arithmetic and comparisons; the paper counts compiled instructions, these are
 * filled in by hand per kernel), those of them on the transcendental unit, border mode.  The
 * three device features are the constants above until a GPU has been used, the device's own
 * answers after. */
int stencil_features(const stencil_t *st, double *features);

/* A classifier over (f(s), Omega(s)) pairs (Section 4.1's D_training):
 *   STENCIL_CLASSIFIER_NEAREST - label of the nearest training scenario; each feature is scaled
 *       by its range over the training set, Euclidean distance, first nearest wins ties;
 *   STENCIL_CLASSIFIER_TREE    - decision tree (the paper's J48 is the fastest of its
 *       classifiers): binary splits `feature <= threshold` by information gain over the
 *       midpoints between consecutive distinct values (features in order, thresholds ascending,
 *       first best wins), grown until pure; a leaf answers with its most frequent label;
 *   STENCIL_CLASSIFIER_ZEROR   - always the most frequent label (the paper's dummy classifier). */
enum stencil_classifier { STENCIL_CLASSIFIER_NEAREST = 0, STENCIL_CLASSIFIER_TREE = 1, STENCIL_CLASSIFIER_ZEROR = 2 };
int stencil_predictor_create(stencil_predictor_t **out, int classifier);
void stencil_predictor_destroy(stencil_predictor_t *p);
int stencil_predictor_add(stencil_predictor_t *p, const double *features, int n_features,
                          int wg_rows, int wg_cols);
/* classify(f(s)) with the classifier chosen at creation (a tree is grown on first use after
 * the last added pair). */
int stencil_predictor_classify(const stencil_predictor_t *p, const double *features,
                               int n_features, int *wg_rows, int *wg_cols);

/* Algorithm 1: classify the scenario; a legal size is returned as classified, otherwise the
 * fallback handler chooses among the candidates (cand_rows/cand_cols, n_cand entries) that are
 * legal for the scenario:
 *   STENCIL_FALLBACK_NEAREST  - the one closest to the prediction in Euclidean distance (first
 *                               wins ties);
 *   STENCIL_FALLBACK_BASELINE - (baseline_rows, baseline_cols), e.g. from stencil_baseline_wg;
 *   STENCIL_FALLBACK_RANDOM   - the (random mod count)-th legal candidate in list order; the
 *                               caller supplies the random number.
 * STENCIL_E_REFUSED if the handler has nothing legal to offer. */
enum stencil_fallback { STENCIL_FALLBACK_NEAREST = 0, STENCIL_FALLBACK_BASELINE = 1, STENCIL_FALLBACK_RANDOM = 2 };
int stencil_predict_wg(const stencil_t *st, const stencil_predictor_t *p,
                       const int *cand_rows, const int *cand_cols, int n_cand,
                       int handler, int baseline_rows, int baseline_cols, uint64_t random,
                       int *wg_rows, int *wg_cols);

/* The classifier stencil_run(st, ..., 0, 0, ...) consults when the handle has no sweep to go by:
 * Algorithm 1 with `handler` over the power-of-two sizes (STENCIL_FALLBACK_BASELINE falls back to
 * the built-in default size).  The predictor stays the caller's and must outlive its use;
 * NULL detaches. */
int stencil_attach_predictor(stencil_t *st, const stencil_predictor_t *p, int handler);

/* The size stencil_run(st, ..., 0, 0, ...) would use now: the last sweep's best, else the attached
 * classifier's prediction repaired by its handler, else the built-in default.  No GPU call. */
int stencil_default_wg(const stencil_t *st, int *wg_rows, int *wg_cols);

/* A classifier from a text file of training pairs (Section 4.1: collected offline, used at run
 * time): '#' starts a comment line; the first other line reads "features <n>"; every further line
 * holds n feature values, then w_r and w_c, separated by blanks.  The files under
 * paper_1511_02490_amd/tuning_data/ (written by autotune_study --export-training) are of this form.
 * STENCIL_E_INVALID if the file cannot be read or a line does not parse. */
int stencil_predictor_load(stencil_predictor_t **out, const char *path, int classifier);

/* ---- prediction with regressors (Sections 4.2 and 4.3, Algorithm 2) -------------------------- */

/* R(f(s), w): a regressor over (f(s), w, y) tuples, y a runtime (Section 4.2) or the speedup of
 * w over a baseline size (Section 4.3).  Nearest-neighbour regression: the prediction for (f, w)
 * is the y of the tuple with the same w whose scenario is nearest to f (features scaled by their
 * range over all tuples, Euclidean distance, first nearest wins ties); NaN if no tuple has w. */
int stencil_regressor_create(stencil_regressor_t **out);
void stencil_regressor_destroy(stencil_regressor_t *r);
int stencil_regressor_add(stencil_regressor_t *r, const double *features, int n_features,
                          int wg_rows, int wg_cols, double value);
int stencil_regressor_predict(const stencil_regressor_t *r, const double *features, int n_features,
                              int wg_rows, int wg_cols, double *value);

/* Section 5's regressor: a random forest of regression trees over the tuples added so far.
 * Inputs of the trees: the features, then w_r, then w_c (n_features + 2 of them).  Tree t is a
 * CART regression tree (cuts minimise the summed squared error of the two sides' means, thresholds
 * midway between consecutive distinct values, at least min_leaf tuples a side, at most max_depth
 * levels) grown on the tuples bootstrap[t*n_rows .. (t+1)*n_rows) (indices into the order of
 * stencil_regressor_add, repetition allowed; NULL: all tuples once) using only the inputs j with
 * masks[t*(n_features+2) + j] != 0 (NULL: all).  The random draws are thus the caller's (host
 * arrays, not kept).  Afterwards stencil_regressor_predict returns the mean of the trees'
 * predictions; adding a tuple discards the forest.  STENCIL_E_INVALID on an index out of range, a
 * tree with no open input, or no tuples. */
int stencil_regressor_fit_forest(stencil_regressor_t *r, int n_trees, int n_rows, const int *bootstrap,
                                 const unsigned char *masks, int min_leaf, int max_depth);

/* Algorithm 2: among the candidates within W_max(s) that the regressor can price, take the one
 * with the highest fitness of the prediction - STENCIL_FITNESS_RECIPROCAL (1/x, for predicted
 * runtimes) or STENCIL_FITNESS_IDENTITY (for predicted speedups); if it turns out to be a refused
 * parameter, strike it from the pool and take the next.  n_refused (may be NULL) = how many were
 * struck.  STENCIL_E_REFUSED if the pool runs dry. */
enum stencil_fitness { STENCIL_FITNESS_RECIPROCAL = 0, STENCIL_FITNESS_IDENTITY = 1 };
int stencil_predict_wg_regression(const stencil_t *st, const stencil_regressor_t *r,
                                  const int *cand_rows, const int *cand_cols, int n_cand, int fitness,
                                  int *wg_rows, int *wg_cols, int *n_refused);

/* Text of the calling thread's most recent error ("" if none). */
const char *stencil_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LIBSTENCIL_H */
