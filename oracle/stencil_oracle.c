/*
 * CPU oracle for the 2D stencil skeleton.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, direct transcription of what the stencil pattern computes
 * (Section 2 of the paper): every output cell is a user function of the input
 * cell and a rectangular border region of `north`, `south`, `east`, `west` cells
 * around it; neighbours that fall outside the matrix are substituted, either by
 * a padding constant or by the nearest in-matrix cell.  A third substitution,
 * periodic wrap, is added for the cellular / diffusion workloads.
 *
 * No tiling, no local memory, no workgroups: the premise of the paper's
 * gold-standard check (Section 5) is that the workgroup size never changes the
 * values, so the oracle is the definition itself.
 *
 * Conventions (the figure that would fix them is not reproduced in the text):
 *   row-major a[r][c]; north = smaller r, south = larger r, west = smaller c,
 *   east = larger c; the region includes the centre cell; weight tables are
 *   (north+south+1) x (east+west+1), row-major, applied as a correlation:
 *   out[r][c] = sum_{dr=-north..south} sum_{dc=-west..east} w[dr+north][dc+west] * V(r+dr, c+dc).
 *
 * Shares no code with the GPU library.  OpenMP splits rows across threads
 * (each output cell is independent within one application); nothing else is
 * tuned.  Compile with -ffp-contract=off so that the fp32 heat step rounds after
 * every operation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_CLAMP = 0, ORACLE_WRAP = 1, ORACLE_CONSTANT = 2 };

static void set_threads(int threads)
{
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Index substitution for one axis (Section 2: nearest cell within the matrix;
 * wrap is this build's addition).  Returns -1 for "use the padding value". */
static inline int64_t resolve(int64_t i, int64_t n, int border)
{
    if (i >= 0 && i < n) return i;
    if (border == ORACLE_CLAMP) return i < 0 ? 0 : n - 1;
    if (border == ORACLE_WRAP) {
        int64_t m = i % n;
        return m < 0 ? m + n : m;
    }
    return -1;
}

/* V(i,j): the value a work-item sees at matrix position (i,j). */
static inline float V_f32(const float *a, int64_t rows, int64_t cols, int64_t i, int64_t j,
                          int border, float pad)
{
    int64_t ri = resolve(i, rows, border), cj = resolve(j, cols, border);
    if (ri < 0 || cj < 0) return pad;
    return a[ri * cols + cj];
}

static inline uint8_t V_u8(const uint8_t *a, int64_t rows, int64_t cols, int64_t i, int64_t j,
                           int border, uint8_t pad)
{
    int64_t ri = resolve(i, rows, border), cj = resolve(j, cols, border);
    if (ri < 0 || cj < 0) return pad;
    return a[ri * cols + cj];
}

static inline double V_f64(const double *a, int64_t rows, int64_t cols, int64_t i, int64_t j,
                           int border, double pad)
{
    int64_t ri = resolve(i, rows, border), cj = resolve(j, cols, border);
    if (ri < 0 || cj < 0) return pad;
    return a[ri * cols + cj];
}

static inline int32_t V_i32(const int32_t *a, int64_t rows, int64_t cols, int64_t i, int64_t j,
                            int border, int32_t pad)
{
    int64_t ri = resolve(i, rows, border), cj = resolve(j, cols, border);
    if (ri < 0 || cj < 0) return pad;
    return a[ri * cols + cj];
}

/* ---- one application of each customising function --------------------------------- */

/* Weighted sum (Gaussian blur and any linear stencil): fp64 accumulation over the fp32
 * inputs in (dr, dc) row-major order, rounded once to fp32. */
static void step_weighted_sum(const float *in, float *out, int64_t rows, int64_t cols,
                              int N, int S, int E, int W, int border, float pad, const float *w)
{
    const int ww = E + W + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            double acc = 0.0;
            for (int dr = -N; dr <= S; ++dr)
                for (int dc = -W; dc <= E; ++dc)
                    acc += (double)w[(dr + N) * ww + (dc + W)] *
                           (double)V_f32(in, rows, cols, r + dr, c + dc, border, pad);
            out[r * cols + c] = (float)acc;
        }
}

/* The weighted sum with different input and output element types (Section 3.3 lists both among
 * a kernel's features): a byte matrix in, a float matrix out - an 8-bit image blurred into floats,
 * the first stage of the Canny detector.  The padding value is a byte like any other cell; fp64
 * accumulation in (dr, dc) row-major order, rounded once to fp32. */
static void step_weighted_sum_u8_f32(const uint8_t *in, float *out, int64_t rows, int64_t cols,
                                     int N, int S, int E, int W, int border, uint8_t pad, const float *w)
{
    const int ww = E + W + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            double acc = 0.0;
            for (int dr = -N; dr <= S; ++dr)
                for (int dc = -W; dc <= E; ++dc)
                    acc += (double)w[(dr + N) * ww + (dc + W)] *
                           (double)V_u8(in, rows, cols, r + dr, c + dc, border, pad);
            out[r * cols + c] = (float)acc;
        }
}

/* The weighted sum on the other element types of the paper's template (Section 3.3).
 * double: accumulated in long double, rounded once.  int32: exact integer arithmetic reduced
 * modulo 2^32 (the weights hold integers). */
static void step_weighted_sum_f64(const double *in, double *out, int64_t rows, int64_t cols,
                                  int N, int S, int E, int W, int border, double pad, const float *w)
{
    const int ww = E + W + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            long double acc = 0.0L;
            for (int dr = -N; dr <= S; ++dr)
                for (int dc = -W; dc <= E; ++dc)
                    acc += (long double)w[(dr + N) * ww + (dc + W)] *
                           (long double)V_f64(in, rows, cols, r + dr, c + dc, border, pad);
            out[r * cols + c] = (double)acc;
        }
}

static void step_weighted_sum_i32(const int32_t *in, int32_t *out, int64_t rows, int64_t cols,
                                  int N, int S, int E, int W, int border, int32_t pad, const float *w)
{
    const int ww = E + W + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            uint64_t acc = 0;   /* two's complement, modulo 2^64 and in the end 2^32 */
            for (int dr = -N; dr <= S; ++dr)
                for (int dc = -W; dc <= E; ++dc)
                    acc += (uint64_t)(int64_t)w[(dr + N) * ww + (dc + W)] *
                           (uint64_t)(int64_t)V_i32(in, rows, cols, r + dr, c + dc, border, pad);
            out[r * cols + c] = (int32_t)(uint32_t)acc;
        }
}

/* Conway's Game of Life, B3/S23, on the region's cells other than the centre.
 * Cells hold 0 or 1.  With the 1/1/1/1 border region this is the 8-neighbourhood. */
static void step_life(const uint8_t *in, uint8_t *out, int64_t rows, int64_t cols,
                      int N, int S, int E, int W, int border, uint8_t pad)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int n = 0;
            for (int dr = -N; dr <= S; ++dr)
                for (int dc = -W; dc <= E; ++dc)
                    if (dr != 0 || dc != 0) n += V_u8(in, rows, cols, r + dr, c + dc, border, pad);
            uint8_t self = in[r * cols + c];
            out[r * cols + c] = (uint8_t)((n == 3) || (self && n == 2));
        }
}

/* Heat equation, explicit 5-point Jacobi step u' = u + alpha (N + S + E + W - 4u),
 * in strict fp32: every operation below rounds to fp32, in this order. */
static void step_heat_f32(const float *in, float *out, int64_t rows, int64_t cols,
                          int border, float pad, float alpha)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            float u = in[r * cols + c];
            float n = V_f32(in, rows, cols, r - 1, c, border, pad);
            float s = V_f32(in, rows, cols, r + 1, c, border, pad);
            float e = V_f32(in, rows, cols, r, c + 1, border, pad);
            float w = V_f32(in, rows, cols, r, c - 1, border, pad);
            float ns = n + s;
            float ew = e + w;
            float sum = ns + ew;
            float four_u = 4.0f * u;
            float t = sum - four_u;
            float at = alpha * t;
            out[r * cols + c] = u + at;
        }
}

/* The three stencils of the Canny edge detector that Table 2 lists (sobel, nms, threshold).
 * The paper names them and gives their border regions (1/1/1/1, 1/1/1/1, none) but not their
 * formulas; these are this build's, each operation rounded to fp32 in the order written.
 *
 * sobel: gradient magnitude of the 3x3 Sobel operator,
 *   gx = ((ne - nw) + 2 (e - w)) + (se - sw),  gy = ((sw - nw) + 2 (s - n)) + (se - ne),
 *   out = sqrt(gx gx + gy gy). */
static void step_sobel_f32(const float *in, float *out, int64_t rows, int64_t cols, int border, float pad)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            float nw = V_f32(in, rows, cols, r - 1, c - 1, border, pad);
            float n = V_f32(in, rows, cols, r - 1, c, border, pad);
            float ne = V_f32(in, rows, cols, r - 1, c + 1, border, pad);
            float w = V_f32(in, rows, cols, r, c - 1, border, pad);
            float e = V_f32(in, rows, cols, r, c + 1, border, pad);
            float sw = V_f32(in, rows, cols, r + 1, c - 1, border, pad);
            float s = V_f32(in, rows, cols, r + 1, c, border, pad);
            float se = V_f32(in, rows, cols, r + 1, c + 1, border, pad);
            float a = ne - nw, b = e - w, d = se - sw;
            float two_b = 2.0f * b;
            float ab = a + two_b;
            float gx = ab + d;
            float f = sw - nw, g = s - n, h = se - ne;
            float two_g = 2.0f * g;
            float fg = f + two_g;
            float gy = fg + h;
            float xx = gx * gx, yy = gy * gy;
            float sum = xx + yy;
            out[r * cols + c] = sqrtf(sum);
        }
}

/* nms: non-maximum suppression along the two axes - a cell keeps its value if it is no smaller
 * than both its west and east neighbours, or no smaller than both its north and south neighbours;
 * otherwise it becomes 0. */
static void step_nms_f32(const float *in, float *out, int64_t rows, int64_t cols, int border, float pad)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            float u = in[r * cols + c];
            float n = V_f32(in, rows, cols, r - 1, c, border, pad);
            float s = V_f32(in, rows, cols, r + 1, c, border, pad);
            float e = V_f32(in, rows, cols, r, c + 1, border, pad);
            float w = V_f32(in, rows, cols, r, c - 1, border, pad);
            int keep = (u >= w && u >= e) || (u >= n && u >= s);
            out[r * cols + c] = keep ? u : 0.0f;
        }
}

/* threshold: no border region; a float matrix in, a byte matrix out: 1 where the value reaches
 * the threshold, else 0 (a NaN reaches nothing). */
static void step_threshold_f32_u8(const float *in, uint8_t *out, int64_t rows, int64_t cols, float level)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) out[r * cols + c] = in[r * cols + c] >= level ? 1 : 0;
}

/* The same step carried in fp64 (state included): used to attribute rounding error and
 * to check conservation, never as the parity reference. */
static void step_heat_f64(const double *in, double *out, int64_t rows, int64_t cols,
                          int border, double pad, double alpha)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            double nb[4];
            const int64_t rr[4] = { r - 1, r + 1, r, r }, cc[4] = { c, c, c + 1, c - 1 };
            for (int k = 0; k < 4; ++k) {
                int64_t ri = resolve(rr[k], rows, border), cj = resolve(cc[k], cols, border);
                nb[k] = (ri < 0 || cj < 0) ? pad : in[ri * cols + cj];
            }
            double u = in[r * cols + c];
            out[r * cols + c] = u + alpha * (((nb[0] + nb[1]) + (nb[2] + nb[3])) - 4.0 * u);
        }
}

/* Compute-intensive synthetic stencil: every cell of the region (centre included)
 * contributes w * sin(x) + cos(x).  The padding value is substituted for x before the
 * function is applied.  sin/cos from libm in fp64, fp64 sum, one rounding to fp32. */
static void step_sincos(const float *in, float *out, int64_t rows, int64_t cols,
                        int N, int S, int E, int W, int border, float pad, const float *w)
{
    const int ww = E + W + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            double acc = 0.0;
            for (int dr = -N; dr <= S; ++dr)
                for (int dc = -W; dc <= E; ++dc) {
                    double x = (double)V_f32(in, rows, cols, r + dr, c + dc, border, pad);
                    acc += (double)w[(dr + N) * ww + (dc + W)] * sin(x) + cos(x);
                }
            out[r * cols + c] = (float)acc;
        }
}

/* ---- iterated drivers: out-of-place (Jacobi) steps, buffers swapped after each ------- */

#define ITERATE(T, STEP_CALL)                                                            \
    size_t bytes = (size_t)rows * (size_t)cols * sizeof(T);                              \
    if (iters <= 0) { memcpy(out, in, bytes); return 0; }                                \
    T *a = (T *)malloc(bytes), *b = (T *)malloc(bytes);                                  \
    if (!a || !b) { free(a); free(b); return -1; }                                       \
    memcpy(a, in, bytes);                                                                \
    for (int it = 0; it < iters; ++it) {                                                 \
        const T *src = a; T *dst = b;                                                    \
        STEP_CALL;                                                                       \
        T *tmp = a; a = b; b = tmp;                                                      \
    }                                                                                    \
    memcpy(out, a, bytes);                                                               \
    free(a); free(b);                                                                    \
    return 0;

int oracle_weighted_sum_f32(const float *in, float *out, int64_t rows, int64_t cols,
                            int N, int S, int E, int W, int border, float pad,
                            const float *w, int iters, int threads)
{
    set_threads(threads);
    ITERATE(float, step_weighted_sum(src, dst, rows, cols, N, S, E, W, border, pad, w))
}

int oracle_weighted_sum_f64(const double *in, double *out, int64_t rows, int64_t cols,
                            int N, int S, int E, int W, int border, double pad,
                            const float *w, int iters, int threads)
{
    set_threads(threads);
    ITERATE(double, step_weighted_sum_f64(src, dst, rows, cols, N, S, E, W, border, pad, w))
}

int oracle_weighted_sum_i32(const int32_t *in, int32_t *out, int64_t rows, int64_t cols,
                            int N, int S, int E, int W, int border, int32_t pad,
                            const float *w, int iters, int threads)
{
    set_threads(threads);
    ITERATE(int32_t, step_weighted_sum_i32(src, dst, rows, cols, N, S, E, W, border, pad, w))
}

int oracle_life_u8(const uint8_t *in, uint8_t *out, int64_t rows, int64_t cols,
                   int N, int S, int E, int W, int border, uint8_t pad, int iters, int threads)
{
    set_threads(threads);
    ITERATE(uint8_t, step_life(src, dst, rows, cols, N, S, E, W, border, pad))
}

int oracle_heat_f32(const float *in, float *out, int64_t rows, int64_t cols,
                    int border, float pad, float alpha, int iters, int threads)
{
    set_threads(threads);
    ITERATE(float, step_heat_f32(src, dst, rows, cols, border, pad, alpha))
}

int oracle_heat_f64(const double *in, double *out, int64_t rows, int64_t cols,
                    int border, double pad, double alpha, int iters, int threads)
{
    set_threads(threads);
    ITERATE(double, step_heat_f64(src, dst, rows, cols, border, pad, alpha))
}

int oracle_sincos_f32(const float *in, float *out, int64_t rows, int64_t cols,
                      int N, int S, int E, int W, int border, float pad,
                      const float *w, int iters, int threads)
{
    set_threads(threads);
    ITERATE(float, step_sincos(src, dst, rows, cols, N, S, E, W, border, pad, w))
}

int oracle_sobel_f32(const float *in, float *out, int64_t rows, int64_t cols, int border, float pad,
                     int iters, int threads)
{
    set_threads(threads);
    ITERATE(float, step_sobel_f32(src, dst, rows, cols, border, pad))
}

int oracle_nms_f32(const float *in, float *out, int64_t rows, int64_t cols, int border, float pad,
                   int iters, int threads)
{
    set_threads(threads);
    ITERATE(float, step_nms_f32(src, dst, rows, cols, border, pad))
}

/* one application only: the output is of another type than the input */
int oracle_weighted_sum_u8_f32(const uint8_t *in, float *out, int64_t rows, int64_t cols,
                               int N, int S, int E, int W, int border, uint8_t pad,
                               const float *w, int threads)
{
    set_threads(threads);
    step_weighted_sum_u8_f32(in, out, rows, cols, N, S, E, W, border, pad, w);
    return 0;
}

/* one application only: the output is of another type than the input */
int oracle_threshold_f32_u8(const float *in, uint8_t *out, int64_t rows, int64_t cols, float level, int threads)
{
    set_threads(threads);
    step_threshold_f32_u8(in, out, rows, cols, level);
    return 0;
}
