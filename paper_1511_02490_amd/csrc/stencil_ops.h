// Customising functions of the stencil skeleton (Section 2 of the paper), written as a
// fold over the border region in (dr, dc) row-major order: init -> visit(dr, dc, weight,
// value) for every cell of the region -> finish.  The fold order is what fixes each output
// bit-for-bit, whatever workgroup size or register blocking the kernel is launched with
// (the paper's gold-standard check, Section 5, compares every workgroup size against one).
//
// Each function names: T, the matrix element; V, what the fold consumes per cell (T itself,
// or something computed from it once per cell); kPlanes and L: V is kept in local memory as
// kPlanes separate planes of L, so that neighbouring lanes read neighbouring addresses.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sk {

enum Border : int { kClamp = 0, kWrap = 1, kConstant = 2 };

// Border substitution for one axis (Section 2): nearest in-matrix index, periodic index, or
// -1 meaning "use the padding value".
template <int B>
__device__ __forceinline__ int resolve(int i, int n) {
    if ((unsigned)i < (unsigned)n) return i;
    if (B == kClamp) return i < 0 ? 0 : n - 1;
    if (B == kWrap) {
        // one period away in all but tiny matrices: an add; the division only beyond that
        const int once = i < 0 ? i + n : i - n;
        if (__builtin_expect((unsigned)once < (unsigned)n, 1)) return once;
        int m = i % n;
        return m < 0 ? m + n : m;
    }
    return -1;
}

// Compile-time border region (north, south, east, west) ...
template <int N_, int S_, int E_, int W_>
struct HaloC {
    static constexpr bool kStatic = true;
    static constexpr bool kMasked = false;
    static constexpr int N = N_, S = S_, E = E_, W = W_;
    __host__ __device__ constexpr int n() const { return N_; }
    __host__ __device__ constexpr int s() const { return S_; }
    __host__ __device__ constexpr int e() const { return E_; }
    __host__ __device__ constexpr int w() const { return W_; }
};
// ... or one only known at launch.
struct HaloD {
    static constexpr bool kStatic = false;
    static constexpr bool kMasked = false;
    static constexpr int N = 0, S = 0, E = 0, W = 0;
    int n_, s_, e_, w_;
    __host__ __device__ int n() const { return n_; }
    __host__ __device__ int s() const { return s_; }
    __host__ __device__ int e() const { return e_; }
    __host__ __device__ int w() const { return w_; }
};

// ---- weighted sum ("gaussian" of Table 2): fp32 fma chain ---------------------------------
struct OpWeightedSum {
    static constexpr bool kRowFold = false;
    using T = float;
    using L = float;
    using V = float;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = true;
    struct State { float acc; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.acc = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int, int, float w, V v) {
        s.acc = __fmaf_rn(w, v, s.acc);
    }
    __device__ static __forceinline__ T finish(const State &s, float) { return s.acc; }
};

// ---- the same weighted sum on the paper's other element types (Section 3.3: integers, single
// or double precision): double with an fp64 fma chain, int32 with wrap-around arithmetic
// (the weight table must then hold integers).
struct OpWeightedSumF64 {
    static constexpr bool kRowFold = false;
    using T = double;
    using L = double;
    using V = double;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = true;
    using Wt = double;
    struct State { double acc; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.acc = 0.0; }
    __device__ static __forceinline__ void visit(State &s, int, int, double w, V v) {
        s.acc = __fma_rn(w, v, s.acc);      // (w is a float's value: the conversion is exact wherever it is made)
    }
    __device__ static __forceinline__ T finish(const State &s, float) { return s.acc; }
};

struct OpWeightedSumI32 {
    static constexpr bool kRowFold = false;
    using T = int32_t;
    using L = int32_t;
    using V = int32_t;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = true;
    struct State { uint32_t acc; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.acc = 0u; }
    __device__ static __forceinline__ void visit(State &s, int, int, float w, V v) {
        s.acc += (uint32_t)(int32_t)w * (uint32_t)v;      // modulo 2^32
    }
    __device__ static __forceinline__ T finish(const State &s, float) { return (T)s.acc; }
};

// The weighted sum of a byte matrix, written as floats: a kernel whose input and output element
// types differ (Section 3.3 lists both among a kernel's features) - an 8-bit image blurred into
// floats, the first stage of the Canny detector.  Cells become floats when they are staged
// (exact); from there on it is the fp32 fma chain above.  O names the output element type where
// it is not T.
struct OpWeightedSumU8 {
    static constexpr bool kRowFold = false;
    using T = uint8_t;
    using O = float;
    using L = float;
    using V = float;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = true;
    struct State { float acc; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = (float)v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = (float)v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.acc = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int, int, float w, V v) {
        s.acc = __fmaf_rn(w, v, s.acc);
    }
    __device__ static __forceinline__ O finish(const State &s, float) { return s.acc; }
};

// The type in which a compile-time weight table travels in the kernel arguments: Op::Wt where the
// function names one (doubles for the fp64 sum: a scalar register pair is an operand of the fp64
// fma, a float would first have to be converted into a pair of vector registers), else float.
template <class Op, class = void>
struct weight_type_of { using type = float; };
template <class Op>
struct weight_type_of<Op, decltype(void(sizeof(typename Op::Wt)))> { using type = typename Op::Wt; };

// The output element type of a customising function: Op::O where it names one, else Op::T.
template <class Op, class = void>
struct out_type_of { using type = typename Op::T; };
template <class Op>
struct out_type_of<Op, decltype(void(sizeof(typename Op::O)))> { using type = typename Op::O; };

// Packed bytes, each below 0x80: 0x01 in every byte of the result whose byte of x is zero.
// (Adding 0x7f carries into a byte's top bit exactly when the byte is not zero, and never beyond.)
__device__ __forceinline__ uint32_t zero_bytes(uint32_t x) {
    return ~((x + 0x7f7f7f7fu) >> 7) & 0x01010101u;
}

// ---- Conway's Game of Life, B3/S23 ("gol") -------------------------------------------------
struct OpLife {
    static constexpr bool kRowFold = false;
    using T = uint8_t;
    using L = uint8_t;
    using V = uint8_t;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = false;
    struct State { int n; int self; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.n = 0; s.self = 0; }
    __device__ static __forceinline__ void visit(State &s, int dr, int dc, float, V v) {
        if (dr == 0 && dc == 0) s.self = v; else s.n += v;
    }
    __device__ static __forceinline__ T finish(const State &s, float) {
        return (T)((s.n == 3) | ((s.self != 0) & (s.n == 2)));
    }
};

// ---- heat equation, explicit 5-point step ("he") --------------------------------------------
// u' = u + alpha * (((n + s) + (e + w)) - 4u), each operation rounded to fp32, in that order.
struct OpHeat {
    static constexpr bool kRowFold = false;
    using T = float;
    using L = float;
    using V = float;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = false;
    struct State { float n, w, u, e, s; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.n = s.w = s.u = s.e = s.s = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int dr, int dc, float, V v) {
        if (dr == -1 && dc == 0) s.n = v;
        else if (dr == 0 && dc == -1) s.w = v;
        else if (dr == 0 && dc == 0) s.u = v;
        else if (dr == 0 && dc == 1) s.e = v;
        else if (dr == 1 && dc == 0) s.s = v;
    }
    __device__ static __forceinline__ T finish(const State &s, float alpha) {
        float ns = __fadd_rn(s.n, s.s);
        float ew = __fadd_rn(s.e, s.w);
        float sum = __fadd_rn(ns, ew);
        // 4u is exact (a power-of-two multiple), so one fma rounds exactly where the separate
        // multiply and subtract would (they differ only where 4u overflows)
        float t = __fmaf_rn(-4.0f, s.u, sum);
        return __fadd_rn(s.u, __fmul_rn(alpha, t));
    }
};

// ---- the Canny detector's stencils (Table 2: sobel, nms, threshold) --------------------------
// The paper names them and gives their border regions; the formulas are this library's, every
// operation rounded to fp32 in the order written.
//
// sobel: gx = ((ne - nw) + 2 (e - w)) + (se - sw), gy = ((sw - nw) + 2 (s - n)) + (se - ne),
// out = sqrt(gx gx + gy gy).  (a + 2 b is one fma: 2 b is exact, so nothing is rounded differently.)
struct OpSobel {
    static constexpr bool kRowFold = false;
    using T = float;
    using L = float;
    using V = float;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = false;
    struct State { float nw, n, ne, w, e, sw, s, se; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.nw = s.n = s.ne = s.w = s.e = s.sw = s.s = s.se = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int dr, int dc, float, V v) {
        if (dr == -1) { if (dc == -1) s.nw = v; else if (dc == 0) s.n = v; else s.ne = v; }
        else if (dr == 0) { if (dc == -1) s.w = v; else if (dc == 1) s.e = v; }
        else { if (dc == -1) s.sw = v; else if (dc == 0) s.s = v; else s.se = v; }
    }
    __device__ static __forceinline__ T finish(const State &s, float) {
        const float gx = __fadd_rn(__fmaf_rn(2.0f, __fsub_rn(s.e, s.w), __fsub_rn(s.ne, s.nw)), __fsub_rn(s.se, s.sw));
        const float gy = __fadd_rn(__fmaf_rn(2.0f, __fsub_rn(s.s, s.n), __fsub_rn(s.sw, s.nw)), __fsub_rn(s.se, s.ne));
        // sqrtf is the correctly rounded root (the shorter intrinsic is not)
        return sqrtf(__fadd_rn(__fmul_rn(gx, gx), __fmul_rn(gy, gy)));
    }
};

// nms: a cell keeps its value if it is no smaller than both its west and east neighbours, or no
// smaller than both its north and south neighbours; otherwise it becomes 0.
struct OpNms {
    static constexpr bool kRowFold = false;
    using T = float;
    using L = float;
    using V = float;
    static constexpr int kPlanes = 1;
    static constexpr bool kWeights = false;
    struct State { float n, w, u, e, s; };
    __device__ static __forceinline__ void stage(T v, L (&out)[1]) { out[0] = v; }
    __device__ static __forceinline__ V combine(const L (&p)[1]) { return p[0]; }
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[1][CC]) {
#pragma unroll
        for (int k = 0; k < CC; ++k) out[0][k] = v[k];
    }
    __device__ static __forceinline__ void init(State &s) { s.n = s.w = s.u = s.e = s.s = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int dr, int dc, float, V v) {
        if (dr == -1 && dc == 0) s.n = v;
        else if (dr == 0 && dc == -1) s.w = v;
        else if (dr == 0 && dc == 0) s.u = v;
        else if (dr == 0 && dc == 1) s.e = v;
        else if (dr == 1 && dc == 0) s.s = v;
    }
    __device__ static __forceinline__ T finish(const State &s, float) {
        const bool keep = (s.u >= s.w && s.u >= s.e) || (s.u >= s.n && s.u >= s.s);
        return keep ? s.u : 0.0f;
    }
};

// ---- compute-intensive synthetic stencil: sum of w * sin(x) + cos(x) over the region ------
// sin and cos are evaluated once per staged cell (fp32) and kept side by side in local
// memory (one plane each).  The fold keeps one fma chain for the sines.  The cosines are summed
// as a fixed tree, the same for every cell whatever kernel computes it, whose inner nodes
// neighbouring cells have in common: the cosines of one region row pairwise from the west end
// ((c0 + c1) + (c2 + c3) + ...), so that the cells of a work-item share pair sums; the row sums
// h(0), h(1), ... (north to south) in chunks of four rows, ((h0 + h1) + (h2 + h3)), then a pair
// (h + h') and a single row for what is left, the chunks added north to south.  Pairs and
// fours of rows that start an even number of rows apart are the same for output rows below
// each other, so a kernel that marches down the matrix forms each of them once.

// sin and cos of x in fp32 for |x| <= 2^16, absolute error below 2e-7: x / (2 pi) is formed
// as a two-term product (1 / (2 pi) split into an fp32 head and tail, fma for the exact
// partial products), its integer part is dropped, and the hardware sine / cosine (which take
// their argument in turns) finish the job.
__device__ __forceinline__ void sincos_small_f32(float x, float &sn_out, float &cs_out) {
    const float kInv2PiHi = 0.15915493667125702f, kInv2PiLo = 6.4206383e-09f;
    const float hi = __fmul_rn(x, kInv2PiHi);
    const float lo = __fmaf_rn(x, kInv2PiLo, __fmaf_rn(x, kInv2PiHi, -hi));
    const float turns = __fadd_rn(__fsub_rn(hi, rintf(hi)), lo);
    sn_out = __builtin_amdgcn_sinf(turns);
    cs_out = __builtin_amdgcn_cosf(turns);
}
// ... and for |x| <= 2, where one rounded product is already that accurate (the angle is off by
// at most |x| * 1e-7) and less than half a turn, so nothing has to be dropped.
__device__ __forceinline__ void sincos_tiny_f32(float x, float &sn_out, float &cs_out) {
    const float turns = __fmul_rn(x, 0.15915493667125702f);
    sn_out = __builtin_amdgcn_sinf(turns);
    cs_out = __builtin_amdgcn_cosf(turns);
}
constexpr float kSinCosTinyLimit = 2.0f;
constexpr float kSinCosSmallLimit = 65536.0f;   // beyond this (or NaN) the library routine is used

struct OpSinCos {
    using T = float;
    using L = float;
    using V = float2;     // (sin x, cos x)
    static constexpr int kPlanes = 2;   // a plane of sines and a plane of cosines
    static constexpr bool kWeights = true;
    static constexpr bool kRowFold = true;
    // s: the sines' fma chain; c: the chunks of cosine row sums added so far; p, q: the chunk being formed
    struct State { float s, c, p, q; };
    // which routine serves an element depends on that element alone, so every mapping computes
    // the same bits for it
    __device__ static __forceinline__ void stage(T v, L (&out)[2]) {
        const float m = fabsf(v);
        if (__builtin_expect(m <= kSinCosTinyLimit, 1))
            sincos_tiny_f32(v, out[0], out[1]);
        else if (m <= kSinCosSmallLimit)
            sincos_small_f32(v, out[0], out[1]);
        else
            sincosf(v, &out[0], &out[1]);
    }
    // CC cells at once: one test of the largest magnitude serves all of them.  (A NaN does not
    // raise the maximum; the short routine turns it into NaN like the others would.  Inf does.)
    template <int CC>
    __device__ static __forceinline__ void stage_vec(const T (&v)[CC], L (&out)[2][CC]) {
        float mag = fabsf(v[0]);
#pragma unroll
        for (int k = 1; k < CC; ++k) mag = fmaxf(mag, fabsf(v[k]));
        if (__builtin_expect(mag <= kSinCosTinyLimit, 1)) {
#pragma unroll
            for (int k = 0; k < CC; ++k) sincos_tiny_f32(v[k], out[0][k], out[1][k]);
        } else {
            // rare: one element per trip of a rolled loop, so that the long routines appear once;
            // inputs and results rotate through scalars (no indexed array, nothing leaves registers)
            static_assert(CC == 4, "four-cell vectors");
            T x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
            L s0 = 0, s1 = 0, s2 = 0, s3 = 0, c0 = 0, c1 = 0, c2 = 0, c3 = 0;
#pragma unroll 1
            for (int k = 0; k < CC; ++k) {
                L one[2];
                stage(x0, one);
                x0 = x1, x1 = x2, x2 = x3;
                s0 = s1, s1 = s2, s2 = s3, s3 = one[0];
                c0 = c1, c1 = c2, c2 = c3, c3 = one[1];
            }
            out[0][0] = s0, out[0][1] = s1, out[0][2] = s2, out[0][3] = s3;
            out[1][0] = c0, out[1][1] = c1, out[1][2] = c2, out[1][3] = c3;
        }
    }
    __device__ static __forceinline__ V combine(const L (&p)[2]) { return make_float2(p[0], p[1]); }
    // The chain starts from -0, the one value that x + (-0) = x holds for with every x, signed
    // zeros included: its first fma is then a plain product and needs no register cleared.
    __device__ static __forceinline__ void init(State &s) { s.s = -0.0f; s.c = s.p = s.q = 0.0f; }

    // The sines of one region row into the fma chain: w(dc) and v(dc) give weight and staged
    // value at column offset dc.
    template <class WAcc, class VAcc>
    __device__ static __forceinline__ void fold_sines(State &s, int W, int E, WAcc w, VAcc v) {
        for (int dc = -W; dc <= E; ++dc) s.s = __fmaf_rn(w(dc), v(dc).x, s.s);
    }
    // h: the cosines of one region row, summed pairwise from the west end.
    template <class VAcc>
    __device__ static __forceinline__ float row_cos(int W, int E, VAcc v) {
        int dc = -W;
        float h;
        if (dc + 1 <= E) {
            h = __fadd_rn(v(dc).y, v(dc + 1).y);
            dc += 2;
        } else {
            h = v(dc).y;
            dc += 1;
        }
        for (; dc + 1 <= E; dc += 2) h = __fadd_rn(h, __fadd_rn(v(dc).y, v(dc + 1).y));
        if (dc <= E) h = __fadd_rn(h, v(dc).y);
        return h;
    }
    // Row sum h of region row k (0 = northernmost) of R into the tree: chunks of four rows
    // ((h + h) + (h + h)), then a pair and a single row for what is left; chunks added north to south.
    __device__ static __forceinline__ void push_cos(State &s, int k, int R, float h) {
        const int m = k & 3;
        if (m == 0) {
            s.p = h;
        } else if (m == 1) {
            s.p = __fadd_rn(s.p, h);
        } else if (m == 2) {
            s.q = h;
        } else {
            s.q = __fadd_rn(s.q, h);
            s.p = __fadd_rn(s.p, s.q);
            s.c = k == 3 ? s.p : __fadd_rn(s.c, s.p);
        }
        if (k == R - 1 && (R & 3) != 0) {
            // one, two or three rows after the last whole chunk: p holds the row or the pair, q a third row
            s.c = R < 4 ? s.p : __fadd_rn(s.c, s.p);
            if ((R & 3) == 3) s.c = __fadd_rn(s.c, s.q);
        }
    }
    // The same tree for a kernel that keeps, for every input row t it has seen, h(t), the pair
    // h(t-1) + h(t) and the four (pair(t-2) + pair(t)): the sum over the R rows that end at the
    // current one.  get(level, back) = level 0 / 1 / 2: row sum / pair / four ending `back` rows
    // before the current row.
    template <int R, class Get>
    __device__ static __forceinline__ float window_cos(Get get) {
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < R / 4; ++i) {                   // rows 4i .. 4i + 3
            const float chunk = get(2, R - 4 - 4 * i);
            acc = i == 0 ? chunk : __fadd_rn(acc, chunk);
        }
        if constexpr ((R & 2) != 0) {                       // the pair after the last four
            const float chunk = get(1, R & 1);
            acc = R < 4 ? chunk : __fadd_rn(acc, chunk);
        }
        if constexpr ((R & 1) != 0) {                       // the last row
            const float chunk = get(0, 0);
            acc = R == 1 ? chunk : __fadd_rn(acc, chunk);
        }
        return acc;
    }
    __device__ static __forceinline__ void set_cos(State &s, float c) { s.c = c; }

    // one row of the region, k-th of R from the north
    template <class WAcc, class VAcc>
    __device__ static __forceinline__ void visit_row(State &s, int k, int R, int W, int E, WAcc w, VAcc v) {
        fold_sines(s, W, E, w, v);
        push_cos(s, k, R, row_cos(W, E, v));
    }
    // The same row fold, one value at a time (j = 0, 1, ... counts the row's cells from its west
    // end): the operations, and so the bits, of visit_row.
    struct RowState { float pending, h; };
    __device__ static __forceinline__ void row_visit(State &s, RowState &rs, int j, float w, V v) {
        s.s = __fmaf_rn(w, v.x, s.s);
        if (j & 1) {
            const float pair = __fadd_rn(rs.pending, v.y);
            rs.h = j == 1 ? pair : __fadd_rn(rs.h, pair);
        } else {
            rs.pending = v.y;
        }
    }
    __device__ static __forceinline__ void row_end(State &s, const RowState &rs, int count, int k, int R) {
        float h = rs.h;
        if (count & 1) h = count == 1 ? rs.pending : __fadd_rn(rs.h, rs.pending);
        push_cos(s, k, R, h);
    }
    __device__ static __forceinline__ T finish(const State &s, float) { return __fadd_rn(s.s, s.c); }
};

// One row of the region - row dr, the k-th of R from the north - folded into a cell's state.
template <class Op, class WAcc, class VAcc>
__device__ __forceinline__ void fold_row(typename Op::State &st, int dr, int k, int R, int W, int E, WAcc w, VAcc v) {
    if constexpr (Op::kRowFold) {
        Op::visit_row(st, k, R, W, E, w, v);
    } else {
        for (int dc = -W; dc <= E; ++dc) Op::visit(st, dr, dc, w(dc), v(dc));
    }
}

}  // namespace sk
