// Customising functions of the stencil skeleton (Section 2 of the paper), written as a
// fold over the border region in (dr, dc) row-major order: init -> visit(dr, dc, weight,
// value) for every cell of the region -> finish.  The fold order is what fixes each output
// bit-for-bit, whatever workgroup size or register blocking the kernel is launched with
// (the paper's gold-standard check, Section 5, compares every workgroup size against one).
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
        int m = i % n;
        return m < 0 ? m + n : m;
    }
    return -1;
}

// Compile-time border region (north, south, east, west) ...
template <int N_, int S_, int E_, int W_>
struct HaloC {
    static constexpr bool kStatic = true;
    static constexpr int N = N_, S = S_, E = E_, W = W_;
    __host__ __device__ constexpr int n() const { return N_; }
    __host__ __device__ constexpr int s() const { return S_; }
    __host__ __device__ constexpr int e() const { return E_; }
    __host__ __device__ constexpr int w() const { return W_; }
};
// ... or one only known at launch.
struct HaloD {
    static constexpr bool kStatic = false;
    static constexpr int N = 0, S = 0, E = 0, W = 0;
    int n_, s_, e_, w_;
    __host__ __device__ int n() const { return n_; }
    __host__ __device__ int s() const { return s_; }
    __host__ __device__ int e() const { return e_; }
    __host__ __device__ int w() const { return w_; }
};

// ---- weighted sum ("gaussian" of Table 2): fp32 fma chain ---------------------------------
struct OpWeightedSum {
    using T = float;      // matrix element
    using L = float;      // what is staged in local memory
    static constexpr bool kWeights = true;
    struct State { float acc; };
    __device__ static __forceinline__ L stage(T v) { return v; }
    __device__ static __forceinline__ void init(State &s) { s.acc = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int, int, float w, L v) {
        s.acc = __fmaf_rn(w, v, s.acc);
    }
    __device__ static __forceinline__ T finish(const State &s, float) { return s.acc; }
};

// ---- Conway's Game of Life, B3/S23 ("gol") -------------------------------------------------
struct OpLife {
    using T = uint8_t;
    using L = uint8_t;
    static constexpr bool kWeights = false;
    struct State { int n; int self; };
    __device__ static __forceinline__ L stage(T v) { return v; }
    __device__ static __forceinline__ void init(State &s) { s.n = 0; s.self = 0; }
    __device__ static __forceinline__ void visit(State &s, int dr, int dc, float, L v) {
        if (dr == 0 && dc == 0) s.self = v; else s.n += v;
    }
    __device__ static __forceinline__ T finish(const State &s, float) {
        return (T)((s.n == 3) | ((s.self != 0) & (s.n == 2)));
    }
};

// ---- heat equation, explicit 5-point step ("he") --------------------------------------------
// u' = u + alpha * (((n + s) + (e + w)) - 4u), each operation rounded to fp32, in that order.
struct OpHeat {
    using T = float;
    using L = float;
    static constexpr bool kWeights = false;
    struct State { float n, w, u, e, s; };
    __device__ static __forceinline__ L stage(T v) { return v; }
    __device__ static __forceinline__ void init(State &s) { s.n = s.w = s.u = s.e = s.s = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int dr, int dc, float, L v) {
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
        float t = __fsub_rn(sum, __fmul_rn(4.0f, s.u));
        return __fadd_rn(s.u, __fmul_rn(alpha, t));
    }
};

// ---- compute-intensive synthetic stencil: sum of w * sin(x) + cos(x) over the region ------
// sin and cos are evaluated once per staged cell (fp32) and kept side by side in local
// memory; the fold keeps one fma chain for the sines and one sum for the cosines.
struct OpSinCos {
    using T = float;
    using L = float2;     // (sin x, cos x)
    static constexpr bool kWeights = true;
    struct State { float s, c; };
    __device__ static __forceinline__ L stage(T v) {
        float sn, cs;
        sincosf(v, &sn, &cs);
        return make_float2(sn, cs);
    }
    __device__ static __forceinline__ void init(State &s) { s.s = 0.0f; s.c = 0.0f; }
    __device__ static __forceinline__ void visit(State &s, int, int, float w, L v) {
        s.s = __fmaf_rn(w, v.x, s.s);
        s.c = __fadd_rn(s.c, v.y);
    }
    __device__ static __forceinline__ T finish(const State &s, float) { return __fadd_rn(s.s, s.c); }
};

}  // namespace sk
