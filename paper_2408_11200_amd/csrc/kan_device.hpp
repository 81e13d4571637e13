// Device-side helpers shared by the KAN / UKAN kernels (gfx950, wave64).
//
// pair_eval() is the per-(sample, input) part of the local B-spline form
// (section "Algorithm", Eq. "matrixform"): interval index, local coordinate
// and the k+1 window weights, plus their x-derivatives and the SiLU base term.
// It runs once per pair and its results are reused for every output, so none
// of it is on the per-edge critical path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// The kernels are written for a window of KAN_MAXK rows (4: degrees up to 3, the default).  The
// generic kernels are compiled a second time with a window of 6 (degrees 4 and 5) in a namespace of
// their own; that translation unit sets both macros before including this header.
#ifndef KAN_MAXK
#define KAN_MAXK 4
#define KAN_NS kan
#endif

namespace KAN_NS {

constexpr int kMaxK = KAN_MAXK;   // window width supported by the kernels (degree k <= kMaxK - 1)
constexpr int kWave = 64;

// Geometry of one spline evaluation problem as the kernels see it.  A bounded
// KAN layer has rows == G + k and cell_base == nullptr; a UKAN layer evaluates
// on a per-input slab of a generated table whose first row is the global
// coefficient (cell_base[i] - K), so its relative cell is cell - cell_base[i].
struct SplineGeom {
    int n_in, n_out;
    int rows;                  // coefficient rows per input
    int slab_rows;             // rows per input in the scale-folded table: rows, or rows + 1 when
                               // the table carries w_b as an extra last row
    int k;                     // degree
    float lo, inv_h;           // grid start and reciprocal cell width
    const int32_t *cell_base;  // per input, or nullptr (== 0)
    int base_act;              // 0 none, 1 SiLU
};

// floor(t) as int32, saturated to +-2^30; NaN maps to -2^30.
__device__ __forceinline__ int32_t saturating_floor(float t)
{
    float f = floorf(t);
    if (!(f > -1073741824.0f)) return -1073741824;
    if (!(f < 1073741824.0f)) return 1073741824;
    return (int32_t)f;
}

// Interval index of x: two separately rounded fp32 operations, never fused,
// so that the integer agrees bit for bit with the plain definition.
__device__ __forceinline__ int32_t interval_index(float x, float lo, float inv_h, float *t_out, float *d_out)
{
    float d = __fsub_rn(x, lo);
    float t = __fmul_rn(d, inv_h);
    *t_out = t;
    *d_out = d;
    return saturating_floor(t);
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }

__device__ __forceinline__ float silu_grad_f(float x)
{
    float s = 1.0f / (1.0f + expf(-x));
    return s * (1.0f + x * (1.0f - s));
}

// Result of pair_eval.  `cell` is the relative cell, clamped to [-kMaxK, rows]
// (any value outside [-k, rows-1] means: every weight is zero).  w[s] / dw[s]
// multiply coefficient row cell + s; entries whose row falls outside
// [0, rows) or with s > k are already zero, so callers may clamp row indices
// freely.
struct Pair {
    int cell;
    float w[kMaxK];
    float dw[kMaxK];
    float base, dbase;
};

template <bool WANT_GRAD>
__device__ __forceinline__ Pair pair_eval(float x, const SplineGeom &g, int i)
{
    Pair p;
    float t, d;
    int32_t idx = interval_index(x, g.lo, g.inv_h, &t, &d);
    long long rel = (long long)idx - (g.cell_base ? (long long)g.cell_base[i] : 0ll);
    rel = rel < -kMaxK ? -kMaxK : (rel > g.rows ? g.rows : rel);
    p.cell = (int)rel;
    // local coordinate: exact product minus the integer, one rounding; the rounding error of the
    // subtraction x - lo (recovered exactly by the two-sum below) is added back, because the
    // x-derivative multiplies it by inv_h twice and fine grids would otherwise lose digits
    const float bb = __fsub_rn(d, x);                                          // ~ -lo
    const float d_err = __fadd_rn(__fsub_rn(x, __fsub_rn(d, bb)), __fsub_rn(-g.lo, bb));
    float u = fmaf(d_err, g.inv_h, fmaf(d, g.inv_h, -floorf(t)));

    // Cox-de Boor on one cell of a uniform grid:
    //   N^d_s = ((u + d - s) N^{d-1}_{s-1} + (s + 1 - u) N^{d-1}_s) / d
    float n[kMaxK], low[kMaxK];
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) { n[s] = (s == 0) ? 1.0f : 0.0f; low[s] = 0.0f; }
#pragma unroll
    for (int dg = 1; dg < kMaxK; ++dg) {
        if (dg <= g.k) {
            float prev[kMaxK];
#pragma unroll
            for (int s = 0; s < kMaxK; ++s) prev[s] = n[s];
            if (dg == g.k) {
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) low[s] = prev[s];
            }
            const float inv_d = 1.0f / (float)dg;
#pragma unroll
            for (int s = 0; s <= dg; ++s) {
                float a = (s >= 1) ? prev[s - 1] : 0.0f;
                float b = (s <= dg - 1) ? prev[s] : 0.0f;
                n[s] = ((u + (float)(dg - s)) * a + ((float)(s + 1) - u) * b) * inv_d;
            }
        }
    }
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) {
        int row = p.cell + s;
        bool ok = (s <= g.k) && (row >= 0) && (row < g.rows);
        p.w[s] = ok ? n[s] : 0.0f;
        if (WANT_GRAD) {
            float a = (s >= 1) ? low[s - 1] : 0.0f;
            float b = (s <= g.k - 1) ? low[s] : 0.0f;
            p.dw[s] = ok ? (a - b) * g.inv_h : 0.0f;
        } else {
            p.dw[s] = 0.0f;
        }
    }
    p.base = (g.base_act == 1) ? silu_f(x) : 0.0f;
    p.dbase = (WANT_GRAD && g.base_act == 1) ? silu_grad_f(x) : 0.0f;
    return p;
}

// Window form of a pair: a window of kMaxK consecutive rows that lies inside the table (first row
// `row0` in [0, rows - kMaxK]) with the weights shifted to match, so that callers never index
// outside the table.  Needs rows >= kMaxK.
template <bool GRAD>
__device__ __forceinline__ void window_of(const Pair &p, int rows, int &row0, float (&w)[kMaxK], float &base)
{
    const int hi = rows - kMaxK;
    const int cc = p.cell < 0 ? 0 : (p.cell > hi ? hi : p.cell);
    const int d = cc - p.cell;
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) {
        float v = 0.0f;
#pragma unroll
        for (int q = 0; q < kMaxK; ++q) {
            const float src = GRAD ? p.dw[q] : p.w[q];
            v = (s + d == q) ? src : v;
        }
        w[s] = v;
    }
    row0 = cc;
    base = GRAD ? p.dbase : p.base;
}

// value of lane `src` (wave-uniform index) as a scalar
__device__ __forceinline__ float lane_f(float v, int src)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src));
}
__device__ __forceinline__ int lane_i(int v, int src) { return __builtin_amdgcn_readlane(v, src); }

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

}  // namespace KAN_NS
