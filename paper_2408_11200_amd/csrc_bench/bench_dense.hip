// Dense basis x coefficient baseline (comparison only, not the product path):
// the layer written as one GEMM,  y = Phi * C,  Phi[b][i*(rows+1) + m] = B_{m,k}(x[b][i]) for m < rows
// and silu(x[b][i]) for m = rows,  C = the scale-folded table [n_in*(rows+1)][n_out].
// This is the O(G) formulation the local kernels avoid (Table "Complexity": Torch KAN vs Warp KAN);
// it materialises Phi in the workspace and runs the contraction through rocBLAS on the matrix cores.
// The backward pass is the same idea: gPhi = gy * C^T and gC = Phi^T * gy as two more GEMMs, dL/dx as
// the row-wise product of gPhi with dPhi/dx.
// This file belongs to the benchmark library (kan_bench.h); of the layer library it shares only the
// header-only pair evaluation.
#include <hip/hip_runtime.h>
#include <rocblas/rocblas.h>
#include "kan_bench.h"
#include "kan_device.hpp"

namespace kan {

// scale-folded table of the baseline: cf[i][m][j] = w_s[i][j] * coef[i][m][j] for m < rows, cf[i][rows][j] = w_b[i][j]
__global__ __launch_bounds__(256) void dense_fold_kernel(const float *__restrict__ coef, const float *__restrict__ w_s,
                                                         const float *__restrict__ w_b, float *__restrict__ cf,
                                                         int n_in, int rows, int n_out)
{
    const int64_t per_in = (int64_t)(rows + 1) * n_out, total = (int64_t)n_in * per_in;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < total; p += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = p / per_in, rem = p - i * per_in;
        const int64_t m = rem / n_out, j = rem % n_out;
        cf[p] = m < rows ? coef[(i * rows + m) * n_out + j] * w_s[i * n_out + j] : (w_b ? w_b[i * n_out + j] : 0.0f);
    }
}

// one thread per (sample, input): evaluate the pair and write its (rows + 1) entries of Phi
__global__ __launch_bounds__(256) void dense_expand_kernel(SplineGeom g, const float *__restrict__ x,
                                                           float *__restrict__ phi, int64_t B)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= B * g.n_in) return;
    const int i = (int)(p % g.n_in);
    const Pair pr = pair_eval<false>(x[p], g, i);
    float *out = phi + p * (g.rows + 1);
    for (int m = 0; m < g.rows; ++m) {
        const int s = m - pr.cell;
        float v = 0.0f;
#pragma unroll
        for (int q = 0; q < kMaxK; ++q) v = (s == q) ? pr.w[q] : v;
        out[m] = v;
    }
    out[g.rows] = pr.base;
}

// the same with the x-derivatives alongside
__global__ __launch_bounds__(256) void dense_expand_grad_kernel(SplineGeom g, const float *__restrict__ x,
                                                                float *__restrict__ phi, float *__restrict__ dphi,
                                                                int64_t B)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= B * g.n_in) return;
    const int i = (int)(p % g.n_in);
    const Pair pr = pair_eval<true>(x[p], g, i);
    float *out = phi + p * (g.rows + 1), *dout = dphi + p * (g.rows + 1);
    for (int m = 0; m < g.rows; ++m) {
        const int s = m - pr.cell;
        float v = 0.0f, dv = 0.0f;
#pragma unroll
        for (int q = 0; q < kMaxK; ++q) { v = (s == q) ? pr.w[q] : v; dv = (s == q) ? pr.dw[q] : dv; }
        out[m] = v;
        dout[m] = dv;
    }
    out[g.rows] = pr.base;
    dout[g.rows] = pr.dbase;
}

// gx[b][i] = sum_m gPhi[b][i][m] * dPhi[b][i][m]; one thread per (sample, input)
__global__ __launch_bounds__(256) void dense_gx_kernel(const float *__restrict__ gphi, const float *__restrict__ dphi,
                                                       float *__restrict__ gx, int64_t pairs, int per)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= pairs) return;
    float s = 0.0f;
    for (int m = 0; m < per; ++m) s = fmaf(gphi[p * per + m], dphi[p * per + m], s);
    gx[p] = s;
}

// gradient of the folded table -> gradients of coef, w_s, w_b; one thread per (input, output)
__global__ __launch_bounds__(256) void dense_unfold_kernel(const float *__restrict__ gcf, const float *__restrict__ coef,
                                                           const float *__restrict__ w_s, float *__restrict__ gcoef,
                                                           float *__restrict__ gw_s, float *__restrict__ gw_b,
                                                           int n_in, int rows, int n_out, int has_base)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)n_in * n_out) return;
    const int i = (int)(e / n_out), j = (int)(e % n_out);
    double s = 0.0;
    for (int m = 0; m < rows; ++m) {
        const float gv = gcf[((int64_t)i * (rows + 1) + m) * n_out + j];
        const int64_t at = ((int64_t)i * rows + m) * n_out + j;
        if (gcoef) gcoef[at] = w_s[e] * gv;
        s += (double)coef[at] * (double)gv;
    }
    if (gw_s) gw_s[e] = (float)s;
    if (gw_b) gw_b[e] = has_base ? gcf[((int64_t)i * (rows + 1) + rows) * n_out + j] : 0.0f;
}

}  // namespace kan

using namespace kan;

namespace {
constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
rocblas_handle g_handle = nullptr;

// brackets one launch with the event pair of kan_profile_* (a no-op while profiling is off)
struct Timed {
    hipStream_t st;
    Timed(const char *family, hipStream_t s) : st(s) { kan_profile_before(family, (void *)s); }
    ~Timed() { kan_profile_after(nullptr, (void *)st); }
};

hipError_t fold(const float *coef, const float *w_s, const float *w_b, float *cf, int n_in, int rows, int n_out,
                hipStream_t st)
{
    const int64_t want = ((int64_t)n_in * (rows + 1) * n_out + 255) / 256;
    Timed tm("dense_fold", st);
    dense_fold_kernel<<<(unsigned)(want < 8192 ? want : 8192), 256, 0, st>>>(coef, w_s, w_b, cf, n_in, rows, n_out);
    return hipGetLastError();
}
}  // namespace

extern "C" size_t kan_dense_baseline_workspace_bytes(const kan_layer_desc *d, int64_t B)
{
    if (!d || d->n_in <= 0 || d->n_out <= 0 || d->G <= 0 || d->k < 1 || d->k > 3 || B < 0) return 0;
    const size_t kd = (size_t)d->n_in * (size_t)(d->G + d->k + 1);
    return align_up(kd * (size_t)d->n_out * sizeof(float)) + align_up((size_t)B * kd * sizeof(float));
}

extern "C" int kan_dense_baseline_forward(const kan_layer_desc *d, int64_t B, const float *x, const float *coef,
                                          const float *w_s, const float *w_b, float *y, void *ws, size_t ws_bytes,
                                          void *stream)
{
    if (!d || !x || !coef || !w_s || !y) return KAN_ERR_INVALID_ARG;
    const size_t need = kan_dense_baseline_workspace_bytes(d, B);
    if (need == 0 || !(d->grid_hi > d->grid_lo)) return KAN_ERR_INVALID_ARG;
    if (d->base_act != KAN_BASE_NONE && !w_b) return KAN_ERR_INVALID_ARG;
    if (B == 0) return KAN_OK;
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < need) return KAN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    SplineGeom g;
    g.n_in = d->n_in; g.n_out = d->n_out; g.rows = d->G + d->k; g.slab_rows = g.rows + 1; g.k = d->k;
    g.lo = d->grid_lo; g.inv_h = (float)d->G / (d->grid_hi - d->grid_lo);
    g.cell_base = nullptr; g.base_act = d->base_act;
    const int64_t kd = (int64_t)g.n_in * g.slab_rows;
    float *cf = (float *)ws;
    float *phi = (float *)((char *)ws + align_up((size_t)kd * g.n_out * sizeof(float)));
    if (fold(coef, w_s, g.base_act ? w_b : nullptr, cf, g.n_in, g.rows, g.n_out, st) != hipSuccess)
        return KAN_ERR_HIP;
    {
        Timed tm("dense_expand", st);
        const int64_t pairs = B * g.n_in;
        dense_expand_kernel<<<(unsigned)((pairs + 255) / 256), 256, 0, st>>>(g, x, phi, B);
        if (hipGetLastError() != hipSuccess) return KAN_ERR_HIP;
    }
    if (!g_handle && rocblas_create_handle(&g_handle) != rocblas_status_success) return KAN_ERR_HIP;
    if (rocblas_set_stream(g_handle, st) != rocblas_status_success) return KAN_ERR_HIP;
    const float one = 1.0f, zero = 0.0f;
    Timed tm("dense_gemm", st);
    // row-major y[B][n_out] = phi[B][kd] * cf[kd][n_out]  ==  column-major y^T = cf^T * phi^T
    rocblas_status rs = rocblas_sgemm(g_handle, rocblas_operation_none, rocblas_operation_none, g.n_out, (int)B,
                                      (int)kd, &one, cf, g.n_out, phi, (int)kd, &zero, y, g.n_out);
    return rs == rocblas_status_success ? KAN_OK : KAN_ERR_HIP;
}

extern "C" size_t kan_dense_baseline_backward_workspace_bytes(const kan_layer_desc *d, int64_t B)
{
    if (!d || d->n_in <= 0 || d->n_out <= 0 || d->G <= 0 || d->k < 1 || d->k > 3 || B < 0) return 0;
    const size_t kd = (size_t)d->n_in * (size_t)(d->G + d->k + 1);
    return 2 * align_up(kd * (size_t)d->n_out * sizeof(float)) + 3 * align_up((size_t)B * kd * sizeof(float));
}

extern "C" int kan_dense_baseline_backward(const kan_layer_desc *d, int64_t B, const float *x, const float *coef,
                                           const float *w_s, const float *w_b, const float *gy, float *gx,
                                           float *gcoef, float *gw_s, float *gw_b, void *ws, size_t ws_bytes,
                                           void *stream)
{
    if (!d || !x || !coef || !w_s || !gy) return KAN_ERR_INVALID_ARG;
    const size_t need = kan_dense_baseline_backward_workspace_bytes(d, B);
    if (need == 0 || !(d->grid_hi > d->grid_lo)) return KAN_ERR_INVALID_ARG;
    if (d->base_act != KAN_BASE_NONE && !w_b) return KAN_ERR_INVALID_ARG;
    if (B == 0) return KAN_OK;
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < need) return KAN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    SplineGeom g;
    g.n_in = d->n_in; g.n_out = d->n_out; g.rows = d->G + d->k; g.slab_rows = g.rows + 1; g.k = d->k;
    g.lo = d->grid_lo; g.inv_h = (float)d->G / (d->grid_hi - d->grid_lo);
    g.cell_base = nullptr; g.base_act = d->base_act;
    const int64_t kd = (int64_t)g.n_in * g.slab_rows;
    const size_t tab = align_up((size_t)kd * g.n_out * sizeof(float)), mat = align_up((size_t)B * kd * sizeof(float));
    char *at = (char *)ws;
    float *cf = (float *)at;   at += tab;
    float *gcf = (float *)at;  at += tab;
    float *phi = (float *)at;  at += mat;
    float *dphi = (float *)at; at += mat;
    float *gphi = (float *)at;
    if (fold(coef, w_s, g.base_act ? w_b : nullptr, cf, g.n_in, g.rows, g.n_out, st) != hipSuccess)
        return KAN_ERR_HIP;
    const int64_t pairs = B * g.n_in;
    {
        Timed tm("dense_expand", st);
        dense_expand_grad_kernel<<<(unsigned)((pairs + 255) / 256), 256, 0, st>>>(g, x, phi, dphi, B);
        if (hipGetLastError() != hipSuccess) return KAN_ERR_HIP;
    }
    if (!g_handle && rocblas_create_handle(&g_handle) != rocblas_status_success) return KAN_ERR_HIP;
    if (rocblas_set_stream(g_handle, st) != rocblas_status_success) return KAN_ERR_HIP;
    const float one = 1.0f, zero = 0.0f;
    if (gx) {
        {
            // row-major gphi[B][kd] = gy[B][n_out] * cf[kd][n_out]^T  ==  column-major gphi^T = cf * gy^T
            Timed tm("dense_gemm", st);
            if (rocblas_sgemm(g_handle, rocblas_operation_transpose, rocblas_operation_none, (int)kd, (int)B, g.n_out,
                              &one, cf, g.n_out, gy, g.n_out, &zero, gphi, (int)kd) != rocblas_status_success)
                return KAN_ERR_HIP;
        }
        Timed tm("dense_gx", st);
        dense_gx_kernel<<<(unsigned)((pairs + 255) / 256), 256, 0, st>>>(gphi, dphi, gx, pairs, g.slab_rows);
        if (hipGetLastError() != hipSuccess) return KAN_ERR_HIP;
    }
    if (gcoef || gw_s || gw_b) {
        {
            // row-major gcf[kd][n_out] = phi[B][kd]^T * gy[B][n_out]  ==  column-major gcf^T = gy^T * phi
            Timed tm("dense_gemm", st);
            if (rocblas_sgemm(g_handle, rocblas_operation_none, rocblas_operation_transpose, g.n_out, (int)kd, (int)B,
                              &one, gy, g.n_out, phi, (int)kd, &zero, gcf, g.n_out) != rocblas_status_success)
                return KAN_ERR_HIP;
        }
        Timed tm("dense_unfold", st);
        const int64_t edges = (int64_t)g.n_in * g.n_out;
        dense_unfold_kernel<<<(unsigned)((edges + 255) / 256), 256, 0, st>>>(gcf, coef, w_s, gcoef, gw_s, gw_b, g.n_in,
                                                                            g.rows, g.n_out, g.base_act ? 1 : 0);
        if (hipGetLastError() != hipSuccess) return KAN_ERR_HIP;
    }
    return KAN_OK;
}
