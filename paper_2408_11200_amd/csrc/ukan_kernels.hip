// Kernels of the UKAN-specific part: cell / group bookkeeping on the unbounded grid,
// the coefficient-generator (CG) MLP forward and backward.  The B-spline evaluation on
// the generated table is done by the same kernels as the bounded layer.
//
// The dense contractions of the CG run on the matrix cores in fp32
// (v_mfma_f32_32x32x2_f32); everything else here is small and bandwidth-bound.
#include <limits.h>
#include "kan_device.hpp"
#include "kan_launch.hpp"
#include "ukan_launch.hpp"

namespace kan {

// floor division by a positive K and the matching non-negative remainder
__device__ __forceinline__ int floordiv(int a, int K) { int q = a / K; return (a % K < 0) ? q - 1 : q; }

// ---- cell / group / offset export -------------------------------------------
__global__ void group_index_kernel(const float *__restrict__ x, int32_t *__restrict__ cell,
                                   int32_t *__restrict__ grp, int32_t *__restrict__ off, int64_t n,
                                   float inv_h, int K)
{
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    float t, d;
    int32_t c = interval_index(x[p], 0.0f, inv_h, &t, &d);
    int32_t g = floordiv(c, K);
    if (cell) cell[p] = c;
    if (grp) grp[p] = g;
    if (off) off[p] = c - g * K;
}

// ---- per-input range of cells -------------------------------------------------
__global__ void range_init_kernel(int32_t *__restrict__ cmin, int32_t *__restrict__ cmax, int n_in)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_in) { cmin[i] = INT_MAX; cmax[i] = INT_MIN; }
}

// lanes <-> inputs (coalesced rows of x); blockIdx.y strides over the batch.  Integer
// min/max atomics: order-independent, so the result is deterministic.
__global__ __launch_bounds__(256) void range_kernel(const float *__restrict__ x, int32_t *__restrict__ cmin,
                                                    int32_t *__restrict__ cmax, int64_t B, int n_in, float inv_h)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_in) return;
    int lo = INT_MAX, hi = INT_MIN;
    int64_t b = blockIdx.y;
    // four rows in flight per thread (the scan is bound by load latency otherwise)
    for (; b + 3 * (int64_t)gridDim.y < B; b += 4 * (int64_t)gridDim.y) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = x[(b + u * (int64_t)gridDim.y) * n_in + i];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float t, d;
            const int c = interval_index(v[u], 0.0f, inv_h, &t, &d);
            lo = c < lo ? c : lo;
            hi = c > hi ? c : hi;
        }
    }
    for (; b < B; b += gridDim.y) {
        float t, d;
        int c = interval_index(x[b * n_in + i], 0.0f, inv_h, &t, &d);
        lo = c < lo ? c : lo;
        hi = c > hi ? c : hi;
    }
    if (lo <= hi) { atomicMin(&cmin[i], lo); atomicMax(&cmax[i], hi); }
}

// cells -> first group held, group count, relative-cell base; the widest span goes to summary[0]
__global__ __launch_bounds__(256) void range_finalize_kernel(const int32_t *__restrict__ cmin,
                                                             const int32_t *__restrict__ cmax,
                                                             int32_t *__restrict__ g_first,
                                                             int32_t *__restrict__ n_groups,
                                                             int32_t *__restrict__ cell_base,
                                                             int32_t *__restrict__ summary, int n_in, int K)
{
    __shared__ long long widest[256];
    long long w = 0;
    for (int i = threadIdx.x; i < n_in; i += blockDim.x) {
        int gmin = floordiv(cmin[i], K), gmax = floordiv(cmax[i], K);
        long long n = (long long)gmax - (long long)gmin + 2;      // groups gmin-1 .. gmax
        g_first[i] = gmin - 1;
        n_groups[i] = n > INT_MAX ? INT_MAX : (int)n;
        cell_base[i] = gmin * K;        // cell c reads table rows c - gmin*K .. + K-1
        w = n > w ? n : w;
    }
    widest[threadIdx.x] = w;
    __syncthreads();
    for (int s = blockDim.x / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s && widest[threadIdx.x + s] > widest[threadIdx.x]) widest[threadIdx.x] = widest[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) summary[0] = widest[0] > INT_MAX ? INT_MAX : (int)widest[0];
}

// overflow[0] = 1 when the widest span found exceeds what the caller provided for, else 0
__global__ void span_check_kernel(const int32_t *__restrict__ summary, int provided, int32_t *__restrict__ overflow)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) overflow[0] = summary[0] > provided ? 1 : 0;
}

// ---- CG input and hidden layer -------------------------------------------------
// Row (i, t) of the generator batch is group g_first[i] + t of input i.  One block per
// row: z = [E[i] ; PE(g)] (PE evaluated in fp64, rounded to fp32),
// pre = W1^T z + b1, hid = silu(pre).
__global__ __launch_bounds__(64) void cg_hidden_kernel(const float *__restrict__ E, const float *__restrict__ W1,
                                                       const float *__restrict__ b1,
                                                       const int32_t *__restrict__ g_first, float *__restrict__ z,
                                                       float *__restrict__ pre, float *__restrict__ hid, int n_g,
                                                       int d_pe, int d_feat, int d_hid)
{
    extern __shared__ float zs[];
    const int row = blockIdx.x;
    const int i = row / n_g, t = row % n_g;
    const int dz = d_feat + d_pe;
    const int g = g_first[i] + t;
    for (int c = threadIdx.x; c < dz; c += blockDim.x) {
        float v;
        if (c < d_feat) {
            v = E[(int64_t)i * d_feat + c];
        } else {
            int q = c - d_feat;
            double freq = pow(10000.0, -2.0 * (double)(q / 2) / (double)d_pe);
            double ang = (double)g * freq;
            v = (float)((q & 1) ? cos(ang) : sin(ang));
        }
        zs[c] = v;
        if (z) z[(int64_t)row * dz + c] = v;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < d_hid; c += blockDim.x) {
        // fp64 accumulation: this layer is tiny and its rounding error would otherwise be
        // amplified into every generated coefficient
        double sd = (double)b1[c];
        for (int p = 0; p < dz; ++p) sd += (double)zs[p] * (double)W1[(int64_t)p * d_hid + c];
        const float s = (float)sd;
        if (pre) pre[(int64_t)row * d_hid + c] = s;
        hid[(int64_t)row * d_hid + c] = (float)(sd / (1.0 + exp(-sd)));
    }
}

// ---- matrix-core GEMM ------------------------------------------------------------
// C(m,n) = sum_k A(m,k) B(k,n), fp32 operands addressed through (row, column) strides so that
// transposed views need no copy.  One block = 4 waves = one 64x64 tile of C; each wave owns a
// 32x32 quadrant; K-slices are staged through LDS.  blockIdx.z selects a slice of K (split-K):
// slice z writes its own copy of C at C + z*c_slice.
//   ACC64 = false: v_mfma_f32_32x32x2_f32, fp32 accumulation folded every 64 terms (forward).
//   ACC64 = true : operands widened to fp64, v_mfma_f64_16x16x4_f64.  Used by the CG backward
//                  pass, whose long sums cancel heavily; the products are then exact and the
//                  only rounding is the final conversion to fp32.
using f32x16 = __attribute__((__vector_size__(16 * sizeof(float)))) float;
using f64x4 = __attribute__((__vector_size__(4 * sizeof(double)))) double;

template <int EPI, typename V>
__device__ __forceinline__ void gemm_store(const GemmArgs &a, float *C, int64_t m, int64_t n, V acc)
{
    if (m >= a.M || n >= a.N) return;
    if (EPI == EPI_PLAIN) {
        C[m * a.ldc + n] = (float)acc;
    } else if (EPI == EPI_CG_OUT) {
        // generator output: add b2, keep the raw value if asked, store the scale-folded one
        float val = (float)acc + a.bias[n];
        const int64_t i = m / a.rows_per_input;
        const float sc = a.scale[i * a.n_out + (n % a.n_out)];
        if (a.C2) a.C2[m * a.ldc + n] = val;
        C[m * a.ldc + n] = val * sc;
    } else {   // EPI_SILU_GRAD: multiply by silu'(pre), evaluated in fp64
        const double x = (double)a.aux[m * a.ldc + n];
        const double sg = 1.0 / (1.0 + exp(-x));
        C[m * a.ldc + n] = (float)((double)acc * (sg * (1.0 + x * (1.0 - sg))));
    }
}

template <int EPI, bool ACC64>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs a)
{
    constexpr int BM = 64, BN = 64, BK = 16, PAD = 4;
    // two LDS stages: the next K step is fetched into registers while the current one is multiplied,
    // then parked in the other stage; one barrier per step
    __shared__ float As[2][BK][BM + PAD];
    __shared__ float Bs[2][BK][BN + PAD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int64_t k_lo = (int64_t)blockIdx.z * a.k_slice;
    const int64_t k_hi = (k_lo + a.k_slice < a.K) ? k_lo + a.k_slice : a.K;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;

    f32x16 acc, tot;
    f64x4 dacc[2][2];
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc[v] = 0.0f; tot[v] = 0.0f; }
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int v = 0; v < 4; ++v) dacc[bi][bj][v] = 0.0;

    // A[BM x BK] and B[BK x BN] of one K step: four elements of each per thread; the thread -> element
    // map follows whichever stride is 1
    constexpr int PER = BM * BK / 256;
    float ra[PER], rb[PER];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int e = tid + u * 256;
            int mm, kk;
            if (a.a_cs == 1) { kk = e % BK; mm = e / BK; } else { mm = e % BM; kk = e / BM; }
            const int64_t m = m0 + mm, k = k0 + kk;
            ra[u] = (m < a.M && k < k_hi) ? a.A[m * a.a_rs + k * a.a_cs] : 0.0f;
            int nn;
            if (a.b_cs == 1) { nn = e % BN; kk = e / BN; } else { kk = e % BK; nn = e / BK; }
            const int64_t n = n0 + nn, kb = k0 + kk;
            rb[u] = (n < a.N && kb < k_hi) ? a.B[kb * a.b_rs + n * a.b_cs] : 0.0f;
        }
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int e = tid + u * 256;
            int mm, kk;
            if (a.a_cs == 1) { kk = e % BK; mm = e / BK; } else { mm = e % BM; kk = e / BM; }
            As[buf][kk][mm] = ra[u];
            int nn;
            if (a.b_cs == 1) { nn = e % BN; kk = e / BN; } else { kk = e % BK; nn = e / BK; }
            Bs[buf][kk][nn] = rb[u];
        }
    };

    int step = 0, buf = 0;
    if (k_lo < k_hi) {
        fetch(k_lo);
        park(0);
    }
    __syncthreads();
    for (int64_t k0 = k_lo; k0 < k_hi; k0 += BK, ++step) {
        if (!ACC64 && (step & 3) == 0 && step > 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) { tot[v] += acc[v]; acc[v] = 0.0f; }
        }
        const bool more = k0 + BK < k_hi;
        if (more) fetch(k0 + BK);
        if constexpr (ACC64) {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 4) {
                const int kr = kk + (lane >> 4), c = lane & 15;
                const double a0 = (double)As[buf][kr][wm + c], a1 = (double)As[buf][kr][wm + 16 + c];
                const double b0 = (double)Bs[buf][kr][wn + c], b1 = (double)Bs[buf][kr][wn + 16 + c];
                dacc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, dacc[0][0], 0, 0, 0);
                dacc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, dacc[0][1], 0, 0, 0);
                dacc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, dacc[1][0], 0, 0, 0);
                dacc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, dacc[1][1], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2) {
                float av = As[buf][kk + (lane >> 5)][wm + (lane & 31)];
                float bv = Bs[buf][kk + (lane >> 5)][wn + (lane & 31)];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
            }
        }
        if (more) park(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    float *C = a.C + (int64_t)blockIdx.z * a.c_slice;
    if constexpr (ACC64) {
        // 16x16 block: register v of lane l is element (4*v + l/16, l%16)
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int bj = 0; bj < 2; ++bj)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    gemm_store<EPI, double>(a, C, m0 + wm + 16 * bi + 4 * v + (lane >> 4),
                                            n0 + wn + 16 * bj + (lane & 15), dacc[bi][bj][v]);
    } else {
        // 32x32 block: register v of lane l is element (8*(v/4) + 4*(l/32) + v%4, l%32)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            gemm_store<EPI, float>(a, C, m0 + wm + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4),
                                   n0 + wn + (lane & 31), tot[v] + acc[v]);
    }
}

// out[n] (or out[m][n] summed over z slices) helpers ---------------------------------
// column sums of a [rows x cols] matrix in row slices: part[z][n] = sum of column n over the rows of
// slice z (rows visited in order); slice_sum_kernel then adds the slices.
__global__ __launch_bounds__(256) void colsum_kernel(const float *__restrict__ A, float *__restrict__ part,
                                                     int64_t rows, int cols, int64_t rows_per_slice)
{
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= cols) return;
    int64_t lo = (int64_t)blockIdx.y * rows_per_slice;
    int64_t hi = lo + rows_per_slice < rows ? lo + rows_per_slice : rows;
    // eight rows in flight; the eight running sums are combined in a fixed order
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int64_t m = lo;
    for (; m + 8 <= hi; m += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = A[(m + u) * cols + n];
#pragma unroll
        for (int u = 0; u < 8; ++u) s[u] += v[u];
    }
    for (; m < hi; ++m) s[0] += A[m * cols + n];
    part[(int64_t)blockIdx.y * cols + n] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
}

// sum of split-K slices: out[e] = sum_z part[z][e]
__global__ __launch_bounds__(256) void slice_sum_kernel(const float *__restrict__ part, float *__restrict__ out,
                                                        int64_t n, int slices)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    double s = 0.0;
    for (int z = 0; z < slices; ++z) s += (double)part[(int64_t)z * n + e];
    out[e] = (float)s;
}

// gE[i][f] = sum_c W1[f][c] * S[i][c],  S[i][c] = sum_t gpre[(i,t)][c].  One block per input: the
// column sums S (fp64, rows in order) go through LDS, then one thread per embedding feature.
__global__ __launch_bounds__(256) void embed_grad_kernel(const float *__restrict__ W1, const float *__restrict__ gpre,
                                                         float *__restrict__ gE, int n_in, int n_g, int d_feat,
                                                         int d_hid)
{
    extern __shared__ double colsum[];          // [d_hid]
    const int i = blockIdx.x;
    for (int c = threadIdx.x; c < d_hid; c += blockDim.x) {
        double s = 0.0;
        for (int t = 0; t < n_g; ++t) s += (double)gpre[((int64_t)i * n_g + t) * d_hid + c];
        colsum[c] = s;
    }
    __syncthreads();
    for (int f = threadIdx.x; f < d_feat; f += blockDim.x) {
        double s = 0.0;
        for (int c = 0; c < d_hid; ++c) s += (double)W1[(int64_t)f * d_hid + c] * colsum[c];
        gE[(int64_t)i * d_feat + f] = (float)s;
    }
}

// UKAN -> KAN export: every input uses the same first group; coef[i][m][j] = table row (m + shift)
__global__ __launch_bounds__(256) void fill_int_kernel(int32_t *__restrict__ p, int32_t v, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ __launch_bounds__(256) void table_rows_kernel(const float *__restrict__ table, float *__restrict__ coef,
                                                         int n_in, int table_rows, int coef_rows, int shift, int n_out)
{
    const int64_t at = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (at >= (int64_t)n_in * coef_rows * n_out) return;
    const int j = (int)(at % n_out);
    const int m = (int)((at / n_out) % coef_rows);
    const int i = (int)(at / ((int64_t)n_out * coef_rows));
    coef[at] = table[((int64_t)i * table_rows + m + shift) * n_out + j];
}

// ---- launchers ----------------------------------------------------------------------

hipError_t launch_fill_int(int32_t *p, int32_t v, int n, hipStream_t st)
{
    fill_int_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, v, n);
    return hipGetLastError();
}

hipError_t launch_table_rows(const float *table, float *coef, int n_in, int table_rows, int coef_rows, int shift,
                             int n_out, hipStream_t st)
{
    const int64_t n = (int64_t)n_in * coef_rows * n_out;
    prof::Timed tm("ukan_table_rows", st);
    table_rows_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(table, coef, n_in, table_rows, coef_rows, shift, n_out);
    return hipGetLastError();
}

hipError_t launch_slice_sum(const float *part, float *out, int64_t n, int slices, hipStream_t st);

hipError_t launch_group_index(const float *x, int32_t *cell, int32_t *grp, int32_t *off, int64_t n, float inv_h,
                              int K, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    prof::Timed tm("group_index", st);
    group_index_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(x, cell, grp, off, n, inv_h, K);
    return hipGetLastError();
}

hipError_t launch_range(const float *x, int64_t B, int n_in, float inv_h, int K, int32_t *cmin, int32_t *cmax,
                        int32_t *g_first, int32_t *n_groups, int32_t *cell_base, int32_t *summary, hipStream_t st)
{
    {
        prof::Timed tm("ukan_range", st);
        range_init_kernel<<<(n_in + 255) / 256, 256, 0, st>>>(cmin, cmax, n_in);
        int64_t strips = (B + 63) / 64;
        dim3 grid((unsigned)((n_in + 255) / 256), (unsigned)(strips < 1024 ? (strips < 1 ? 1 : strips) : 1024));
        range_kernel<<<grid, 256, 0, st>>>(x, cmin, cmax, B, n_in, inv_h);
        range_finalize_kernel<<<1, 256, 0, st>>>(cmin, cmax, g_first, n_groups, cell_base, summary, n_in, K);
    }
    return hipGetLastError();
}

hipError_t launch_span_check(const int32_t *summary, int provided, int32_t *overflow, hipStream_t st)
{
    span_check_kernel<<<1, 64, 0, st>>>(summary, provided, overflow);
    return hipGetLastError();
}

hipError_t launch_cg_hidden(const float *E, const float *W1, const float *b1, const int32_t *g_first, float *z,
                            float *pre, float *hid, int n_in, int n_g, int d_pe, int d_feat, int d_hid,
                            hipStream_t st)
{
    prof::Timed tm("cg_hidden", st);
    size_t lds = (size_t)(d_feat + d_pe) * sizeof(float);
    cg_hidden_kernel<<<(unsigned)(n_in * n_g), 64, lds, st>>>(E, W1, b1, g_first, z, pre, hid, n_g, d_pe, d_feat,
                                                             d_hid);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs &a, int epi, int slices, const char *family, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    prof::Timed tm(family, st);
    dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64), (unsigned)slices);
    switch (epi) {
    case EPI_PLAIN: gemm_mfma_kernel<EPI_PLAIN, true><<<grid, 256, 0, st>>>(a); break;
    case EPI_CG_OUT: gemm_mfma_kernel<EPI_CG_OUT, false><<<grid, 256, 0, st>>>(a); break;
    default: gemm_mfma_kernel<EPI_SILU_GRAD, true><<<grid, 256, 0, st>>>(a); break;
    }
    return hipGetLastError();
}

hipError_t launch_colsum(const float *A, float *part, float *out, int64_t rows, int cols, hipStream_t st)
{
    const int slices = colsum_slices(rows);
    const int64_t per = (rows + slices - 1) / slices;
    {
        prof::Timed tm("cg_colsum", st);
        colsum_kernel<<<dim3((cols + 255) / 256, slices), 256, 0, st>>>(A, part, rows, cols, per);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_slice_sum(part, out, cols, slices, st);
}

hipError_t launch_slice_sum(const float *part, float *out, int64_t n, int slices, hipStream_t st)
{
    prof::Timed tm("cg_slice_sum", st);
    slice_sum_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(part, out, n, slices);
    return hipGetLastError();
}

hipError_t launch_embed_grad(const float *W1, const float *gpre, float *gE, int n_in, int n_g, int d_feat,
                             int d_hid, hipStream_t st)
{
    prof::Timed tm("cg_embed_grad", st);
    embed_grad_kernel<<<n_in, 256, (size_t)d_hid * sizeof(double), st>>>(W1, gpre, gE, n_in, n_g, d_feat, d_hid);
    return hipGetLastError();
}

}  // namespace kan
