// Generic kernels of the local B-spline layer: they work for every shape the
// library accepts (any n_in, n_out, grid size, per-input cell offsets; degrees up to
// kMaxK - 1: 3 in the default build, 5 in the build of kan_generic_k5.hip) and are the
// fallback when no specialised kernel applies.
//
// Common mapping: lanes <-> outputs.  One wave owns T samples and a tile of
// 64*R outputs; the per-(sample, input) quantities (cell, window weights, base
// value) are wave-uniform, evaluated 64 pairs at a time with one pair per lane
// and then broadcast lane by lane into scalar registers, so the per-edge work is
// K multiply-adds whose coefficient operands are unit-stride across lanes.
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace KAN_NS {

// ---- helpers --------------------------------------------------------------

template <int R> struct VecOf;
template <> struct VecOf<1> { using type = float; };
template <> struct VecOf<2> { using type = float2; };
template <> struct VecOf<4> { using type = float4; };

template <int R>
__device__ __forceinline__ void load_vec(const float *p, float (&v)[R])
{
    if constexpr (R == 1) {
        v[0] = *p;
    } else if constexpr (R == 2) {
        float2 t = *reinterpret_cast<const float2 *>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
        float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
}

template <int R>
__device__ __forceinline__ void store_vec(float *p, const float (&v)[R])
{
    if constexpr (R == 1) {
        *p = v[0];
    } else if constexpr (R == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
    } else {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

// ---- interval index export --------------------------------------------------

__global__ void interval_index_kernel(const float *__restrict__ x, int32_t *__restrict__ idx, int64_t n,
                                      float lo, float inv_h)
{
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) {
        float t, d;
        idx[p] = interval_index(x[p], lo, inv_h, &t, &d);
    }
}

// ---- fold the per-edge spline scale into the coefficients -------------------
// cf[i][m][j] = w_s[i][j] * coef[i][m][j] for m < rows, and cf[i][rows][j] = w_b[i][j] (zero without
// a base term): afterwards the spline term costs K multiply-adds per edge with no separate scale,
// and one input's operands are one contiguous (rows + 1) x n_out block.
__global__ void fold_scale_kernel(const float *__restrict__ coef, const float *__restrict__ w_s,
                                  const float *__restrict__ w_b, float *__restrict__ cf, int n_in, int rows,
                                  int n_out)
{
    const int64_t per_in = (int64_t)(rows + 1) * n_out;
    const int64_t total = (int64_t)n_in * per_in;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < total;
         p += (int64_t)gridDim.x * blockDim.x) {
        const int i = (int)(p / per_in);
        const int64_t rem = p - (int64_t)i * per_in;
        const int m = (int)(rem / n_out), j = (int)(rem % n_out);
        float v;
        if (m < rows)
            v = coef[((int64_t)i * rows + m) * n_out + j] * w_s[(int64_t)i * n_out + j];
        else
            v = w_b ? w_b[(int64_t)i * n_out + j] : 0.0f;
        cf[p] = v;
    }
}

// ---- forward ---------------------------------------------------------------
// grid.x = batch tiles of 4*T samples, grid.y = output tiles of 64*R.
template <int R, int T>
__global__ __launch_bounds__(256) void forward_generic_kernel(SplineGeom g, const float *__restrict__ x,
                                                              const float *__restrict__ cf,
                                                              const float *__restrict__ w_b,
                                                              float *__restrict__ y, int64_t B)
{
    constexpr int IPV = kWave / T;      // inputs covered by one vector evaluation
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b0 = ((int64_t)blockIdx.x * 4 + wave) * T;
    if (b0 >= B) return;                // whole wave out of range (uniform)
    const int j = blockIdx.y * (kWave * R) + lane * R;
    const bool j_ok = j < g.n_out;      // n_out is a multiple of R
    const int jc = j_ok ? j : 0;

    // two-level sum over the inputs: `acc` collects kFoldInputs inputs, then is folded into
    // `tot`; keeps the rounding error of a long fp32 sum well inside the tolerance
    constexpr int kFoldInputs = 32;
    float acc[T][R], tot[T][R];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int r = 0; r < R; ++r) { acc[t][r] = 0.0f; tot[t][r] = 0.0f; }

    const int my_t = lane % T, my_ii = lane / T;
    const int64_t my_b = (b0 + my_t < B) ? b0 + my_t : B - 1;

    for (int i0 = 0; i0 < g.n_in; i0 += IPV) {
        if (i0 % kFoldInputs == 0 && i0 > 0) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int r = 0; r < R; ++r) { tot[t][r] += acc[t][r]; acc[t][r] = 0.0f; }
        }
        const int my_i = i0 + my_ii;
        const bool i_ok = my_i < g.n_in;
        const int ic = i_ok ? my_i : g.n_in - 1;
        Pair p = pair_eval<false>(x[my_b * g.n_in + ic], g, ic);
        if (!i_ok) { p.cell = -kMaxK; p.base = 0.0f; }

        const int n_ii = (g.n_in - i0 < IPV) ? g.n_in - i0 : IPV;
        for (int ii = 0; ii < n_ii; ++ii) {
            const float *slab = cf + (int64_t)(i0 + ii) * g.slab_rows * g.n_out + jc;
            float wb[R];
#pragma unroll
            for (int r = 0; r < R; ++r) wb[r] = 0.0f;
            if (g.base_act) load_vec<R>(w_b + (int64_t)(i0 + ii) * g.n_out + jc, wb);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int src = ii * T + t;
                // no branch on "window outside the table": those weights are zero and the rows are
                // clamped, so the loads of all T samples can be in flight together
                const int cell = lane_i(p.cell, src);
                float c[kMaxK][R];
#pragma unroll
                for (int s = 0; s < kMaxK; ++s)
                    load_vec<R>(slab + (int64_t)clampi(cell + s, 0, g.rows - 1) * g.n_out, c[s]);
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) {
                    const float ws = lane_f(p.w[s], src);
#pragma unroll
                    for (int r = 0; r < R; ++r) acc[t][r] = fmaf(ws, c[s][r], acc[t][r]);
                }
                if (g.base_act) {
                    const float bs = lane_f(p.base, src);
#pragma unroll
                    for (int r = 0; r < R; ++r) acc[t][r] = fmaf(bs, wb[r], acc[t][r]);
                }
            }
        }
    }
    if (j_ok) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
#pragma unroll
            for (int r = 0; r < R; ++r) tot[t][r] += acc[t][r];
            if (b0 + t < B) store_vec<R>(y + (b0 + t) * g.n_out + j, tot[t]);
        }
    }
}

// ---- backward: dL/dx ---------------------------------------------------------
// One wave owns T samples and walks over every output tile; per pair it forms the
// per-lane partial  q = sum_r gy_r * (sum_s dw_s * cf_s[r] + dbase * w_b[r])  and the
// 64 partial vectors of one evaluation round are reduced together by a butterfly
// that ends with lane p holding the total of pair p, which is the lane that
// evaluated the pair and now stores gx for it.
template <int N>
__device__ __forceinline__ void butterfly_step(float (&q)[kWave], int lane)
{
    // q[0..2N) -> q[0..N): lanes with bit N clear keep the low half, the others the high half
    const bool up = (lane & N) != 0;
#pragma unroll
    for (int m = 0; m < N; ++m) {
        float keep = up ? q[m + N] : q[m];
        float send = up ? q[m] : q[m + N];
        q[m] = keep + __shfl_xor(send, N, kWave);
    }
}

template <int R, int T>
__global__ __launch_bounds__(256) void dx_generic_kernel(SplineGeom g, const float *__restrict__ x,
                                                         const float *__restrict__ cf,
                                                         const float *__restrict__ w_b,
                                                         const float *__restrict__ gy,
                                                         float *__restrict__ gx, int64_t B)
{
    constexpr int IPV = kWave / T;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b0 = ((int64_t)blockIdx.x * 4 + wave) * T;
    if (b0 >= B) return;
    const int my_t = lane % T, my_ii = lane / T;
    const int64_t my_b = (b0 + my_t < B) ? b0 + my_t : B - 1;
    const int n_jt = (g.n_out + kWave * R - 1) / (kWave * R);

    for (int i0 = 0; i0 < g.n_in; i0 += IPV) {
        const int my_i = i0 + my_ii;
        const bool i_ok = my_i < g.n_in;
        const int ic = i_ok ? my_i : g.n_in - 1;
        Pair p = pair_eval<true>(x[my_b * g.n_in + ic], g, ic);
        if (!i_ok) { p.cell = -kMaxK; p.dbase = 0.0f; }

        float q[kWave];
#pragma unroll
        for (int m = 0; m < kWave; ++m) q[m] = 0.0f;

        for (int jt = 0; jt < n_jt; ++jt) {
            const int j = jt * (kWave * R) + lane * R;
            const bool j_ok = j < g.n_out;
            const int jc = j_ok ? j : 0;
            float gyv[T][R];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int64_t b = (b0 + t < B) ? b0 + t : B - 1;
                load_vec<R>(gy + b * g.n_out + jc, gyv[t]);
                if (!j_ok) {
#pragma unroll
                    for (int r = 0; r < R; ++r) gyv[t][r] = 0.0f;
                }
            }
#pragma unroll
            for (int ii = 0; ii < IPV; ++ii) {
                if (i0 + ii < g.n_in) {
                    const float *slab = cf + (int64_t)(i0 + ii) * g.slab_rows * g.n_out + jc;
                    float wb[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) wb[r] = 0.0f;
                    if (g.base_act) load_vec<R>(w_b + (int64_t)(i0 + ii) * g.n_out + jc, wb);
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        const int src = ii * T + t;
                        const int cell = lane_i(p.cell, src);
                        float d[R];
#pragma unroll
                        for (int r = 0; r < R; ++r) d[r] = 0.0f;
                        if (cell > -kMaxK && cell < g.rows) {
                            float c[kMaxK][R];
#pragma unroll
                            for (int s = 0; s < kMaxK; ++s)
                                load_vec<R>(slab + (int64_t)clampi(cell + s, 0, g.rows - 1) * g.n_out, c[s]);
#pragma unroll
                            for (int s = 0; s < kMaxK; ++s) {
                                const float dws = lane_f(p.dw[s], src);
#pragma unroll
                                for (int r = 0; r < R; ++r) d[r] = fmaf(dws, c[s][r], d[r]);
                            }
                        }
                        if (g.base_act) {
                            const float dbs = lane_f(p.dbase, src);
#pragma unroll
                            for (int r = 0; r < R; ++r) d[r] = fmaf(dbs, wb[r], d[r]);
                        }
#pragma unroll
                        for (int r = 0; r < R; ++r) q[src] = fmaf(gyv[t][r], d[r], q[src]);
                    }
                }
            }
        }
        butterfly_step<32>(q, lane);
        butterfly_step<16>(q, lane);
        butterfly_step<8>(q, lane);
        butterfly_step<4>(q, lane);
        butterfly_step<2>(q, lane);
        butterfly_step<1>(q, lane);
        if (i_ok && b0 + my_t < B) gx[(b0 + my_t) * g.n_in + my_i] = q[0];
    }
}

// ---- backward: parameter gradients -------------------------------------------
// Stage 1.  One wave owns input i, a tile of 64*R outputs, one block of kRowBlock coefficient rows
// and one chunk of the batch, and keeps
//   acc[m][j] = sum_{b in chunk} gy[b][j] * N_{m - cell(b,i)}(u(b,i))      (m in its row block)
// in LDS that only this wave touches.  Samples are visited in index order and every row has exactly
// one owner, so the sum order is fixed.  Samples whose window misses the row block are skipped with
// a scalar test, which is what keeps large grids cheap: the LDS footprint per wave is a row block,
// not the whole slab, so many waves fit on a CU.  The raw sums go to part_c[chunk][i][m][j]; the
// base-term sums  sum_b gy[b][j] * silu(x[b][i])  are taken by the block that owns the sample's
// clamped cell and go to part_b[chunk * n_row_blocks + block][i][j].
constexpr int kRowBlock = 16;

template <int R>
__global__ __launch_bounds__(64) void dparam_generic_kernel(SplineGeom g, const float *__restrict__ x,
                                                            const float *__restrict__ gy,
                                                            float *__restrict__ part_c,
                                                            float *__restrict__ part_b, int64_t B,
                                                            int64_t chunk_len, int n_jt)
{
    constexpr int TJ = kWave * R;
    __shared__ float acc[kRowBlock * TJ];
    const int lane = threadIdx.x;
    // grid.x carries (row block, output tile): it may exceed the 65535 limit of grid.y for long tables
    const int i = blockIdx.y;
    const int jt = blockIdx.x % n_jt, rb = blockIdx.x / n_jt;
    const int n_rb = gridDim.x / n_jt;
    const int lo = rb * kRowBlock;
    const int hi = (lo + kRowBlock < g.rows) ? lo + kRowBlock : g.rows;
    const int j = jt * TJ + lane * R;
    const bool j_ok = j < g.n_out;
    const int jc = j_ok ? j : 0;
    const int64_t b_lo = (int64_t)blockIdx.z * chunk_len;
    const int64_t b_hi = (b_lo + chunk_len < B) ? b_lo + chunk_len : B;

    for (int m = 0; m < kRowBlock; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[m * TJ + lane * R + r] = 0.0f;
    // the base sums go in two levels (accb is folded into accb_hi every 256 samples) so that a chunk of a
    // thousand O(1) terms keeps fp32 accuracy
    float accb[R], accb_hi[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { accb[r] = 0.0f; accb_hi[r] = 0.0f; }

    for (int64_t b0 = b_lo; b0 < b_hi; b0 += kWave) {
        if (((b0 - b_lo) & 255) == 0) {
#pragma unroll
            for (int r = 0; r < R; ++r) { accb_hi[r] += accb[r]; accb[r] = 0.0f; }
        }
        const int64_t my_b = (b0 + lane < b_hi) ? b0 + lane : b_hi - 1;
        Pair p = pair_eval<false>(x[my_b * g.n_in + i], g, i);
        const int n_b = (b_hi - b0 < kWave) ? (int)(b_hi - b0) : kWave;
        for (int t = 0; t < n_b; ++t) {
            const int cell = lane_i(p.cell, t);
            const int owner = clampi(cell, 0, g.rows - 1);
            const bool touches = cell + kMaxK > lo && cell < hi;
            const bool owns = owner >= lo && owner < hi;
            if (!(touches || (owns && part_b))) continue;          // uniform
            float gv[R];
            load_vec<R>(gy + (b0 + t) * g.n_out + jc, gv);
            if (touches) {
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) {
                    const int m = cell + s;
                    if (m >= lo && m < hi) {                        // uniform
                        const float ws = lane_f(p.w[s], t);
                        float *row = acc + (m - lo) * TJ + lane * R;
#pragma unroll
                        for (int r = 0; r < R; ++r) row[r] = fmaf(ws, gv[r], row[r]);
                    }
                }
            }
            if (owns && part_b) {
                const float bs = lane_f(p.base, t);
#pragma unroll
                for (int r = 0; r < R; ++r) accb[r] = fmaf(bs, gv[r], accb[r]);
            }
        }
    }
    if (!j_ok) return;
    float *pc = part_c + ((int64_t)blockIdx.z * g.n_in + i) * g.rows * g.n_out + j;
    for (int m = lo; m < hi; ++m) {
        float a[R];
#pragma unroll
        for (int r = 0; r < R; ++r) a[r] = acc[(m - lo) * TJ + lane * R + r];
        store_vec<R>(pc + (int64_t)m * g.n_out, a);
    }
    if (part_b) {
#pragma unroll
        for (int r = 0; r < R; ++r) accb[r] += accb_hi[r];
        store_vec<R>(part_b + (((int64_t)blockIdx.z * n_rb + rb) * g.n_in + i) * g.n_out + j, accb);
    }
}

// Stage 2.  Sum the partial sums (n_chunks slabs for the coefficient rows, n_slices_b slices for the
// base term) in order with an fp64 accumulator, so that the long batch sum costs no accuracy, and
// turn them into the three gradients:
//   gcoef = w_s * acc,   gw_s = sum_m coef * acc,   gw_b = base sums.
// 2a: one thread per table element (input, row, output): the chunk sum, gcoef, and the summed
//     acc written back over chunk 0 of part_c for 2b.
__global__ __launch_bounds__(256) void dparam_reduce_rows_kernel(float *__restrict__ part_c,
                                                                 const float *__restrict__ w_s,
                                                                 float *__restrict__ gcoef, int n_in, int rows,
                                                                 int n_out, int n_chunks, int keep_sum)
{
    const int64_t slab = (int64_t)n_in * rows * n_out;
    const int64_t at = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (at >= slab) return;
    double a = 0.0;
    for (int c = 0; c < n_chunks; ++c) a += (double)part_c[c * slab + at];
    const int j = (int)(at % n_out);
    const int i = (int)(at / ((int64_t)rows * n_out));
    if (gcoef) gcoef[at] = (float)((double)w_s[(int64_t)i * n_out + j] * a);
    if (keep_sum) part_c[at] = (float)a;
}

// 2a for n_out % 4 == 0: four consecutive outputs per thread, 16-byte accesses.
__global__ __launch_bounds__(256) void dparam_reduce_rows4_kernel(float *__restrict__ part_c,
                                                                  const float *__restrict__ w_s,
                                                                  float *__restrict__ gcoef, int n_in, int rows,
                                                                  int n_out, int n_chunks, int keep_sum)
{
    const int64_t slab = (int64_t)n_in * rows * n_out;
    const int64_t at = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (at >= slab) return;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    int c = 0;
    for (; c + 4 <= n_chunks; c += 4) {          // four loads in flight, summed in chunk order
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4 *>(part_c + (c + u) * slab + at);
#pragma unroll
        for (int u = 0; u < 4; ++u) { a0 += (double)v[u].x; a1 += (double)v[u].y; a2 += (double)v[u].z; a3 += (double)v[u].w; }
    }
    for (; c < n_chunks; ++c) {
        const float4 v = *reinterpret_cast<const float4 *>(part_c + c * slab + at);
        a0 += (double)v.x; a1 += (double)v.y; a2 += (double)v.z; a3 += (double)v.w;
    }
    const int j = (int)(at % n_out);
    const int i = (int)(at / ((int64_t)rows * n_out));
    if (gcoef) {
        const float4 w = *reinterpret_cast<const float4 *>(w_s + (int64_t)i * n_out + j);
        *reinterpret_cast<float4 *>(gcoef + at) = make_float4((float)((double)w.x * a0), (float)((double)w.y * a1),
                                                              (float)((double)w.z * a2), (float)((double)w.w * a3));
    }
    if (keep_sum) *reinterpret_cast<float4 *>(part_c + at) = make_float4((float)a0, (float)a1, (float)a2, (float)a3);
}

// 2b: gw_s from the summed acc, gw_b from the base slices.  grid (n_in, ceil(n_out / 64), n_rs), 256
// threads: lane <-> output, the four waves split the rows (or slices) of the block's row slice
// between them and their fp64 partial sums are added in wave order.  With n_rs > 1 row slices the
// block sums go to slice_sums[rs][i][j] (fp64) and dparam_reduce_edges_final_kernel adds them up in
// slice order; with one slice the result is written directly.
__global__ __launch_bounds__(256) void dparam_reduce_edges_kernel(const float *__restrict__ acc_sum,
                                                                  const float *__restrict__ part_b,
                                                                  const float *__restrict__ coef,
                                                                  float *__restrict__ gw_s, float *__restrict__ gw_b,
                                                                  double *__restrict__ slice_sums, int n_in, int rows,
                                                                  int n_out, int n_slices_b)
{
    __shared__ double part[2][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = blockIdx.x, j = blockIdx.y * 64 + lane;
    const int n_rs = gridDim.z, rs = blockIdx.z;
    const int per = (rows + n_rs - 1) / n_rs;
    const int m_lo = rs * per, m_hi = (m_lo + per < rows) ? m_lo + per : rows;
    const bool ok = j < n_out;
    const int jc = ok ? j : 0;
    double s = 0.0, a = 0.0;
    if (gw_s) {
        const float *cp = coef + (int64_t)i * rows * n_out + jc, *ap = acc_sum + (int64_t)i * rows * n_out + jc;
        int m = m_lo + wave;
        for (; m + 12 < m_hi; m += 16) {        // four rows of this wave in flight
            float cv[4], av[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { cv[u] = cp[(int64_t)(m + 4 * u) * n_out]; av[u] = ap[(int64_t)(m + 4 * u) * n_out]; }
#pragma unroll
            for (int u = 0; u < 4; ++u) s += (double)cv[u] * (double)av[u];
        }
        for (; m < m_hi; m += 4) s += (double)cp[(int64_t)m * n_out] * (double)ap[(int64_t)m * n_out];
    }
    if (gw_b && part_b && rs == 0) {
        const float *bp = part_b + (int64_t)i * n_out + jc;
        for (int c = wave; c < n_slices_b; c += 4) a += (double)bp[(int64_t)c * n_in * n_out];
    }
    part[0][wave][lane] = s;
    part[1][wave][lane] = a;
    __syncthreads();
    if (wave == 0 && ok) {
        const int64_t e = (int64_t)i * n_out + j;
        const double ss = ((part[0][0][lane] + part[0][1][lane]) + part[0][2][lane]) + part[0][3][lane];
        if (gw_s) {
            if (n_rs > 1) slice_sums[(int64_t)rs * n_in * n_out + e] = ss;
            else gw_s[e] = (float)ss;
        }
        // no base term: the gradient is identically zero
        if (gw_b && rs == 0) gw_b[e] = (float)(((part[1][0][lane] + part[1][1][lane]) + part[1][2][lane]) + part[1][3][lane]);
    }
}

__global__ __launch_bounds__(256) void dparam_reduce_edges_final_kernel(const double *__restrict__ slice_sums,
                                                                        float *__restrict__ gw_s, int64_t edges,
                                                                        int n_rs)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= edges) return;
    double s = 0.0;
    for (int r = 0; r < n_rs; ++r) s += slice_sums[(int64_t)r * edges + e];
    gw_s[e] = (float)s;
}

// ---- launchers -------------------------------------------------------------

static int pick_r(int n_out)
{
    if (n_out % 4 == 0 && n_out >= 256) return 4;
    if (n_out % 2 == 0 && n_out >= 128) return 2;
    return 1;
}

hipError_t launch_interval_index(const float *x, int32_t *idx, int64_t n, float lo, float inv_h,
                                 hipStream_t st)
{
    if (n == 0) return hipSuccess;
    unsigned blocks = (unsigned)((n + 255) / 256);
    prof::Timed tm("interval_index", st);
    interval_index_kernel<<<blocks, 256, 0, st>>>(x, idx, n, lo, inv_h);
    return hipGetLastError();
}

hipError_t launch_fold_scale(const float *coef, const float *w_s, const float *w_b, float *cf, int n_in, int rows,
                             int n_out, hipStream_t st)
{
    int64_t total = (int64_t)n_in * (rows + 1) * n_out;
    int64_t want = (total + 255) / 256;
    unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
    prof::Timed tm("fold_scale", st);
    fold_scale_kernel<<<blocks, 256, 0, st>>>(coef, w_s, w_b, cf, n_in, rows, n_out);
    return hipGetLastError();
}

template <int R, int T>
static hipError_t forward_rt(const SplineGeom &g, const float *x, const float *cf, const float *w_b, float *y,
                             int64_t B, hipStream_t st)
{
    dim3 grid((unsigned)((B + 4 * T - 1) / (4 * T)), (unsigned)((g.n_out + 64 * R - 1) / (64 * R)));
    prof::Timed tm("forward_generic", st);
    forward_generic_kernel<R, T><<<grid, 256, 0, st>>>(g, x, cf, w_b, y, B);
    return hipGetLastError();
}

// samples per wave: as many as still leave the chip about four waves per SIMD (the kernel lives on
// loads in flight), between 2 and 8 (16 for the one- and two-output-per-lane variants)
template <int R>
static hipError_t forward_r(const SplineGeom &g, const float *x, const float *cf, const float *w_b, float *y,
                            int64_t B, hipStream_t st)
{
    const int64_t tiles = (g.n_out + 64 * R - 1) / (64 * R);
    auto waves = [&](int t) { return (B + t - 1) / t * tiles; };
    if constexpr (R != 4) {
        if (waves(16) >= 4096) return forward_rt<R, 16>(g, x, cf, w_b, y, B, st);
    }
    if (waves(8) >= 4096) return forward_rt<R, 8>(g, x, cf, w_b, y, B, st);
    if (waves(4) >= 4096) return forward_rt<R, 4>(g, x, cf, w_b, y, B, st);
    return forward_rt<R, 2>(g, x, cf, w_b, y, B, st);
}

hipError_t launch_forward_generic(const SplineGeom &g, const float *x, const float *cf, const float *w_b,
                                  float *y, int64_t B, hipStream_t st)
{
    switch (pick_r(g.n_out)) {
    case 4: return forward_r<4>(g, x, cf, w_b, y, B, st);
    case 2: return forward_r<2>(g, x, cf, w_b, y, B, st);
    default: return forward_r<1>(g, x, cf, w_b, y, B, st);
    }
}

template <int R>
static hipError_t dx_r(const SplineGeom &g, const float *x, const float *cf, const float *w_b, const float *gy,
                       float *gx, int64_t B, hipStream_t st)
{
    constexpr int T = 8;
    dim3 grid((unsigned)((B + 4 * T - 1) / (4 * T)));
    prof::Timed tm("dx_generic", st);
    dx_generic_kernel<R, T><<<grid, 256, 0, st>>>(g, x, cf, w_b, gy, gx, B);
    return hipGetLastError();
}

hipError_t launch_dx_generic(const SplineGeom &g, const float *x, const float *cf, const float *w_b,
                             const float *gy, float *gx, int64_t B, hipStream_t st)
{
    switch (pick_r(g.n_out)) {
    case 4: return dx_r<4>(g, x, cf, w_b, gy, gx, B, st);
    case 2: return dx_r<2>(g, x, cf, w_b, gy, gx, B, st);
    default: return dx_r<1>(g, x, cf, w_b, gy, gx, B, st);
    }
}

int dparam_generic_row_blocks(int rows) { return (rows + kRowBlock - 1) / kRowBlock; }

hipError_t launch_dparam_generic(const SplineGeom &g, const float *x, const float *gy, float *part_c,
                                 float *part_b, int64_t B, int n_chunks, int64_t chunk_len, hipStream_t st)
{
    const int R = pick_r(g.n_out);
    const int n_jt = (g.n_out + 64 * R - 1) / (64 * R);
    const int n_rb = dparam_generic_row_blocks(g.rows);
    if (g.n_in > 65535 || n_chunks > 65535) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)(n_jt * n_rb), (unsigned)g.n_in, (unsigned)n_chunks);
    prof::Timed tm("dparam_generic", st);
    switch (R) {
    case 4: dparam_generic_kernel<4><<<grid, 64, 0, st>>>(g, x, gy, part_c, part_b, B, chunk_len, n_jt); break;
    case 2: dparam_generic_kernel<2><<<grid, 64, 0, st>>>(g, x, gy, part_c, part_b, B, chunk_len, n_jt); break;
    default: dparam_generic_kernel<1><<<grid, 64, 0, st>>>(g, x, gy, part_c, part_b, B, chunk_len, n_jt); break;
    }
    return hipGetLastError();
}

size_t dparam_reduce_tail_bytes(int n_in, int n_out) { return 64 * (size_t)n_in * n_out * sizeof(double) + 8; }

hipError_t launch_dparam_reduce(float *part_c, const float *part_b, const float *coef, const float *w_s,
                                float *gcoef, float *gw_s, float *gw_b, int n_in, int rows, int n_out,
                                int n_chunks, int n_slices_b, hipStream_t st, size_t tail_scratch)
{
    const int64_t slab = (int64_t)n_in * rows * n_out, edges = (int64_t)n_in * n_out;
    const bool vec4 = n_out % 4 == 0 && ((uintptr_t)part_c % 16) == 0 && (!gcoef || ((uintptr_t)gcoef % 16) == 0) &&
                      ((uintptr_t)w_s % 16) == 0;
    if (gcoef || gw_s) {
        prof::Timed tm("dparam_reduce", st);
        if (vec4)
            dparam_reduce_rows4_kernel<<<(unsigned)((slab / 4 + 255) / 256), 256, 0, st>>>(part_c, w_s, gcoef, n_in, rows,
                                                                                     n_out, n_chunks, gw_s ? 1 : 0);
        else
            dparam_reduce_rows_kernel<<<(unsigned)((slab + 255) / 256), 256, 0, st>>>(part_c, w_s, gcoef, n_in, rows,
                                                                                    n_out, n_chunks, gw_s ? 1 : 0);
    }
    if (gw_s || gw_b) {
        // Long tables: the row sum behind gw_s is cut into row slices.  Their fp64 block sums live in
        // the second chunk's partial slab, which is dead once the chunks have been summed (or in the
        // scratch the caller left behind a single slab).
        int n_rs = 1;
        double *slice_sums = nullptr;
        if (gw_s && (n_chunks >= 2 || tail_scratch >= dparam_reduce_tail_bytes(n_in, n_out)) && rows >= 512) {
            n_rs = rows / 256 < 64 ? rows / 256 : 64;
            slice_sums = (double *)(((uintptr_t)(part_c + slab) + 7) & ~(uintptr_t)7);
        }
        prof::Timed te("dparam_reduce_edges", st);
        dparam_reduce_edges_kernel<<<dim3((unsigned)n_in, (unsigned)((n_out + 63) / 64), (unsigned)n_rs), 256, 0, st>>>(
            part_c, part_b, coef, gw_s, gw_b, slice_sums, n_in, rows, n_out, n_slices_b);
        if (n_rs > 1)
            dparam_reduce_edges_final_kernel<<<(unsigned)((edges + 255) / 256), 256, 0, st>>>(slice_sums, gw_s, edges,
                                                                                            n_rs);
    }
    return hipGetLastError();
}

}  // namespace KAN_NS
