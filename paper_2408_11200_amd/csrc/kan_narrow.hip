// Kernels for narrow layers (at most 16 outputs), e.g. the 5 -> 1 layer of a small KAN or the last
// layer of a regression stack.  With so few outputs the lanes <-> outputs mapping of the other
// kernels would leave most of a wave idle, so here lanes <-> samples (forward, dL/dx: every lane
// evaluates its own pair and gathers its own window; nothing is reduced across lanes) and
// lanes <-> coefficient rows (parameter gradients: a wave owns 64 rows of one input and visits the
// samples in order, so the reduction stays atomic-free and bit-reproducible).
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace kan {

// ---- forward ------------------------------------------------------------------------------
template <int NO>
__global__ __launch_bounds__(256) void forward_narrow_kernel(SplineGeom g, const float *__restrict__ x,
                                                             const float *__restrict__ cf,
                                                             const float *__restrict__ w_b, float *__restrict__ y,
                                                             int64_t B)
{
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    float acc[NO];
#pragma unroll
    for (int j = 0; j < NO; ++j) acc[j] = 0.0f;
    for (int i = 0; i < g.n_in; ++i) {
        const Pair p = pair_eval<false>(x[b * g.n_in + i], g, i);
        const float *slab = cf + (int64_t)i * g.slab_rows * g.n_out;
#pragma unroll
        for (int s = 0; s < kMaxK; ++s) {
            const float *row = slab + (int64_t)clampi(p.cell + s, 0, g.rows - 1) * g.n_out;
#pragma unroll
            for (int j = 0; j < NO; ++j)
                if (j < g.n_out) acc[j] = fmaf(p.w[s], row[j], acc[j]);
        }
        if (g.base_act) {
            const float *wb = w_b + (int64_t)i * g.n_out;
#pragma unroll
            for (int j = 0; j < NO; ++j)
                if (j < g.n_out) acc[j] = fmaf(p.base, wb[j], acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < NO; ++j)
        if (j < g.n_out) y[b * g.n_out + j] = acc[j];
}

// ---- backward: dL/dx ------------------------------------------------------------------------
template <int NO>
__global__ __launch_bounds__(256) void dx_narrow_kernel(SplineGeom g, const float *__restrict__ x,
                                                        const float *__restrict__ cf, const float *__restrict__ w_b,
                                                        const float *__restrict__ gy, float *__restrict__ gx,
                                                        int64_t B)
{
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    float gv[NO];
#pragma unroll
    for (int j = 0; j < NO; ++j) gv[j] = (j < g.n_out) ? gy[b * g.n_out + j] : 0.0f;
    for (int i = 0; i < g.n_in; ++i) {
        const Pair p = pair_eval<true>(x[b * g.n_in + i], g, i);
        const float *slab = cf + (int64_t)i * g.slab_rows * g.n_out;
        float acc = 0.0f;
#pragma unroll
        for (int s = 0; s < kMaxK; ++s) {
            const float *row = slab + (int64_t)clampi(p.cell + s, 0, g.rows - 1) * g.n_out;
            float ts = 0.0f;
#pragma unroll
            for (int j = 0; j < NO; ++j)
                if (j < g.n_out) ts = fmaf(gv[j], row[j], ts);
            acc = fmaf(p.dw[s], ts, acc);
        }
        if (g.base_act) {
            const float *wb = w_b + (int64_t)i * g.n_out;
            float tb = 0.0f;
#pragma unroll
            for (int j = 0; j < NO; ++j)
                if (j < g.n_out) tb = fmaf(gv[j], wb[j], tb);
            acc = fmaf(p.dbase, tb, acc);
        }
        gx[b * g.n_in + i] = acc;
    }
}

// ---- backward: parameter gradients, stage 1 ----------------------------------------------------
// grid (n_in, ceil(rows / 64), chunks), one wave per block.  Lane l owns coefficient row lo + l of the
// input and accumulates  acc[j] = sum_b gy[b][j] * N_{row - cell(b)}(u(b))  over the chunk in
// registers.  Samples are evaluated 64 at a time (one per lane) and then visited one by one with
// their cell and weights broadcast; a sample whose window misses the wave's rows is skipped by a
// scalar test.  Output as for the generic kernel: part_c[chunk][i][row][j] and the base-term sums
// (taken by the wave that owns the sample's clamped cell) part_b[chunk * blocks + block][i][j].
template <int NO>
__global__ __launch_bounds__(64) void dparam_narrow_kernel(SplineGeom g, const float *__restrict__ x,
                                                           const float *__restrict__ gy,
                                                           float *__restrict__ part_c, float *__restrict__ part_b,
                                                           int64_t B, int64_t chunk_len)
{
    const int lane = threadIdx.x;
    const int i = blockIdx.x;
    const int lo = blockIdx.y * kWave;
    const int hi = (lo + kWave < g.rows) ? lo + kWave : g.rows;
    const int row = lo + lane;
    const int64_t b_lo = (int64_t)blockIdx.z * chunk_len;
    const int64_t b_hi = (b_lo + chunk_len < B) ? b_lo + chunk_len : B;

    float acc[NO], accb[NO];
#pragma unroll
    for (int j = 0; j < NO; ++j) { acc[j] = 0.0f; accb[j] = 0.0f; }

    for (int64_t b0 = b_lo; b0 < b_hi; b0 += kWave) {
        const int64_t my_b = (b0 + lane < b_hi) ? b0 + lane : b_hi - 1;
        const Pair p = pair_eval<false>(x[my_b * g.n_in + i], g, i);
        const int n_b = (b_hi - b0 < kWave) ? (int)(b_hi - b0) : kWave;
        for (int t = 0; t < n_b; ++t) {
            const int cell = lane_i(p.cell, t);
            const int owner = clampi(cell, 0, g.rows - 1);
            const bool touches = cell + kMaxK > lo && cell < hi;
            const bool owns = owner >= lo && owner < hi && part_b != nullptr;
            if (!(touches || owns)) continue;                       // uniform
            const float *gr = gy + (b0 + t) * g.n_out;              // uniform address: scalar loads
            if (touches) {
                const int s = row - cell;                           // which window slot this lane's row is
                float w = 0.0f;
#pragma unroll
                for (int q = 0; q < kMaxK; ++q) w = (s == q) ? lane_f(p.w[q], t) : w;
#pragma unroll
                for (int j = 0; j < NO; ++j)
                    if (j < g.n_out) acc[j] = fmaf(w, gr[j], acc[j]);
            }
            if (owns) {
                const float bs = lane_f(p.base, t);
#pragma unroll
                for (int j = 0; j < NO; ++j)
                    if (j < g.n_out) accb[j] = fmaf(bs, gr[j], accb[j]);
            }
        }
    }
    if (row < hi) {
        float *pc = part_c + (((int64_t)blockIdx.z * g.n_in + i) * g.rows + row) * g.n_out;
#pragma unroll
        for (int j = 0; j < NO; ++j)
            if (j < g.n_out) pc[j] = acc[j];
    }
    if (part_b && lane == 0) {      // accb is the same in every lane
        float *pb = part_b + (((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * g.n_in + i) * g.n_out;
#pragma unroll
        for (int j = 0; j < NO; ++j)
            if (j < g.n_out) pb[j] = accb[j];
    }
}

// ---- launch -------------------------------------------------------------------------------------

int narrow_applicable(const SplineGeom &g) { return g.n_out <= 16 ? 1 : 0; }
int dparam_narrow_row_blocks(int rows) { return (rows + kWave - 1) / kWave; }

#define KAN_NARROW_DISPATCH(n_out, CALL)        \
    if ((n_out) <= 1) { CALL(1); }               \
    else if ((n_out) <= 2) { CALL(2); }          \
    else if ((n_out) <= 4) { CALL(4); }          \
    else if ((n_out) <= 8) { CALL(8); }          \
    else { CALL(16); }

hipError_t launch_forward_narrow(const SplineGeom &g, const float *x, const float *cf, const float *w_b, float *y,
                                 int64_t B, hipStream_t st)
{
    prof::Timed tm("forward_narrow", st);
    const unsigned blocks = (unsigned)((B + 255) / 256);
#define CALL(N) forward_narrow_kernel<N><<<blocks, 256, 0, st>>>(g, x, cf, w_b, y, B)
    KAN_NARROW_DISPATCH(g.n_out, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_dx_narrow(const SplineGeom &g, const float *x, const float *cf, const float *w_b, const float *gy,
                            float *gx, int64_t B, hipStream_t st)
{
    prof::Timed tm("dx_narrow", st);
    const unsigned blocks = (unsigned)((B + 255) / 256);
#define CALL(N) dx_narrow_kernel<N><<<blocks, 256, 0, st>>>(g, x, cf, w_b, gy, gx, B)
    KAN_NARROW_DISPATCH(g.n_out, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_dparam_narrow(const SplineGeom &g, const float *x, const float *gy, float *part_c, float *part_b,
                                int64_t B, int n_chunks, int64_t chunk_len, hipStream_t st)
{
    prof::Timed tm("dparam_narrow", st);
    dim3 grid((unsigned)g.n_in, (unsigned)dparam_narrow_row_blocks(g.rows), (unsigned)n_chunks);
#define CALL(N) dparam_narrow_kernel<N><<<grid, 64, 0, st>>>(g, x, gy, part_c, part_b, B, chunk_len)
    KAN_NARROW_DISPATCH(g.n_out, CALL)
#undef CALL
    return hipGetLastError();
}

}  // namespace kan
