// Kernels for narrow layers (at most 16 outputs), e.g. the 5 -> 1 layer of a small KAN or the last
// layer of a regression stack.  With so few outputs the lanes <-> outputs mapping of the other
// kernels would leave most of a wave idle, so here lanes <-> samples (forward, dL/dx: every lane
// evaluates its own pair and gathers its own window; nothing is reduced across lanes).  The
// parameter gradients of narrow layers are taken by the chunk-sorted walk.
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace kan {

// ---- forward ------------------------------------------------------------------------------
// Four lanes per sample: lane q of the quad takes inputs q, q + 4, ... and the four partial sums are
// added across the quad at the end (with one thread per sample a batch of a few ten thousand leaves
// most of the chip idle).
template <int NO>
__global__ __launch_bounds__(256) void forward_narrow_kernel(SplineGeom g, const float *__restrict__ x,
                                                             const float *__restrict__ cf,
                                                             const float *__restrict__ w_b, float *__restrict__ y,
                                                             int64_t B)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t b = t >> 2;
    const int q = (int)(t & 3);
    const int64_t bc = b < B ? b : B - 1;        // lanes past the batch recompute the last sample: quads stay whole
    float acc[NO];
#pragma unroll
    for (int j = 0; j < NO; ++j) acc[j] = 0.0f;
    for (int i = q; i < g.n_in; i += 4) {
        const Pair p = pair_eval<false>(x[bc * g.n_in + i], g, i);
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
    for (int j = 0; j < NO; ++j) {
        float v = acc[j];
        v += __shfl_xor(v, 1, 64);
        v += __shfl_xor(v, 2, 64);
        acc[j] = v;
    }
    if (q == 0 && b < B) {
#pragma unroll
        for (int j = 0; j < NO; ++j)
            if (j < g.n_out) y[b * g.n_out + j] = acc[j];
    }
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

// ---- launch -------------------------------------------------------------------------------------

int narrow_applicable(const SplineGeom &g) { return g.n_out <= 16 ? 1 : 0; }

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
    const unsigned blocks = (unsigned)((4 * B + 255) / 256);
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

}  // namespace kan
