// Forward kernel for layers of 17 .. 64 outputs (the paper's own 32 -> 32 benchmark shape, 64 -> 64).
//
// With lanes <-> outputs and one sample at a time such a layer fills a quarter to a half of a wave,
// and every coefficient load moves 128-256 bytes, so the texture path spends its time on load
// instructions rather than on bytes.  Here a wave works on FOUR samples at once, one per DPP row of
// 16 lanes; a lane holds T = 2 or 4 outputs of its row's sample.  Lane l of a row evaluates the pair
// (row's sample, input i0 + l); the window weights and the window row of input i0 + ii are then read
// from lane ii of the same row with row_newbcast, so the four rows proceed in lockstep on
// different samples with no scalar state.  One 8- or 16-byte load per lane fetches a table row for all
// four samples.
#include <type_traits>
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace KAN_NS {

namespace {

template <int N>
__device__ __forceinline__ int row_bcast(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + N, 0xF, 0xF, true);
}
template <int N>
__device__ __forceinline__ float row_bcast(float v)
{
    return __builtin_bit_cast(float, row_bcast<N>(__builtin_bit_cast(int, v)));
}

template <int N, int END, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N < END) {
        f(std::integral_constant<int, N>{});
        static_for<N + 1, END>(f);
    }
}

template <int T>
__device__ __forceinline__ void load_t(const float *p, float (&v)[T])
{
    if constexpr (T == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        v[0] = t.x; v[1] = t.y;
    }
}
template <int T>
__device__ __forceinline__ void store_t(float *p, const float (&v)[T])
{
    if constexpr (T == 4) *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
}

constexpr int kSamplesPerRow = 8;      // samples a DPP row handles one after the other

}  // namespace

// grid: ceil(B / (4 waves * 4 rows * kSamplesPerRow)), 256 threads.  Needs rows >= kMaxK, a table with
// the w_b row appended (slab_rows == rows + 1) and n_out % T == 0, n_out <= 16 * T.
template <int T>
__global__ __launch_bounds__(256) void forward_rows_kernel(SplineGeom g, const float *__restrict__ x,
                                                           const float *__restrict__ cf, float *__restrict__ y,
                                                           int64_t B)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = lane >> 4, l16 = lane & 15;
    const int j = l16 * T;
    const bool jok = j < g.n_out;
    const int jc = jok ? j : 0;
    const int64_t first = (((int64_t)blockIdx.x * 4 + wave) * 4 + row) * kSamplesPerRow;
    const int64_t slab_floats = (int64_t)g.slab_rows * g.n_out;

    for (int q = 0; q < kSamplesPerRow; ++q) {
        // rows past the end of the batch recompute the last sample and store nothing: all four rows of
        // the wave stay in step
        const int64_t b = first + q;
        const int64_t bc = b < B ? b : B - 1;
        float acc[T], tot[T];
#pragma unroll
        for (int r = 0; r < T; ++r) { acc[r] = 0.0f; tot[r] = 0.0f; }
        for (int i0 = 0; i0 < g.n_in; i0 += 16) {
            const int mi = i0 + l16;
            const int ic = mi < g.n_in ? mi : g.n_in - 1;
            const Pair p = pair_eval<false>(x[bc * g.n_in + ic], g, ic);
            int row0;
            float w[kMaxK], base;
            window_of<false>(p, g.rows, row0, w, base);
            if (mi >= g.n_in) {
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) w[s] = 0.0f;
                base = 0.0f;
            }
            // float offset of window row 0 in input ic's slab
            const int off = row0 * g.n_out;
            const float *slab0 = cf + (int64_t)i0 * slab_floats;
            static_for<0, 16>([&](auto n) {
                constexpr int N = decltype(n)::value;
                // inputs past n_in read input n_in - 1's slab with zero weights
                const int in = i0 + N < g.n_in ? N : g.n_in - 1 - i0;
                const float *slab = slab0 + (int64_t)in * slab_floats;        // uniform
                const int o = row_bcast<N>(off) + jc;
                float c[kMaxK][T], wb[T];
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) load_t<T>(slab + s * g.n_out + o, c[s]);
                load_t<T>(slab + g.rows * g.n_out + jc, wb);
                float ws[kMaxK];
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) ws[s] = row_bcast<N>(w[s]);
                const float bs = row_bcast<N>(base);
#pragma unroll
                for (int r = 0; r < T; ++r) {
#pragma unroll
                    for (int s = 0; s < kMaxK; ++s) acc[r] = fmaf(ws[s], c[s][r], acc[r]);
                    acc[r] = fmaf(bs, wb[r], acc[r]);
                }
            });
            if ((i0 & 16) != 0) {       // two-level sum over the inputs, folded every 32
#pragma unroll
                for (int r = 0; r < T; ++r) { tot[r] += acc[r]; acc[r] = 0.0f; }
            }
        }
#pragma unroll
        for (int r = 0; r < T; ++r) tot[r] += acc[r];
        if (jok && b < B) store_t<T>(y + b * g.n_out + j, tot);
    }
}

// 0: not applicable, else outputs per lane
int forward_rows_plan(const SplineGeom &g)
{
    if (g.rows < kMaxK || g.slab_rows != g.rows + 1 || g.n_out <= 16 || g.n_out > 64) return 0;
    if (g.n_out <= 32 && g.n_out % 2 == 0) return 2;
    if (g.n_out % 4 == 0) return 4;
    return 0;
}

hipError_t launch_forward_rows(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                               hipStream_t st)
{
    const unsigned blocks = (unsigned)((B + 16 * kSamplesPerRow - 1) / (16 * kSamplesPerRow));
    prof::Timed tm("forward_rows", st);
    switch (forward_rows_plan(g)) {
    case 2: forward_rows_kernel<2><<<blocks, 256, 0, st>>>(g, x, cf, y, B); break;
    case 4: forward_rows_kernel<4><<<blocks, 256, 0, st>>>(g, x, cf, y, B); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace KAN_NS
