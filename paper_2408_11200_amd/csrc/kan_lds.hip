// LDS-staged forward kernel of the local B-spline layer for grids whose per-input coefficient
// slab fits in LDS (the common case: G + k up to a few dozen rows).
//
// A workgroup of NW waves owns NW*T samples and a tile of TJ = 64*R outputs.  It walks over
// the inputs; the scale-folded coefficient slab of the current input ((rows + 1) x TJ floats,
// the extra row being w_b) sits in LDS, double-buffered so that the next slab is fetched from
// L2 while the current one is used.  Lanes <-> outputs: per (sample, input) pair a wave reads
// the K window rows plus the base row with unit-stride 16-byte LDS reads and does K + 1
// multiply-adds per output, with the pair's weights in scalar registers.  Accumulators stay in
// VGPRs for the whole kernel.
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace KAN_NS {

namespace {

// Per-pair quantities in the form the LDS kernels want: a window of K consecutive rows that
// lies inside the slab (first row `row0` in [0, rows - K]) with the weights shifted to match,
// so that one base address and K immediate offsets address the whole window.
struct WinPair {
    int row0;
    float w[kMaxK];
    float base;
};

template <bool GRAD>
__device__ __forceinline__ WinPair window_pair(float x, const SplineGeom &g, int i)
{
    const Pair p = pair_eval<GRAD>(x, g, i);
    WinPair o;
    window_of<GRAD>(p, g.rows, o.row0, o.w, o.base);
    return o;
}

template <int R>
__device__ __forceinline__ void lds_row(const float *row, int lane, float (&v)[R])
{
    // lane l owns outputs 4l..4l+3 of each 256-wide half of the tile: every 16-byte read of a
    // wave covers one contiguous KB of LDS
#pragma unroll
    for (int h = 0; h < R / 4; ++h) {
        float4 t = *reinterpret_cast<const float4 *>(row + h * 256 + lane * 4);
        v[4 * h + 0] = t.x; v[4 * h + 1] = t.y; v[4 * h + 2] = t.z; v[4 * h + 3] = t.w;
    }
}

}  // namespace

// Slab staging.  The slab of input i is the TJ-wide column block j0.. of the contiguous
// (rows + 1) x n_out block of the folded table.  Thread `tid` of NT copies quads tid, tid + NT, ...
// (NQ of them) of the slab, first into registers, later from registers into LDS.  The per-thread
// element offsets do not depend on the input, so they are computed once (SlabMap); per input the
// copy is NQ loads off a scalar base.  Quads outside the slab or the layer load element 0 and are
// zeroed on the way to LDS (MASK); the LDS slab is padded to NQ*NT quads so stores need no guard.
template <int NQ>
struct SlabMap {
    int off[NQ];          // float offset inside one input's block
    unsigned ok;          // bit c: quad c is real
};

template <int R, int NT, int NQ>
__device__ __forceinline__ SlabMap<NQ> slab_map(const SplineGeom &g, int j0, int tid)
{
    constexpr int quads_per_row = 64 * R / 4;
    SlabMap<NQ> m;
    m.ok = 0u;
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        const int e = tid + c * NT;
        const int row = e / quads_per_row, j = j0 + (e % quads_per_row) * 4;
        const bool ok = row < g.slab_rows && j < g.n_out;
        m.off[c] = ok ? row * g.n_out + j : 0;
        m.ok |= ok ? (1u << c) : 0u;
    }
    return m;
}

template <int NQ>
__device__ __forceinline__ void slab_fetch(float4 (&q)[NQ], const SlabMap<NQ> &m, const float *__restrict__ block)
{
#pragma unroll
    for (int c = 0; c < NQ; ++c) q[c] = *reinterpret_cast<const float4 *>(block + m.off[c]);
}

template <int NT, int NQ, bool MASK>
__device__ __forceinline__ void slab_store(const float4 (&q)[NQ], const SlabMap<NQ> &m, float *slab, int tid)
{
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        float4 v = q[c];
        if (MASK) {
            const bool ok = (m.ok >> c) & 1u;
            v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
        }
        *reinterpret_cast<float4 *>(slab + (int64_t)(tid + c * NT) * 4) = v;
    }
}

// ---- forward ---------------------------------------------------------------------
template <int R, int T, int NW, int NQ, bool MASK>
__global__ __launch_bounds__(64 * NW) void forward_lds_kernel(SplineGeom g, const float *__restrict__ x,
                                                              const float *__restrict__ cf,
                                                              float *__restrict__ y, int64_t B)
{
    constexpr int TJ = 64 * R, NT = 64 * NW, IPV = kWave / T;
    constexpr int slab_floats = NQ * NT * 4;            // padded slab
    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t b0 = ((int64_t)blockIdx.x * NW + wave) * T;
    const int j0 = blockIdx.y * TJ;

    float acc[T][R];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[t][r] = 0.0f;

    const int my_t = lane % T, my_ii = lane / T;
    int64_t my_b = b0 + my_t;
    if (my_b >= B) my_b = B - 1;

    const SlabMap<NQ> map = slab_map<R, NT, NQ>(g, j0, tid);
    const int64_t block_floats = (int64_t)g.slab_rows * g.n_out;
    float4 q[NQ];
    slab_fetch<NQ>(q, map, cf);
    slab_store<NT, NQ, MASK>(q, map, lds, tid);
    __syncthreads();

    for (int i0 = 0; i0 < g.n_in; i0 += IPV) {
        const int mi = i0 + my_ii;
        const int ic = mi < g.n_in ? mi : g.n_in - 1;
        const WinPair p = window_pair<false>(x[my_b * g.n_in + ic], g, ic);
        const int n_ii = (g.n_in - i0 < IPV) ? g.n_in - i0 : IPV;
        for (int ii = 0; ii < n_ii; ++ii) {
            const int i = i0 + ii;
            const float *cur = lds + (i & 1) * slab_floats;
            float *nxt = lds + ((i + 1) & 1) * slab_floats;
            // prefetch the next slab (the last iteration re-fetches its own slab: harmless)
            slab_fetch<NQ>(q, map, cf + (int64_t)(i + 1 < g.n_in ? i + 1 : i) * block_floats);

            float wb[R];
            lds_row<R>(cur + g.rows * TJ, lane, wb);   // last slab row: w_b
            if constexpr (NW <= 8) {
                // few waves per SIMD: software pipeline over the wave's samples, the window rows of
                // sample t+1 are read while sample t is accumulated
                float c[2][kMaxK][R];
                {
                    const float *win = cur + lane_i(p.row0, ii * T) * TJ;
#pragma unroll
                    for (int s = 0; s < kMaxK; ++s) lds_row<R>(win + s * TJ, lane, c[0][s]);
                }
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const int src = ii * T + t;
                    if (t + 1 < T) {
                        const float *win = cur + lane_i(p.row0, src + 1) * TJ;
#pragma unroll
                        for (int s = 0; s < kMaxK; ++s) lds_row<R>(win + s * TJ, lane, c[(t + 1) & 1][s]);
                    }
#pragma unroll
                    for (int s = 0; s < kMaxK; ++s) {
                        const float ws = lane_f(p.w[s], src);
#pragma unroll
                        for (int r = 0; r < R; ++r) acc[t][r] = fmaf(ws, c[t & 1][s][r], acc[t][r]);
                    }
                    const float bs = lane_f(p.base, src);
#pragma unroll
                    for (int r = 0; r < R; ++r) acc[t][r] = fmaf(bs, wb[r], acc[t][r]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // many waves per SIMD hide the LDS latency; keep the register count low instead
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const int src = ii * T + t;
                    const float *win = cur + lane_i(p.row0, src) * TJ;
                    float c[kMaxK][R];
#pragma unroll
                    for (int s = 0; s < kMaxK; ++s) lds_row<R>(win + s * TJ, lane, c[s]);
#pragma unroll
                    for (int s = 0; s < kMaxK; ++s) {
                        const float ws = lane_f(p.w[s], src);
#pragma unroll
                        for (int r = 0; r < R; ++r) acc[t][r] = fmaf(ws, c[s][r], acc[t][r]);
                    }
                    const float bs = lane_f(p.base, src);
#pragma unroll
                    for (int r = 0; r < R; ++r) acc[t][r] = fmaf(bs, wb[r], acc[t][r]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            slab_store<NT, NQ, MASK>(q, map, nxt, tid);
            __syncthreads();
        }
    }

#pragma unroll
    for (int t = 0; t < T; ++t) {
        if (b0 + t < B) {
#pragma unroll
            for (int h = 0; h < R / 4; ++h) {
                const int j = j0 + h * 256 + lane * 4;
                if (j < g.n_out) {
                    float4 o = make_float4(acc[t][4 * h], acc[t][4 * h + 1], acc[t][4 * h + 2], acc[t][4 * h + 3]);
                    *reinterpret_cast<float4 *>(y + (b0 + t) * g.n_out + j) = o;
                }
            }
        }
    }
}

// ---- forward, pair data through LDS -------------------------------------------------------------
// The same walk over the inputs as forward_lds_kernel, with one difference in how a wave gets at the
// per-pair quantities (window row, K weights, base value), which are uniform over the outputs: the lane that
// evaluated a pair writes them to a small area of LDS owned by the wave, and the wave reads them back with
// reads whose address is the same in every lane (one 16-byte and one 8-byte read per pair).  That replaces
// six v_readlane per pair (each a VALU slot, plus the wait states between a lane read and the use of the
// scalar it wrote), so that a pair costs K + 1 multiply-adds per output and one address addition.
template <int R, int T, int NW, int NQ, bool MASK>
__global__ __launch_bounds__(64 * NW) void forward_pairs_kernel(SplineGeom g, const float *__restrict__ x,
                                                                const float *__restrict__ cf,
                                                                float *__restrict__ y, int64_t B)
{
    constexpr int TJ = 64 * R, NT = 64 * NW, IPV = kWave / T;
    constexpr int slab_floats = NQ * NT * 4;            // padded slab
    // one pair: the window weights, the base value and the byte offset of the window row, as two quadruples:
    // window of four rows  {w0 w1 w2 w3} {base offset - -},  window of six rows  {w0 w1 w2 w3} {w4 w5 base offset}
    constexpr int kPairFloats = 8;
    static_assert(kMaxK == 4 || kMaxK == 6, "pair records are laid out for windows of four and six rows");
    extern __shared__ float lds[];                      // two slabs, then NW areas of 64 pairs
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t b0 = ((int64_t)blockIdx.x * NW + wave) * T;
    const int j0 = blockIdx.y * TJ;
    float *pairs = lds + 2 * slab_floats + wave * (64 * kPairFloats);

    float acc[T][R];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[t][r] = 0.0f;

    const int my_t = lane % T, my_ii = lane / T;
    int64_t my_b = b0 + my_t;
    if (my_b >= B) my_b = B - 1;

    const SlabMap<NQ> map = slab_map<R, NT, NQ>(g, j0, tid);
    const int64_t block_floats = (int64_t)g.slab_rows * g.n_out;
    float4 q[NQ];
    slab_fetch<NQ>(q, map, cf);
    slab_store<NT, NQ, MASK>(q, map, lds, tid);
    __syncthreads();

    for (int i0 = 0; i0 < g.n_in; i0 += IPV) {
        const int mi = i0 + my_ii;
        const int ic = mi < g.n_in ? mi : g.n_in - 1;
        const WinPair p = window_pair<false>(x[my_b * g.n_in + ic], g, ic);
        // pair (input i0 + ii, sample t) sits at index ii * T + t == lane of the lane that evaluated it
        *reinterpret_cast<float4 *>(pairs + lane * kPairFloats) = make_float4(p.w[0], p.w[1], p.w[2], p.w[3]);
        if constexpr (kMaxK == 4)
            *reinterpret_cast<float2 *>(pairs + lane * kPairFloats + 4) =
                make_float2(p.base, __int_as_float(p.row0 * TJ * 4));
        else
            *reinterpret_cast<float4 *>(pairs + lane * kPairFloats + 4) =
                make_float4(p.w[kMaxK - 2], p.w[kMaxK - 1], p.base, __int_as_float(p.row0 * TJ * 4));
        const int n_ii = (g.n_in - i0 < IPV) ? g.n_in - i0 : IPV;
        for (int ii = 0; ii < n_ii; ++ii) {
            const int i = i0 + ii;
            const float *cur = lds + (i & 1) * slab_floats;
            float *nxt = lds + ((i + 1) & 1) * slab_floats;
            // prefetch the next slab (the last iteration re-fetches its own slab: harmless)
            slab_fetch<NQ>(q, map, cf + (int64_t)(i + 1 < g.n_in ? i + 1 : i) * block_floats);

            // the T pairs of this input: same address in every lane
            float ws[T][kMaxK], bs[T];
            int off[T];
            const float *pp = pairs + ii * (T * kPairFloats);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float4 wv = *reinterpret_cast<const float4 *>(pp + t * kPairFloats);
                ws[t][0] = wv.x; ws[t][1] = wv.y; ws[t][2] = wv.z; ws[t][3] = wv.w;
                if constexpr (kMaxK == 4) {
                    const float2 bv = *reinterpret_cast<const float2 *>(pp + t * kPairFloats + 4);
                    bs[t] = bv.x; off[t] = __float_as_int(bv.y);
                } else {
                    const float4 bv = *reinterpret_cast<const float4 *>(pp + t * kPairFloats + 4);
                    ws[t][kMaxK - 2] = bv.x; ws[t][kMaxK - 1] = bv.y;
                    bs[t] = bv.z; off[t] = __float_as_int(bv.w);
                }
            }
            float wb[R];
            lds_row<R>(cur + g.rows * TJ, lane, wb);   // last slab row: w_b
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float *win = reinterpret_cast<const float *>(reinterpret_cast<const char *>(cur) + off[t]);
                float c[kMaxK][R];
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) lds_row<R>(win + s * TJ, lane, c[s]);
#pragma unroll
                for (int s = 0; s < kMaxK; ++s)
#pragma unroll
                    for (int r = 0; r < R; ++r) acc[t][r] = fmaf(ws[t][s], c[s][r], acc[t][r]);
#pragma unroll
                for (int r = 0; r < R; ++r) acc[t][r] = fmaf(bs[t], wb[r], acc[t][r]);
                __builtin_amdgcn_sched_barrier(0);
            }
            slab_store<NT, NQ, MASK>(q, map, nxt, tid);
            __syncthreads();
        }
    }

#pragma unroll
    for (int t = 0; t < T; ++t) {
        if (b0 + t < B) {
#pragma unroll
            for (int h = 0; h < R / 4; ++h) {
                const int j = j0 + h * 256 + lane * 4;
                if (j < g.n_out) {
                    float4 o = make_float4(acc[t][4 * h], acc[t][4 * h + 1], acc[t][4 * h + 2], acc[t][4 * h + 3]);
                    *reinterpret_cast<float4 *>(y + (b0 + t) * g.n_out + j) = o;
                }
            }
        }
    }
}

// ---- launch --------------------------------------------------------------------------

namespace {
constexpr size_t kLdsBudget = 160 * 1024;

// quads each thread must hold to copy one slab, rounded up to an instantiated size (0: too many)
int quads_needed(int rows, int R, int NW)
{
    const int need = ((rows + 1) * (64 * R / 4) + 64 * NW - 1) / (64 * NW);
    const int sizes[] = {2, 3, 4, 6, 8, 12, 16};
    for (int s : sizes)
        if (need <= s) return s;
    return 0;
}
// two padded slabs of NQ * NT quads
size_t lds_bytes(int rows, int R, int NW) { return 2ull * (size_t)quads_needed(rows, R, NW) * 64 * NW * 16; }
}  // namespace

// 0 = not applicable, otherwise the outputs-per-lane the launcher will use
int forward_lds_plan(const SplineGeom &g)
{
    if (g.rows < kMaxK || g.n_out % 4 != 0 || g.slab_rows != g.rows + 1) return 0;
    // eight outputs per lane: two slabs and the waves' pair areas (32 KB) must fit, the slab in at most 4 quads per thread
    if (g.n_out > 256 && quads_needed(g.rows, 8, 16) && quads_needed(g.rows, 8, 16) <= 4 &&
        lds_bytes(g.rows, 8, 16) + 16 * 64 * 8 * sizeof(float) <= kLdsBudget)
        return 8;
    if (g.n_out >= 128 && quads_needed(g.rows, 4, 8) && lds_bytes(g.rows, 4, 8) <= kLdsBudget) return 4;
    return 0;
}

template <int R, int T, int NW, int NQ>
static hipError_t forward_pairs_launch(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                                       hipStream_t st)
{
    const size_t lds = 2ull * NQ * 64 * NW * 16 + (size_t)NW * 64 * 8 * sizeof(float);
    const bool mask = (g.n_out % (64 * R)) != 0 || (int64_t)g.slab_rows * (64 * R / 4) != (int64_t)NQ * 64 * NW;
    auto kern = mask ? forward_pairs_kernel<R, T, NW, NQ, true> : forward_pairs_kernel<R, T, NW, NQ, false>;
    struct Masked; struct Plain;
    hipError_t e = mask ? ensure_dynamic_lds<Masked>(reinterpret_cast<const void *>(kern), (int)lds)
                        : ensure_dynamic_lds<Plain>(reinterpret_cast<const void *>(kern), (int)lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((B + NW * T - 1) / (NW * T)), (unsigned)((g.n_out + 64 * R - 1) / (64 * R)));
    prof::Timed tm("forward_pairs", st);
    kern<<<grid, 64 * NW, lds, st>>>(g, x, cf, y, B);
    return hipGetLastError();
}

template <int R, int T, int NW, int NQ>
static hipError_t forward_lds_launch(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                                     hipStream_t st)
{
    const size_t lds = 2ull * NQ * 64 * NW * 16;
    // masking is needed only when some quad of the padded slab is not a real element
    const bool mask = (g.n_out % (64 * R)) != 0 || (int64_t)g.slab_rows * (64 * R / 4) != (int64_t)NQ * 64 * NW;
    auto kern = mask ? forward_lds_kernel<R, T, NW, NQ, true> : forward_lds_kernel<R, T, NW, NQ, false>;
    struct Masked; struct Plain;
    hipError_t e = mask ? ensure_dynamic_lds<Masked>(reinterpret_cast<const void *>(kern), (int)lds)
                        : ensure_dynamic_lds<Plain>(reinterpret_cast<const void *>(kern), (int)lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((B + NW * T - 1) / (NW * T)), (unsigned)((g.n_out + 64 * R - 1) / (64 * R)));
    prof::Timed tm("forward_lds", st);
    kern<<<grid, 64 * NW, lds, st>>>(g, x, cf, y, B);
    return hipGetLastError();
}

template <int R, int T, int NW>
static hipError_t forward_lds_by_quads(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                                       hipStream_t st)
{
    switch (quads_needed(g.rows, R, NW)) {
    case 2: return forward_lds_launch<R, T, NW, 2>(g, x, cf, y, B, st);
    case 3: return forward_lds_launch<R, T, NW, 3>(g, x, cf, y, B, st);
    case 4: return forward_lds_launch<R, T, NW, 4>(g, x, cf, y, B, st);
    case 6: return forward_lds_launch<R, T, NW, 6>(g, x, cf, y, B, st);
    case 8: return forward_lds_launch<R, T, NW, 8>(g, x, cf, y, B, st);
    case 12: return forward_lds_launch<R, T, NW, 12>(g, x, cf, y, B, st);
    case 16: return forward_lds_launch<R, T, NW, 16>(g, x, cf, y, B, st);
    default: return hipErrorInvalidValue;
    }
}

template <int R, int T, int NW>
static hipError_t forward_pairs_by_quads(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                                         hipStream_t st)
{
    switch (quads_needed(g.rows, R, NW)) {
    case 2: return forward_pairs_launch<R, T, NW, 2>(g, x, cf, y, B, st);
    case 3: return forward_pairs_launch<R, T, NW, 3>(g, x, cf, y, B, st);
    case 4: return forward_pairs_launch<R, T, NW, 4>(g, x, cf, y, B, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_forward_lds(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                              hipStream_t st)
{
    switch (forward_lds_plan(g)) {
    case 8: return forward_pairs_by_quads<8, 4, 16>(g, x, cf, y, B, st);
    case 4: return forward_lds_by_quads<4, 16, 8>(g, x, cf, y, B, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace KAN_NS
