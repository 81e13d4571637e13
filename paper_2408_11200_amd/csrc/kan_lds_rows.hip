// LDS-staged forward kernel for tables too long for forward_lds_kernel (a slab of a 256- or
// 512-wide output tile no longer fits LDS): hundreds of rows per input, as on large grids and on
// the generated tables of UKAN layers.
//
// Such layers used to gather their window rows straight from L2 (forward_generic_kernel), four
// 1 KB rows per (sample, input) pair, and ran at the rate at which a CU can pull lines out of L2.
// Here a workgroup takes a NARROW output tile (TJ = 64 or 32 outputs) and MANY samples
// (NW waves x SPW x S): the slab of the current input for that tile (slab_rows x TJ floats) is
// staged in LDS, double-buffered, and every row fetched from L2 once serves all the workgroup's
// samples, which cuts the L2 traffic by (samples x K) / slab_rows.
//
// Mapping inside a wave: the 64 lanes are SPW = 64 / LPS groups of LPS lanes; a group works on one
// sample at a time and its lanes hold four consecutive outputs each (LPS * 4 = TJ), so one 16-byte
// LDS read per lane fetches a window row for SPW samples at once (each group reads its own row).
// Every group handles S samples (slots), accumulators for all of them stay in registers
// (S x 4 per lane) while the workgroup walks over the inputs.  The per-pair quantities (K weights,
// base value, byte offset of the window row) go through a small per-wave area of LDS, written by the
// lane that evaluated the pair and read back by the group that owns the sample.
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace kan {

namespace {

constexpr int kPairFloats = 8;      // w[0..3], base, byte offset of the window row, 2 unused

template <int NQ>
struct TileMap {
    int off[NQ];          // float offset of the thread's quads inside one input's block of the table
    unsigned ok;          // bit c: quad c is a real element
};

}  // namespace

// grid (ceil(B / (NW * SPW * S)), ceil(n_out / TJ)), NW waves.  Needs rows >= kMaxK, n_out % 4 == 0.
// The table has slab_rows rows per input; with slab_rows == rows + 1 the last one is the w_b row.
template <int LPS, int S, int NW, int NQ>
__global__ __launch_bounds__(64 * NW) void forward_lds_rows_kernel(SplineGeom g, const float *__restrict__ x,
                                                                   const float *__restrict__ cf,
                                                                   float *__restrict__ y, int64_t B)
{
    constexpr int TJ = LPS * 4, SPW = 64 / LPS, NT = 64 * NW;
    constexpr int SMP = SPW * S;                        // samples per wave
    constexpr int IPV = 64 / SMP;                       // inputs one round of pair evaluations covers
    constexpr int slab_floats = NQ * NT * 4;            // padded slab
    static_assert(SMP <= 64 && 64 % SMP == 0, "the wave's samples must tile its lanes");
    extern __shared__ float lds[];                      // two slabs, then NW areas of 64 pairs
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = lane / LPS, lj = lane % LPS;
    const int64_t b0 = ((int64_t)blockIdx.x * NW + wave) * SMP;
    const int j0 = blockIdx.y * TJ;
    const int j = j0 + lj * 4;
    float *pairs = lds + 2 * slab_floats + wave * (64 * kPairFloats);
    const bool has_base = g.slab_rows == g.rows + 1;

    // two-level sum over the inputs (acc is folded into tot every 32 inputs): keeps the rounding error
    // of a sum over hundreds of inputs inside the forward tolerance
    constexpr int kFoldInputs = 32;
    float acc[S][4], tot[S][4];
#pragma unroll
    for (int q = 0; q < S; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) { acc[q][r] = 0.0f; tot[q][r] = 0.0f; }

    // pair evaluation: lane <-> (input my_ii of the round, sample my_smp of the wave)
    const int my_smp = lane % SMP, my_ii = lane / SMP;
    int64_t my_b = b0 + my_smp;
    if (my_b >= B) my_b = B - 1;

    // slab copy: thread tid moves quads tid, tid + NT, ... of the padded slab
    TileMap<NQ> map;
    map.ok = 0u;
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        const int e = tid + c * NT;
        const int row = e / LPS, jj = j0 + (e % LPS) * 4;
        const bool ok = row < g.slab_rows && jj < g.n_out;
        map.off[c] = ok ? row * g.n_out + jj : 0;
        map.ok |= ok ? (1u << c) : 0u;
    }
    const int64_t block_floats = (int64_t)g.slab_rows * g.n_out;
    float4 qd[NQ];
    auto fetch = [&](const float *__restrict__ block) {
#pragma unroll
        for (int c = 0; c < NQ; ++c) qd[c] = *reinterpret_cast<const float4 *>(block + map.off[c]);
    };
    auto stage = [&](float *slab) {
#pragma unroll
        for (int c = 0; c < NQ; ++c) {
            float4 v = qd[c];
            const bool ok = (map.ok >> c) & 1u;
            v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
            *reinterpret_cast<float4 *>(slab + (int64_t)(tid + c * NT) * 4) = v;
        }
    };
    fetch(cf);
    stage(lds);
    __syncthreads();

    for (int i0 = 0; i0 < g.n_in; i0 += IPV) {
        if (i0 % kFoldInputs == 0 && i0 > 0) {
#pragma unroll
            for (int q = 0; q < S; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) { tot[q][r] += acc[q][r]; acc[q][r] = 0.0f; }
        }
        const int mi = i0 + my_ii;
        const int ic = mi < g.n_in ? mi : g.n_in - 1;
        {
            const Pair pr = pair_eval<false>(x[my_b * g.n_in + ic], g, ic);
            int row0;
            float w[kMaxK], base;
            window_of<false>(pr, g.rows, row0, w, base);
            // pair (input i0 + ii, sample smp) sits at index ii * SMP + smp == the lane that evaluated it
            *reinterpret_cast<float4 *>(pairs + lane * kPairFloats) = make_float4(w[0], w[1], w[2], w[3]);
            *reinterpret_cast<float2 *>(pairs + lane * kPairFloats + 4) =
                make_float2(has_base ? base : 0.0f, __int_as_float(row0 * TJ * 4));
        }
        const int n_ii = (g.n_in - i0 < IPV) ? g.n_in - i0 : IPV;
        for (int ii = 0; ii < n_ii; ++ii) {
            const int i = i0 + ii;
            const float *cur = lds + (i & 1) * slab_floats;
            float *nxt = lds + ((i + 1) & 1) * slab_floats;
            // prefetch the next slab (the last iteration re-fetches its own slab: harmless)
            fetch(cf + (int64_t)(i + 1 < g.n_in ? i + 1 : i) * block_floats);

            float4 wb = make_float4(0.f, 0.f, 0.f, 0.f);
            if (has_base) wb = *reinterpret_cast<const float4 *>(cur + g.rows * TJ + lj * 4);
            const float *pp = pairs + (ii * SMP + grp * S) * kPairFloats;     // the group's S samples
#pragma unroll
            for (int q = 0; q < S; ++q) {
                const float4 wv = *reinterpret_cast<const float4 *>(pp + q * kPairFloats);
                const float2 bv = *reinterpret_cast<const float2 *>(pp + q * kPairFloats + 4);
                const float *win = reinterpret_cast<const float *>(reinterpret_cast<const char *>(cur) +
                                                                   __float_as_int(bv.y)) + lj * 4;
                float4 c[kMaxK];
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) c[s] = *reinterpret_cast<const float4 *>(win + s * TJ);
                const float ws[kMaxK] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
                for (int s = 0; s < kMaxK; ++s) {
                    acc[q][0] = fmaf(ws[s], c[s].x, acc[q][0]);
                    acc[q][1] = fmaf(ws[s], c[s].y, acc[q][1]);
                    acc[q][2] = fmaf(ws[s], c[s].z, acc[q][2]);
                    acc[q][3] = fmaf(ws[s], c[s].w, acc[q][3]);
                }
                acc[q][0] = fmaf(bv.x, wb.x, acc[q][0]);
                acc[q][1] = fmaf(bv.x, wb.y, acc[q][1]);
                acc[q][2] = fmaf(bv.x, wb.z, acc[q][2]);
                acc[q][3] = fmaf(bv.x, wb.w, acc[q][3]);
            }
            stage(nxt);
            __syncthreads();
        }
    }

    if (j < g.n_out) {
#pragma unroll
        for (int q = 0; q < S; ++q) {
            const int64_t b = b0 + grp * S + q;
            if (b < B)
                *reinterpret_cast<float4 *>(y + b * g.n_out + j) =
                    make_float4(tot[q][0] + acc[q][0], tot[q][1] + acc[q][1], tot[q][2] + acc[q][2], tot[q][3] + acc[q][3]);
        }
    }
}

namespace {

constexpr size_t kLdsBudget = 160 * 1024;
constexpr int kSlots = 4;           // S: samples a lane group works through

struct RowsPlan { int lps, nw, nq; };

// tile width, workgroup size and copy depth for a layer (lps == 0: not applicable)
RowsPlan plan_of(const SplineGeom &g, int64_t B)
{
    RowsPlan none = {0, 0, 0};
    if (g.rows < kMaxK || g.n_out % 4 != 0 || g.n_out < 32) return none;
    if (g.slab_rows != g.rows + 1 && (g.slab_rows != g.rows || g.base_act != 0)) return none;
    const int lps_opts[] = {16, 8};
    for (int lps : lps_opts) {
        const int tj = lps * 4, spw = 64 / lps;
        if (g.n_out < tj) continue;
        const int64_t tiles = (g.n_out + tj - 1) / tj;
        // 16 waves when that still leaves about a workgroup per CU, else 8
        const int nw_opts[] = {16, 8};
        for (int nw : nw_opts) {
            const int64_t per_wg = (int64_t)nw * spw * kSlots;
            const int64_t wgs = (B + per_wg - 1) / per_wg * tiles;
            if (nw == 16 && wgs < 256) continue;
            // eight waves (two per SIMD) only when one tile covers the layer: with several tiles every tile
            // evaluates the pairs again and the smaller workgroup did not beat the generic kernel (256 -> 256,
            // G = 200, B = 8192: 0.38 ms against 0.34 ms)
            if (nw == 8 && tiles > 1) continue;
            const int64_t quads = (int64_t)g.slab_rows * lps;
            const int64_t need = (quads + 64 * nw - 1) / (64 * nw);
            const int sizes[] = {2, 4, 8, 16};
            int nq = 0;
            for (int s2 : sizes)
                if (need <= s2) { nq = s2; break; }
            if (!nq) continue;
            const size_t lds = 2ull * nq * 64 * nw * 16 + (size_t)nw * 64 * kPairFloats * sizeof(float);
            if (lds > kLdsBudget) continue;
            // worth it only when a staged row serves many samples (the copy into LDS costs as much LDS
            // time per row as several reads of it): samples * K >= 4 * slab rows
            if (per_wg * kMaxK < 4 * (int64_t)g.slab_rows) continue;
            RowsPlan p = {lps, nw, nq};
            return p;
        }
    }
    return none;
}

template <int LPS, int NW, int NQ>
hipError_t launch_variant(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B, hipStream_t st)
{
    constexpr int SPW = 64 / LPS;
    const size_t lds = 2ull * NQ * 64 * NW * 16 + (size_t)NW * 64 * kPairFloats * sizeof(float);
    auto kern = forward_lds_rows_kernel<LPS, kSlots, NW, NQ>;
    struct Tag;
    hipError_t e = ensure_dynamic_lds<Tag>(reinterpret_cast<const void *>(kern), (int)lds);
    if (e != hipSuccess) return e;
    const int64_t per_wg = (int64_t)NW * SPW * kSlots;
    dim3 grid((unsigned)((B + per_wg - 1) / per_wg), (unsigned)((g.n_out + LPS * 4 - 1) / (LPS * 4)));
    prof::Timed tm("forward_lds_rows", st);
    kern<<<grid, 64 * NW, lds, st>>>(g, x, cf, y, B);
    return hipGetLastError();
}

template <int LPS, int NW>
hipError_t launch_by_quads(int nq, const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                           hipStream_t st)
{
    switch (nq) {
    case 2: return launch_variant<LPS, NW, 2>(g, x, cf, y, B, st);
    case 4: return launch_variant<LPS, NW, 4>(g, x, cf, y, B, st);
    case 8: return launch_variant<LPS, NW, 8>(g, x, cf, y, B, st);
    case 16: return launch_variant<LPS, NW, 16>(g, x, cf, y, B, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

int forward_lds_rows_plan(const SplineGeom &g, int64_t B) { return plan_of(g, B).lps; }

hipError_t launch_forward_lds_rows(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                                   hipStream_t st)
{
    const RowsPlan p = plan_of(g, B);
    if (p.lps == 16 && p.nw == 16) return launch_by_quads<16, 16>(p.nq, g, x, cf, y, B, st);
    if (p.lps == 16 && p.nw == 8) return launch_by_quads<16, 8>(p.nq, g, x, cf, y, B, st);
    if (p.lps == 8 && p.nw == 16) return launch_by_quads<8, 16>(p.nq, g, x, cf, y, B, st);
    if (p.lps == 8 && p.nw == 8) return launch_by_quads<8, 8>(p.nq, g, x, cf, y, B, st);
    return hipErrorInvalidValue;
}

}  // namespace kan
