// Sorted records of the backward walk for spline degrees 4 and 5 (window of six rows).
//
// The walk kernel keeps a window of FOUR table rows in its accumulators (one matrix-core register
// quadruple per output).  A pair whose window has six rows is therefore handed to it as TWO records in
// its four-row format: record A covers rows 0..3 of the window and carries the base term, record B
// covers rows 4..5 (its four-row window is shifted so that it stays inside the table, the unused
// positions carry zero weights).  Both go into the same sorted list (2 S entries per chunk of S
// samples and input), sorted by their own first row, so to the walk they are just more records; the
// parameter gradients add up in the table rows, and dL/dx comes out as two partial results per pair
// (bit 31 of a record says which), which the caller sums.
//
// This translation unit is built for a window of six rows (kMaxK = 6) in a namespace of its own, like
// kan_generic_k5.hip, and exposes one function through kan_highk.hpp.
#define KAN_MAXK 6
#define KAN_NS kan_k5
#include "kan_device.hpp"
#include "kan_launch.hpp"
#include "kan_highk.hpp"

namespace kan_k5 {

namespace {

constexpr int kWalkK = 4;           // rows of a record's window (the walk kernel's ring)

// one four-row record of a pair: first row `start` (inside [0, rows - 4]), weights of rows start .. start + 3
// taken from the six-row window that begins at row0, restricted to window positions lo .. hi
template <bool GRAD>
__device__ __forceinline__ void sub_record(const float (&w6)[kMaxK], int row0, int start, int lo, int hi,
                                           float (&w)[kWalkK])
{
#pragma unroll
    for (int s = 0; s < kWalkK; ++s) {
        const int q = start + s - row0;          // position in the six-row window
        float v = 0.0f;
#pragma unroll
        for (int u = 0; u < kMaxK; ++u) v = (u == q && q >= lo && q <= hi) ? w6[u] : v;
        w[s] = v;
    }
}

// grid (n_chunks, n_in), NW waves.  The 2 S keys of a list are  row << (sbits + 1) | (2 * sample + which):
// distinct, so a stable counting sort by the row digits keeps equal rows in (sample, which) order, which
// fixes the summation order downstream.  Same radix sort as the four-row kernel (8-bit digits, per-wave
// digit counts, ranks inside a batch of 64 from ballots).  Entries of samples past the end of the batch get
// the largest row and zero weights and end up behind every real record.
template <int NW>
__global__ __launch_bounds__(64 * NW) void cell_sort_two_records_kernel(SplineGeom g, const float *__restrict__ xT,
                                                                        int64_t B, int S, int sbits, int row_bits,
                                                                        int *__restrict__ rec_rt,
                                                                        float *__restrict__ rec_base,
                                                                        float *__restrict__ rec_w4,
                                                                        float *__restrict__ rec_dbase,
                                                                        float *__restrict__ rec_dw4)
{
    constexpr int kSortThreads = 64 * NW;
    const int L = 2 * S, lbits = sbits + 1;
    extern __shared__ unsigned lds_u[];
    unsigned *src = lds_u, *dst = lds_u + L;
    float *xs = reinterpret_cast<float *>(lds_u + 2 * L);
    __shared__ unsigned slot[NW][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = blockIdx.x, i = blockIdx.y;
    const int64_t b0 = (int64_t)c * S;
    const int n_c = (int)((B - b0) < S ? (B - b0) : S);
    const int last = g.rows - kWalkK;              // largest first row of a record

    for (int e = tid; e < S; e += kSortThreads) {
        const bool live = e < n_c;
        const float xv = live ? xT[(int64_t)i * B + b0 + e] : 0.0f;
        xs[e] = xv;
        int ra = last, rb = last;
        if (live) {
            const Pair p = pair_eval<false>(xv, g, i);
            float w[kMaxK], base;
            int row0;
            window_of<false>(p, g.rows, row0, w, base);
            ra = row0;                              // <= rows - 6
            rb = row0 + kWalkK < last ? row0 + kWalkK : last;
        }
        src[2 * e] = ((unsigned)ra << lbits) | (unsigned)(2 * e);
        src[2 * e + 1] = ((unsigned)rb << lbits) | (unsigned)(2 * e + 1);
    }
    __syncthreads();

    const int per_wave = L / NW;                    // a multiple of 64
    const int n_pass = (row_bits + 7) / 8;
    const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int pass = 0; pass < n_pass; ++pass) {
        const int shift = lbits + 8 * pass;
        const int nbits = row_bits - 8 * pass < 8 ? row_bits - 8 * pass : 8;
        for (int d = tid; d < NW * 256; d += kSortThreads) (&slot[0][0])[d] = 0u;
        __syncthreads();
        for (int e = wave * per_wave + lane; e < (wave + 1) * per_wave; e += 64)
            atomicAdd(&slot[wave][(src[e] >> shift) & 255u], 1u);
        __syncthreads();
        // first slot of every (digit, wave): exclusive prefix over digits, then over waves; done by
        // the first wave, four digits per lane
        if (wave == 0) {
            unsigned tot[4], mine_tot = 0;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                tot[qd] = 0;
                for (int w2 = 0; w2 < NW; ++w2) tot[qd] += slot[w2][4 * lane + qd];
                mine_tot += tot[qd];
            }
            unsigned inc = mine_tot;
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned v = __shfl_up(inc, o, 64);
                if (lane >= o) inc += v;
            }
            unsigned at = inc - mine_tot;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                unsigned a = at;
                for (int w2 = 0; w2 < NW; ++w2) {
                    const unsigned cnt = slot[w2][4 * lane + qd];
                    slot[w2][4 * lane + qd] = a;
                    a += cnt;
                }
                at += tot[qd];
            }
        }
        __syncthreads();
        for (int e0 = wave * per_wave; e0 < (wave + 1) * per_wave; e0 += 64) {
            const unsigned key = src[e0 + lane];
            const int d = (int)((key >> shift) & 255u);
            unsigned long long same = ~0ull;
            for (int bit = 0; bit < nbits; ++bit) {
                const bool set = ((d >> bit) & 1) != 0;
                const unsigned long long m = __ballot(set);
                same &= set ? m : ~m;
            }
            const unsigned rank = (unsigned)__builtin_popcountll(same & below);
            const unsigned first = slot[wave][d];
            dst[first + rank] = key;
            atomicAdd(&slot[wave][d], 1u);
        }
        __syncthreads();
        unsigned *t = src; src = dst; dst = t;
    }

    const int64_t list = ((int64_t)c * g.n_in + i) * L;
    for (int p = tid; p < L; p += kSortThreads) {
        const int idx = (int)(src[p] & (unsigned)(L - 1));
        const int e = idx >> 1, which = idx & 1;
        const bool live = e < n_c;
        const Pair pr = rec_dw4 ? pair_eval<true>(xs[e], g, i) : pair_eval<false>(xs[e], g, i);
        float w6[kMaxK], dw6[kMaxK], base, dbase;
        int row0;
        window_of<false>(pr, g.rows, row0, w6, base);
        window_of<true>(pr, g.rows, row0, dw6, dbase);
        int start = which ? (row0 + kWalkK < last ? row0 + kWalkK : last) : row0;
        float w[kWalkK], dw[kWalkK];
        sub_record<false>(w6, row0, start, which ? kWalkK : 0, which ? kMaxK - 1 : kWalkK - 1, w);
        sub_record<true>(dw6, row0, start, which ? kWalkK : 0, which ? kMaxK - 1 : kWalkK - 1, dw);
        if (which) { base = 0.0f; dbase = 0.0f; }                 // the base term rides on the first record
        if (!live) {
            start = last;
#pragma unroll
            for (int s = 0; s < kWalkK; ++s) { w[s] = 0.0f; dw[s] = 0.0f; }
            base = 0.0f; dbase = 0.0f;
        }
        // the walk keeps its four window rows in a ring indexed by (row mod 4): weight of row start + s goes to
        // position (start + s) mod 4
        float wr[kWalkK], dwr[kWalkK];
#pragma unroll
        for (int q = 0; q < kWalkK; ++q) {
            float v = 0.0f, dv = 0.0f;
#pragma unroll
            for (int s = 0; s < kWalkK; ++s) {
                const bool hit = ((start + s) & (kWalkK - 1)) == q;
                v = hit ? w[s] : v;
                dv = hit ? dw[s] : dv;
            }
            wr[q] = v; dwr[q] = dv;
        }
        rec_rt[list + p] = (int)((unsigned)start | ((unsigned)(live ? e : 0) << kRtRowBits) |
                                 ((unsigned)(live ? which : 0) << 31));
        rec_base[list + p] = base;
        *reinterpret_cast<float4 *>(rec_w4 + (list + p) * 4) = make_float4(wr[0], wr[1], wr[2], wr[3]);
        if (rec_dw4) {
            rec_dbase[list + p] = dbase;
            *reinterpret_cast<float4 *>(rec_dw4 + (list + p) * 4) = make_float4(dwr[0], dwr[1], dwr[2], dwr[3]);
        }
    }
}

}  // namespace

}  // namespace kan_k5

namespace kan {

hipError_t highk_sorted_records(const HighKLayer &l, const float *xT, int64_t B, int S, int row_bits, int *rt,
                                float *base, float *w4, float *dbase, float *dw4, hipStream_t st)
{
    if (S < 256 || S > 4096 || (S & (S - 1)) != 0 || l.rows < 6) return hipErrorInvalidValue;
    kan_k5::SplineGeom g;
    g.n_in = l.n_in; g.n_out = l.n_out; g.rows = l.rows; g.slab_rows = l.slab_rows ? l.slab_rows : l.rows + 1; g.k = l.k;
    g.lo = l.lo; g.inv_h = l.inv_h; g.cell_base = l.cell_base; g.base_act = l.base_act;
    int sbits = 0;
    while ((1 << sbits) < S) ++sbits;
    const size_t lds = (size_t)S * 20;              // two key arrays of 2 S entries and the S sample values
    auto kern = S >= 2048 ? kan_k5::cell_sort_two_records_kernel<16> : kan_k5::cell_sort_two_records_kernel<4>;
    struct Long; struct Short;
    hipError_t e = S >= 2048 ? kan_k5::ensure_dynamic_lds<Long>(reinterpret_cast<const void *>(kern), (int)lds)
                             : kan_k5::ensure_dynamic_lds<Short>(reinterpret_cast<const void *>(kern), (int)lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((B + S - 1) / S), (unsigned)l.n_in);
    kanprof::Timed tm("walk_sort", st);
    kern<<<grid, S >= 2048 ? 1024 : 256, lds, st>>>(g, xT, B, S, sbits, row_bits, rt, base, w4, dbase, dw4);
    return hipGetLastError();
}

}  // namespace kan
