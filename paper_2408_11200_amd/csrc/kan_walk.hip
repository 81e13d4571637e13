// Backward kernels built on pair records that are sorted by window row over a whole chunk of
// the batch: the parameter gradients of every layer shape they cover, and dL/dx with them where
// that is the faster way.
//
// With many coefficient rows per input (G + k in the hundreds, or a generated UKAN table) a tile of
// 64 samples touches each row at most a few times, so any scheme that keeps "all rows of an input"
// or "a block of rows" in registers spends its time on rows that receive nothing.  Here the samples
// of one chunk (S = 256 .. 8192 samples) are sorted by the first row of their window, per input.  A
// stream then walks a sorted list once: the window rows of consecutive records never move
// backwards, so K accumulators per output follow the window along the rows; a row is written out
// the moment the window has passed it and rows that no sample touched are written as zeros on the
// way (or jumped over).  Work per stream is (records) x (K + 1) multiply-adds plus one 16-byte
// store per row -- independent of the grid size (section "Algorithm": cost of the local form does
// not grow with G).
//
//   1. transpose_kernel      x[B][n_in] -> xT[n_in][B], so that one input's samples are contiguous
//   2. cell_sort_kernel      per (chunk, input): stable LSD radix sort of the S samples by window row
//                            in LDS, then one record per sample in sorted order (structure of
//                            arrays: window row | sample, base value, the K weights)
//   3. backward_walk_kernel  the walk; partial sums per chunk, reduced by dparam_reduce (fp64,
//                            fixed order), so results are bit-reproducible
//   4. walk_carry_kernel     when a list is cut into several segments (one stream each): adds what a
//                            segment's window held past its last own row to the next segment's rows
//
// Lanes <-> outputs.  A wave holds 64 / LPS streams of LPS lanes each (LPS = 16, 32 or 64), so that
// narrow layers still fill the wave.  Records are loaded 16 at a time, one per lane of each DPP row
// of 16 lanes, and broadcast inside the row with row_newbcast; there is no scalar state, hence
// streams in one wave may diverge freely.
//
// The accumulation itself, acc[row s][output j] += w_s * gy[j] for the K = 4 window rows, is a
// rank-1 update, and runs on the matrix cores as v_mfma_f32_4x4x1 (16 blocks of 4x4 outer
// products): a lane's B operand is gy of its output, the A operand of every block is the weight
// quadruple of the current record, which the instruction itself broadcasts from the four lanes that
// hold it (cbsz / abid), so the weights of 16 records are one coalesced 256-byte load and cost no
// VALU work.  None of the 256 multiply-adds of an instruction is padding.
#include "kan_device.hpp"
#include "kan_launch.hpp"
#include "kan_highk.hpp"

namespace kan {

namespace {

// ---- 1. transpose --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ x, float *__restrict__ xT,
                                                        int64_t B, int n_in)
{
    __shared__ float tile[64][65];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t b0 = (int64_t)blockIdx.x * 64;
    const int i0 = blockIdx.y * 64;
    for (int r = ty; r < 64; r += 4)
        tile[r][tx] = (b0 + r < B && i0 + tx < n_in) ? x[(b0 + r) * n_in + i0 + tx] : 0.0f;
    __syncthreads();
    for (int r = ty; r < 64; r += 4)
        if (i0 + r < n_in && b0 + tx < B) xT[(int64_t)(i0 + r) * B + b0 + tx] = tile[tx][r];
}

// ---- 2. sort + records ---------------------------------------------------------------------
// grid (n_chunks, n_in), NW waves.  key = window row << sbits | sample index in the chunk
// (sbits = log2 S): keys are distinct, and sorting them by the row digits with a stable counting
// sort keeps samples of equal row in batch order, which fixes the summation order downstream.
// Each wave owns a contiguous share of the sequence; digit counts are taken per wave, the
// (digit, wave) prefix gives every wave its first slot per digit, and the wave then places its
// keys batch by batch (rank inside a batch from ballots), so nothing depends on timing.
// Entries past the end of the batch get the largest row and end up behind every real record.
template <int NW>
__global__ __launch_bounds__(64 * NW) void cell_sort_kernel(SplineGeom g, const float *__restrict__ xT, int64_t B,
                                                            int S, int sbits, int row_bits, WalkRecords rec)
{
    constexpr int kSortThreads = 64 * NW;
    extern __shared__ unsigned lds_u[];
    unsigned *src = lds_u, *dst = lds_u + S;
    float *xs = reinterpret_cast<float *>(lds_u + 2 * S);
    __shared__ unsigned slot[NW][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = blockIdx.x, i = blockIdx.y;
    const int64_t b0 = (int64_t)c * S;
    const int n_c = (int)((B - b0) < S ? (B - b0) : S);

    for (int e = tid; e < S; e += kSortThreads) {
        const bool live = e < n_c;
        const float xv = live ? xT[(int64_t)i * B + b0 + e] : 0.0f;
        xs[e] = xv;
        int row0 = g.rows - kMaxK;
        if (live) {
            const Pair p = pair_eval<false>(xv, g, i);
            float w[kMaxK], base;
            window_of<false>(p, g.rows, row0, w, base);
        }
        src[e] = ((unsigned)row0 << sbits) | (unsigned)e;
    }
    __syncthreads();

    const int per_wave = S / NW;                    // a multiple of 64
    const int n_pass = (row_bits + 7) / 8;
    const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int pass = 0; pass < n_pass; ++pass) {
        const int shift = sbits + 8 * pass;
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
            // lanes holding the same digit: intersect, bit by bit, the ballots of "my value of that bit"
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

    const int64_t list = ((int64_t)c * g.n_in + i) * S;
    for (int p = tid; p < S; p += kSortThreads) {
        const int e = (int)(src[p] & (unsigned)(S - 1));
        const bool live = e < n_c;
        const Pair pr = rec.dw4 ? pair_eval<true>(xs[e], g, i) : pair_eval<false>(xs[e], g, i);
        float w[kMaxK], dw[kMaxK], base, dbase;
        int row0;
        window_of<false>(pr, g.rows, row0, w, base);
        window_of<true>(pr, g.rows, row0, dw, dbase);
        if (!live) {
            row0 = g.rows - kMaxK;
#pragma unroll
            for (int s = 0; s < kMaxK; ++s) { w[s] = 0.0f; dw[s] = 0.0f; }
            base = 0.0f; dbase = 0.0f;
        }
        // The consumer keeps its K window rows in a ring indexed by (row mod K): store the weight of
        // window row row0 + s in position (row0 + s) mod K, so that it needs no shifting there.
        float wr[kMaxK], dwr[kMaxK];
#pragma unroll
        for (int q = 0; q < kMaxK; ++q) {
            float v = 0.0f, dv = 0.0f;
#pragma unroll
            for (int s = 0; s < kMaxK; ++s) {
                const bool hit = ((row0 + s) & (kMaxK - 1)) == q;
                v = hit ? w[s] : v;
                dv = hit ? dw[s] : dv;
            }
            wr[q] = v; dwr[q] = dv;
        }
        rec.rt[list + p] = row0 | ((live ? e : 0) << kRtRowBits);
        rec.base[list + p] = base;
        *reinterpret_cast<float4 *>(rec.w4 + (list + p) * 4) = make_float4(wr[0], wr[1], wr[2], wr[3]);
        if (rec.dw4) {
            rec.dbase[list + p] = dbase;
            *reinterpret_cast<float4 *>(rec.dw4 + (list + p) * 4) = make_float4(dwr[0], dwr[1], dwr[2], dwr[3]);
        }
    }
}

// Adds the carry rows of segments 1 .. n_seg-1 to the partial slabs, in segment order.  One thread
// per (chunk, input, output).
__global__ __launch_bounds__(256) void walk_carry_kernel(SplineGeom g, const int *__restrict__ rt,
                                                         const float *__restrict__ carry, float *__restrict__ part_c,
                                                         int L, int n_chunks, int n_seg, int chunk0, int shared)
{
    // n_chunks chunks starting at chunk0 of the batch; shared: the launch's chunk number l adds to slab l
    const int64_t at = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (at >= (int64_t)n_chunks * g.n_in * g.n_out) return;
    const int j = (int)(at % g.n_out);
    const int64_t ci = (int64_t)chunk0 * g.n_in + at / g.n_out;               // chunk * n_in + input
    const int seg_len = L / n_seg;              // L: entries per sorted list
    float *slab = part_c + (shared ? at / g.n_out : ci) * g.rows * g.n_out + j;
    for (int k = 1; k < n_seg; ++k) {
        const int rf = rt[ci * L + (int64_t)k * seg_len] & kRtRowMask;
        const float *cr = carry + ((ci * n_seg + k) * kMaxK) * g.n_out + j;
        for (int s = 0; s < kMaxK; ++s)
            if (rf + s < g.rows) slab[(int64_t)(rf + s) * g.n_out] += cr[(int64_t)s * g.n_out];
    }
}

// plain zero fill (a kernel rather than a memset so that the call sequence can be captured in a graph)
__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ p, int64_t n)
{
    const int64_t at = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (at + 3 < n) {
        *reinterpret_cast<float4 *>(p + at) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    } else {
        for (int64_t e = at; e < n; ++e) p[e] = 0.0f;
    }
}

// gx = sum over the output tiles' partial gx
__global__ __launch_bounds__(256) void gx_sum_kernel(const float *__restrict__ part, float *__restrict__ gx, int64_t n,
                                                     int n_jt)
{
    const int64_t at = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (at >= n) return;
    float v = part[at];
    for (int t = 1; t < n_jt; ++t) v += part[(int64_t)t * n + at];
    gx[at] = v;
}

int log2_exact(int v) { int b = 0; while ((1 << b) < v) ++b; return b; }

}  // namespace

// ---- planning and launch ---------------------------------------------------------------------

WalkPlan plan_walk(const SplineGeom &g, int64_t B, bool allow_shared, bool high_degree)
{
    WalkPlan p = {};
    if (g.rows < kMaxK || g.rows > kRtRowMask || B < 1) return p;
    if (high_degree && g.rows < 6) return p;          // a six-row window must fit the table
    if (g.n_out % 8 == 0 && g.n_out > 256) {
        p.T = 8;            // one tile covers 512 outputs: the per-record work is shared by twice as many
        p.streams = 1;
    } else if (g.n_out % 2 == 0 && g.n_out > 16 && g.n_out <= 32) {
        p.T = 2;            // 16 lanes x 2 outputs cover the layer: no idle lanes in a stream
        p.streams = 4;
    } else if (g.n_out % 4 == 0) {
        p.T = 4;
        p.streams = g.n_out > 128 ? 1 : (g.n_out > 64 ? 2 : 4);
    } else if (g.n_out <= 16) {
        p.T = 1;
        p.streams = 4;
    } else {
        return p;
    }
    const int tile = (64 / p.streams) * p.T;
    p.n_jt = (g.n_out + tile - 1) / tile;
    // chunk length: a power of two between 256 and 8192 samples, the smaller of
    //   - what keeps the gy rows of one chunk inside an XCD's L2 (4 MiB),
    //   - an eighth of the batch (one chunk per XCD at least),
    // then raised until the partial sums fit 2 GiB.  Few, long chunks keep the partial sums small;
    // the parallelism comes from cutting each sorted list into segments (below).
    // (two records per pair for degrees 4 and 5: the sort holds 2 S keys and a record has 12 bits for the sample)
    const int s_max = high_degree ? 4096 : 8192;
    auto pow2_floor = [s_max](int64_t v) { int64_t q = 256; while (q * 2 <= v && q < s_max) q *= 2; return (int)q; };
    int S = pow2_floor((4ll << 20) / ((int64_t)g.n_out * 4));
    if (p.T == 8 && S > 1024) S = 1024;      // eight outputs per lane: stay with single-level sums (registers)
    const int s_b8 = pow2_floor(B / 8);
    S = S < s_b8 ? S : s_b8;
    const int64_t slab = (int64_t)g.n_in * g.rows * g.n_out * (int64_t)sizeof(float);
    while (S < s_max && ((B + S - 1) / S) * slab > (2ll << 30)) S *= 2;
    p.S = S;
    p.hk = high_degree ? 1 : 0;
    p.L = high_degree ? 2 * S : S;
    p.sbits = log2_exact(S);
    p.n_chunks = (int)((B + S - 1) / S);
    // segments per list: enough for about 2048 waves, at least 64 records each
    int bits = 0;
    while ((1 << bits) < g.rows - kMaxK + 1) ++bits;
    p.row_bits = bits < 1 ? 1 : bits;
    p.ok = (int64_t)p.n_chunks * slab <= (4ll << 30) ? 1 : 0;
    p.shared = 0;
    p.n_slabs = p.n_chunks;
    auto plan_segments = [&](int chunks_per_launch) {
        p.n_seg = 1;
        while (p.L / (p.n_seg * 2) >= 64 &&
               (int64_t)chunks_per_launch * p.n_seg * p.n_jt * g.n_in < (int64_t)2048 * p.streams)
            p.n_seg *= 2;
    };
    plan_segments(p.n_chunks);
    // Tables too large for one partial slab per chunk: as many slabs as fit the budget (at least one),
    // the chunks walked in rounds of that many, one launch per round, chunk number l of a round adding its
    // sums to the rows it touches in slab l (the launches are ordered by the stream and every row of a slab
    // has one writer per launch, so the summation order is still fixed).
    if (!p.ok && allow_shared && slab <= (8ll << 30)) {
        p.ok = 1;
        p.shared = 1;
        const int64_t fit = (4ll << 30) / slab;
        p.n_slabs = (int)(fit < 1 ? 1 : (fit > p.n_chunks ? p.n_chunks : fit));
        plan_segments(p.n_slabs);
    }
    return p;
}

// one translation unit per kernel variant (kan_walk_s*t*.hip)
#define KAN_WALK_VARIANT(name)                                                                                      \
    void name(bool dx, unsigned blocks, hipStream_t st, const SplineGeom &g, const WalkRecords &rec, const float *gy, \
              const float *cf, const float *w_b, float *part_c, float *part_b, float *gx, int64_t B,              \
              const WalkPlan &p, int bpc, int m, int prezeroed, float *carry, int chunk0, int n_chunks)
KAN_WALK_VARIANT(walk_launch_s1t8);
KAN_WALK_VARIANT(walk_launch_s1t4);
KAN_WALK_VARIANT(walk_launch_s2t4);
KAN_WALK_VARIANT(walk_launch_s4t4);
KAN_WALK_VARIANT(walk_launch_s4t2);
KAN_WALK_VARIANT(walk_launch_s4t1);
#undef KAN_WALK_VARIANT

namespace {
size_t up256(size_t v) { return (v + 255) / 256 * 256; }
}

// transposed x | records (row|sample, base, weights, derivative base, derivative weights) |
// per-tile partial gx (layers wider than one tile) | carry rows of the list segments
static size_t walk_carry_bytes(const WalkPlan &p, int n_in, int n_out)
{
    return up256((size_t)p.n_chunks * n_in * (p.n_seg + 1) * kMaxK * n_out * sizeof(float));
}

size_t walk_scratch_bytes(const WalkPlan &p, int64_t B, int n_in, int n_out)
{
    const size_t n = (size_t)p.n_chunks * n_in * p.L;
    const int n_part = p.n_jt * (p.hk ? 2 : 1);       // partial dL/dx results per (sample, input)
    const size_t gxp = n_part > 1 ? up256((size_t)n_part * B * n_in * sizeof(float)) : 0;
    return up256((size_t)B * n_in * sizeof(float)) + 3 * up256(n * 4) + 2 * up256(n * 16) + gxp +
           walk_carry_bytes(p, n_in, n_out);
}

// x -> xT, then per (chunk of S samples, input) the records in sorted order.  S: a power of two >= 256.
hipError_t launch_sorted_records(const SplineGeom &g, const float *x, float *xT, int64_t B, int S, int row_bits,
                                 const WalkRecords &rec, hipStream_t st)
{
    {
        dim3 grid((unsigned)((B + 63) / 64), (unsigned)((g.n_in + 63) / 64));
        prof::Timed tm("walk_transpose", st);
        transpose_kernel<<<grid, 256, 0, st>>>(x, xT, B, g.n_in);
    }
    const size_t lds = (size_t)S * 12;
    // waves per sort, measured: 16 for chunks of 8192 samples, 8 for 4096, 4 below
    dim3 grid((unsigned)((B + S - 1) / S), (unsigned)g.n_in);
    prof::Timed tm("walk_sort", st);
    struct W16; struct W8; struct W4;
    hipError_t e;
    if (S >= 8192) {
        auto kern = cell_sort_kernel<16>;
        if ((e = ensure_dynamic_lds<W16>(reinterpret_cast<const void *>(kern), (int)lds)) != hipSuccess) return e;
        kern<<<grid, 1024, lds, st>>>(g, xT, B, S, log2_exact(S), row_bits, rec);
    } else if (S >= 4096) {
        auto kern = cell_sort_kernel<8>;
        if ((e = ensure_dynamic_lds<W8>(reinterpret_cast<const void *>(kern), (int)lds)) != hipSuccess) return e;
        kern<<<grid, 512, lds, st>>>(g, xT, B, S, log2_exact(S), row_bits, rec);
    } else {
        auto kern = cell_sort_kernel<4>;
        if ((e = ensure_dynamic_lds<W4>(reinterpret_cast<const void *>(kern), (int)lds)) != hipSuccess) return e;
        kern<<<grid, 256, lds, st>>>(g, xT, B, S, log2_exact(S), row_bits, rec);
    }
    return hipGetLastError();
}

// gx == nullptr: parameter gradients only.  part_c == nullptr: dL/dx only.  cf is the scale-folded
// table ([n_in][slab_rows][n_out]); w_b may be null when the layer has no base term.
hipError_t launch_backward_walk(const SplineGeom &g, const WalkPlan &p, const float *x, const float *gy,
                                const float *cf, const float *w_b, void *scratch, float *gx, float *part_c,
                                float *part_b, int64_t B, hipStream_t st)
{
    const size_t n = (size_t)p.n_chunks * g.n_in * p.L;
    const int n_part = p.n_jt * (p.hk ? 2 : 1);
    const bool dx = gx != nullptr;
    char *at = (char *)scratch;
    float *xT = (float *)at;            at += up256((size_t)B * g.n_in * sizeof(float));
    WalkRecords rec;
    rec.rt = (int *)at;                 at += up256(n * 4);
    rec.base = (float *)at;             at += up256(n * 4);
    rec.w4 = (float *)at;               at += up256(n * 16);
    rec.dbase = dx ? (float *)at : nullptr; at += up256(n * 4);
    rec.dw4 = dx ? (float *)at : nullptr;   at += up256(n * 16);
    float *gx_part = (float *)at;       at += n_part > 1 ? up256((size_t)n_part * B * g.n_in * sizeof(float)) : 0;
    float *carry = (float *)at;
    if (p.hk) {
        // degrees 4 and 5: the records come from the kernel built for a window of six rows
        {
            dim3 grid((unsigned)((B + 63) / 64), (unsigned)((g.n_in + 63) / 64));
            prof::Timed tm("walk_transpose", st);
            transpose_kernel<<<grid, 256, 0, st>>>(x, xT, B, g.n_in);
        }
        HighKLayer l = {};
        l.n_in = g.n_in; l.n_out = g.n_out; l.rows = g.rows; l.k = g.k; l.lo = g.lo; l.inv_h = g.inv_h; l.base_act = g.base_act;
        l.slab_rows = g.slab_rows; l.cell_base = g.cell_base;
        if (hipError_t e = highk_sorted_records(l, xT, B, p.S, p.row_bits, rec.rt, rec.base, rec.w4, rec.dbase, rec.dw4, st);
            e != hipSuccess)
            return e;
    } else if (hipError_t e = launch_sorted_records(g, x, xT, B, p.S, p.row_bits, rec, st); e != hipSuccess) {
        return e;
    }
    const int bpc = (p.n_seg * p.n_jt * g.n_in + 4 * p.streams - 1) / (4 * p.streams);
    float *gx_out = dx ? (n_part > 1 ? gx_part : gx) : nullptr;
    // Sparse regime (far more rows than a chunk has samples): most rows of a chunk's partial slab
    // receive nothing.  The slab is zeroed with a streaming fill and the walk skips the gaps instead of
    // stepping through them row by row.  A shared slab is always used this way.
    const int prezeroed = (part_c != nullptr && (g.rows > 2 * p.S || p.shared)) ? 1 : 0;
    if (prezeroed) {
        const int64_t n4 = (int64_t)p.n_slabs * g.n_in * g.rows * g.n_out;
        prof::Timed tm("walk_zero_fill", st);
        fill_zero_kernel<<<(unsigned)((n4 + 1023) / 1024), 256, 0, st>>>(part_c, n4);
    }
    // one launch for all chunks, or (shared slabs) one launch per round of n_slabs chunks, each followed by
    // its carry rows
    const int per_launch = p.shared ? p.n_slabs : p.n_chunks;
    const int launches = (p.n_chunks + per_launch - 1) / per_launch;
    int m = 1;
    while (m * 2 <= 8 && m * 2 <= per_launch) m *= 2;
    const int bpc_sub = (bpc + 8 / m - 1) / (8 / m);
    const unsigned blocks = (unsigned)(8 * bpc_sub * ((per_launch + m - 1) / m));
    for (int l = 0; l < launches; ++l) {
        const int chunk0 = l * per_launch;
        const int here = p.n_chunks - chunk0 < per_launch ? p.n_chunks - chunk0 : per_launch;
        {
            prof::Timed tm(dx ? "backward_walk" : "dparam_walk", st);
            if (p.T == 8 && p.streams == 1)
                walk_launch_s1t8(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry, chunk0, here);
            else if (p.T == 4 && p.streams == 1)
                walk_launch_s1t4(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry, chunk0, here);
            else if (p.T == 4 && p.streams == 2)
                walk_launch_s2t4(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry, chunk0, here);
            else if (p.T == 4 && p.streams == 4)
                walk_launch_s4t4(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry, chunk0, here);
            else if (p.T == 2 && p.streams == 4)
                walk_launch_s4t2(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry, chunk0, here);
            else if (p.T == 1 && p.streams == 4)
                walk_launch_s4t1(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry, chunk0, here);
            else
                return hipErrorInvalidValue;
        }
        if (part_c != nullptr && p.n_seg > 1) {
            const int64_t nn = (int64_t)here * g.n_in * g.n_out;
            prof::Timed tm("walk_carry", st);
            walk_carry_kernel<<<(unsigned)((nn + 255) / 256), 256, 0, st>>>(g, rec.rt, carry, part_c, p.L, here,
                                                                           p.n_seg, chunk0, p.shared);
        }
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    if (dx && n_part > 1) {
        const int64_t nn = B * g.n_in;
        prof::Timed tm("walk_gx_sum", st);
        gx_sum_kernel<<<(unsigned)((nn + 255) / 256), 256, 0, st>>>(gx_part, gx, nn, n_part);
    }
    return hipGetLastError();
}

}  // namespace kan
