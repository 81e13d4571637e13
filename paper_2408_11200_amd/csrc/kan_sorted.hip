// Backward kernels for small grids, built on per-input sorted pair records.
//
// A pre-pass evaluates every (sample, input) pair once and, for every tile of 64 samples and every
// input, writes the 64 pair records sorted by window row (stable rank, so the order is fixed).  The
// consumer kernels give each wave ONE input for a whole chunk of the batch: because the records of a
// tile arrive in row order, the wave walks the rows with a statically unrolled loop and keeps
// everything that is indexed by the row (the parameter-gradient accumulators, or the coefficient
// rows for dL/dx) in statically named registers.  A tile's 64 records sit one per lane and are
// broadcast lane by lane into scalar registers; dL/dcoef is reduced without atomics in a fixed order.
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace kan {

namespace {

constexpr int kTile = 64;          // samples per tile = lanes per wave

}  // namespace

// ---- pre-pass: pair records ----------------------------------------------------------------------
// grid (tiles, ceil(n_in / 64)); block = 4 waves.  The block loads a 64 x 64 tile of x through LDS
// (coalesced rows), then each wave takes 16 of the inputs; lane t is sample t of the tile and writes its
// record at [tile][input][rank of its window row among the 64].  rec_w: value records;
// rec_d: derivative records; either may be null.  Samples past the end of the batch get records
// that contribute nothing.
__global__ __launch_bounds__(256) void pair_record_kernel(SplineGeom g, const float *__restrict__ x, int64_t B,
                                                          PairRecord *__restrict__ rec_w,
                                                          PairRecord *__restrict__ rec_d)
{
    __shared__ float xs[kTile][kTile + 1];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t tile = blockIdx.x;
    const int64_t b0 = tile * kTile;
    const int i0 = blockIdx.y * kTile;
    for (int e = tid; e < kTile * kTile; e += 256) {
        const int t = e / kTile, ii = e % kTile;
        const int64_t b = b0 + t;
        const int i = i0 + ii;
        xs[t][ii] = (b < B && i < g.n_in) ? x[b * g.n_in + i] : 0.0f;
    }
    __syncthreads();
    const bool live = b0 + lane < B;
    for (int ii = wave; ii < kTile; ii += 4) {
        const int i = i0 + ii;
        if (i >= g.n_in) break;
        Pair p = pair_eval<true>(xs[lane][ii], g, i);
        if (!live) {
            p.cell = -kMaxK;
#pragma unroll
            for (int s = 0; s < kMaxK; ++s) { p.w[s] = 0.0f; p.dw[s] = 0.0f; }
            p.base = 0.0f; p.dbase = 0.0f;
        }
        int row0;
        float w[kMaxK], dw[kMaxK], base, dbase;
        window_of<false>(p, g.rows, row0, w, base);
        window_of<true>(p, g.rows, row0, dw, dbase);
        // stable rank of this lane's row among the 64 rows of the tile
        int rank = 0;
        for (int l2 = 0; l2 < kTile; ++l2) {
            const int k2 = lane_i(row0, l2);
            rank += (k2 < row0 || (k2 == row0 && l2 < lane)) ? 1 : 0;
        }
        const int64_t at = (tile * g.n_in + i) * kTile + rank;
        if (rec_w) {
            PairRecord r;
            r.rt = row0 | (lane << 16); r.base = base;
#pragma unroll
            for (int s = 0; s < kMaxK; ++s) r.w[s] = w[s];
            rec_w[at] = r;
        }
        if (rec_d) {
            PairRecord r;
            r.rt = row0 | (lane << 16); r.base = dbase;
#pragma unroll
            for (int s = 0; s < kMaxK; ++s) r.w[s] = dw[s];
            rec_d[at] = r;
        }
    }
}

// ---- dL/dcoef, dL/dw_s, dL/dw_b: partial sums per batch chunk ---------------------------------
// Work item = (input i, block of ROWS coefficient rows); a workgroup of NW waves takes NW consecutive
// items (grid.x), one j-tile of 256 outputs (grid.y) and one chunk of the batch (grid.z).  The gy tile
// (64 samples x 256 outputs) of the current sample tile is shared through LDS, double-buffered.
// acc[m] collects   sum_b gy[b][j] * N_{m - row(b,i)}(u(b,i))   over the chunk for the rows
// lo .. lo+ROWS-1 of the item, in registers.  A record whose window starts at row lo + d touches the
// item's rows for d in -3 .. ROWS-1; because the records of a tile are sorted by row, those records are
// one contiguous run (found with a ballot), and the run is walked with a loop that is statically
// unrolled over d, so every accumulator index is a compile-time constant.  Results go to
// part_c[chunk][i][m][j]; the base-term sums (taken by the item that holds the record's first row)
// to part_b[chunk * blocks + block][i][j]; both are reduced over chunks in fixed order in fp64.
template <int ROWS, int NW>
__global__ __launch_bounds__(64 * NW) void dparam_sorted_kernel(SplineGeom g, const PairRecord *__restrict__ rec,
                                                                const float *__restrict__ gy,
                                                                float *__restrict__ part_c,
                                                                float *__restrict__ part_b, int64_t B,
                                                                int64_t tiles_per_chunk, int n_rb)
{
    constexpr int TJ = 256, NT = 64 * NW;
    extern __shared__ float lds[];                      // 2 x [64][256]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int item = blockIdx.x * NW + wave;
    const bool have_item = item < g.n_in * n_rb;
    const int i = have_item ? item / n_rb : g.n_in - 1;
    const int rb = have_item ? item % n_rb : 0;
    const int lo = rb * ROWS;
    const int j0 = blockIdx.y * TJ;
    const int j = j0 + lane * 4;
    const int64_t n_tiles = (B + kTile - 1) / kTile;
    const int64_t tile_lo = (int64_t)blockIdx.z * tiles_per_chunk;
    const int64_t tile_hi = tile_lo + tiles_per_chunk < n_tiles ? tile_lo + tiles_per_chunk : n_tiles;
    if (tile_lo >= tile_hi) return;

    float acc[ROWS][4], accb[4];
#pragma unroll
    for (int m = 0; m < ROWS; ++m)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[m][r] = 0.0f;
#pragma unroll
    for (int r = 0; r < 4; ++r) accb[r] = 0.0f;

    // gy tile copy straight from global memory into LDS (no registers): one row of the tile is 256
    // floats = 64 lanes x 16 bytes = one wave-wide global_load_lds_dwordx4.  Rows past the end of the
    // batch and columns past n_out are not copied; LDS is zeroed once so that what they leave behind
    // is finite (their records have zero weights / their lanes store nothing).
    for (int e = tid; e < 2 * kTile * TJ / 4; e += NT)
        *reinterpret_cast<float4 *>(lds + (int64_t)e * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
    auto copy_tile = [&](int64_t tile, float *buf) {
        for (int t = wave; t < kTile; t += NW) {
            const int64_t b = tile * kTile + t;
            if (b < B && j < g.n_out)
                __builtin_amdgcn_global_load_lds(gy + b * g.n_out + j,
                                                 (__attribute__((address_space(3))) void *)(buf + t * TJ), 16, 0, 0);
        }
    };
    copy_tile(tile_lo, lds);
    // this lane's record of the current tile; the next tile's is fetched while the current is used
    PairRecord mine = rec[(tile_lo * g.n_in + i) * kTile + lane];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int64_t tile = tile_lo; tile < tile_hi; ++tile) {
        const float *cur = lds + ((tile - tile_lo) & 1) * (kTile * TJ) + lane * 4;
        float *nxt = lds + ((tile - tile_lo + 1) & 1) * (kTile * TJ);
        const int64_t tile_next = tile + 1 < tile_hi ? tile + 1 : tile;
        copy_tile(tile_next, nxt);
        const PairRecord upcoming = rec[(tile_next * g.n_in + i) * kTile + lane];
        if (have_item) {
            // the records whose window touches this item's rows: a contiguous run of the sorted list
            const int r0 = mine.rt & 0xffff;
            const unsigned long long hit = __ballot(r0 + kMaxK > lo && r0 < lo + ROWS);
            if (hit) {
                int pos = __builtin_ctzll(hit);
                const int end = pos + __builtin_popcountll(hit);
                int rt = lane_i(mine.rt, pos);
#pragma unroll
                for (int d = 1 - kMaxK; d < ROWS; ++d) {        // window start relative to the item's rows
                    while (pos < end && (rt & 0xffff) == lo + d) {
                        const float4 gv = *reinterpret_cast<const float4 *>(cur + (rt >> 16) * TJ);
                        const float gr[4] = {gv.x, gv.y, gv.z, gv.w};
                        float ws[kMaxK];
#pragma unroll
                        for (int s = 0; s < kMaxK; ++s) ws[s] = lane_f(mine.w[s], pos);
                        const float bs = lane_f(mine.base, pos);
                        ++pos;
                        rt = lane_i(mine.rt, pos & (kTile - 1));
#pragma unroll
                        for (int s = 0; s < kMaxK; ++s) {
                            if (d + s >= 0 && d + s < ROWS) {
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    acc[d + s < 0 ? 0 : d + s][r] = fmaf(ws[s], gr[r], acc[d + s < 0 ? 0 : d + s][r]);
                            }
                        }
                        if (d >= 0) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) accb[r] = fmaf(bs, gr[r], accb[r]);
                        }
                    }
                }
            }
        }
        mine = upcoming;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    if (!have_item || j >= g.n_out) return;
    float *pc = part_c + (((int64_t)blockIdx.z * g.n_in + i) * g.rows) * g.n_out + j;
#pragma unroll
    for (int m = 0; m < ROWS; ++m)
        if (lo + m < g.rows)
            *reinterpret_cast<float4 *>(pc + (int64_t)(lo + m) * g.n_out) =
                make_float4(acc[m][0], acc[m][1], acc[m][2], acc[m][3]);
    if (part_b)
        *reinterpret_cast<float4 *>(part_b + (((int64_t)blockIdx.z * n_rb + rb) * g.n_in + i) * g.n_out + j) =
            make_float4(accb[0], accb[1], accb[2], accb[3]);
}

// ---- launch ---------------------------------------------------------------------------------

int sorted_rows_template(int rows)
{
    if (rows < kMaxK) return 0;
    return rows <= 16 ? 16 : 24;
}

// row blocks per input = base-term partial slices per chunk
int dparam_sorted_row_blocks(int rows)
{
    const int t = sorted_rows_template(rows);
    return t ? (rows + t - 1) / t : 0;
}

int dparam_sorted_waves(int rows) { (void)rows; return 16; }

int backward_sorted_applicable(const SplineGeom &g)
{
    return (sorted_rows_template(g.rows) != 0 && g.rows <= 0xffff && g.n_out % 4 == 0 && g.n_out >= 64) ? 1 : 0;
}

size_t pair_record_bytes(int64_t B, int n_in)
{
    const int64_t tiles = (B + kTile - 1) / kTile;
    return (size_t)((tiles * n_in * kTile + 4) * (int64_t)sizeof(PairRecord));
}

hipError_t launch_pair_records(const SplineGeom &g, const float *x, int64_t B, PairRecord *rec_w, PairRecord *rec_d,
                            hipStream_t st)
{
    const int64_t tiles = (B + kTile - 1) / kTile;
    dim3 grid((unsigned)tiles, (unsigned)((g.n_in + kTile - 1) / kTile));
    prof::Timed tm("pair_records", st);
    pair_record_kernel<<<grid, 256, 0, st>>>(g, x, B, rec_w, rec_d);
    return hipGetLastError();
}

template <int ROWS, int NW>
static hipError_t dparam_sorted_launch(const SplineGeom &g, const PairRecord *rec, const float *gy, float *part_c,
                                       float *part_b, int64_t B, int n_chunks, int64_t chunk_len, hipStream_t st)
{
    const size_t lds = 2ull * kTile * 256 * sizeof(float);
    auto kern = dparam_sorted_kernel<ROWS, NW>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int n_rb = (g.rows + ROWS - 1) / ROWS;
    dim3 grid((unsigned)((g.n_in * n_rb + NW - 1) / NW), (unsigned)((g.n_out + 255) / 256), (unsigned)n_chunks);
    prof::Timed tm("dparam_sorted", st);
    kern<<<grid, 64 * NW, lds, st>>>(g, rec, gy, part_c, part_b, B, chunk_len / kTile, n_rb);
    return hipGetLastError();
}

// chunk_len must be a multiple of 64 (whole tiles per chunk)
hipError_t launch_dparam_sorted(const SplineGeom &g, const PairRecord *rec, const float *gy, float *part_c,
                                float *part_b, int64_t B, int n_chunks, int64_t chunk_len, hipStream_t st)
{
    switch (sorted_rows_template(g.rows)) {
    case 16: return dparam_sorted_launch<16, 16>(g, rec, gy, part_c, part_b, B, n_chunks, chunk_len, st);
    case 24: return dparam_sorted_launch<24, 16>(g, rec, gy, part_c, part_b, B, n_chunks, chunk_len, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kan
