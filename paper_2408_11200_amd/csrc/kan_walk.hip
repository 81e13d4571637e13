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
#include <type_traits>
#include "kan_device.hpp"
#include "kan_launch.hpp"

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
    __shared__ unsigned wave_tot[4];
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
        // the first 256 threads (one digit each)
        unsigned tot = 0, inc = 0;
        if (tid < 256) {
            for (int w2 = 0; w2 < NW; ++w2) tot += slot[w2][tid];
            inc = tot;
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned v = __shfl_up(inc, o, 64);
                if (lane >= o) inc += v;
            }
            if (lane == 63) wave_tot[wave] = inc;
        }
        __syncthreads();
        if (tid < 256) {
            unsigned at = inc - tot;
            for (int w2 = 0; w2 < wave; ++w2) at += wave_tot[w2];
            for (int w2 = 0; w2 < NW; ++w2) {
                const unsigned cnt = slot[w2][tid];
                slot[w2][tid] = at;
                at += cnt;
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
        rec.rt[list + p] = row0 | ((live ? e : 0) << 16);
        rec.base[list + p] = base;
        *reinterpret_cast<float4 *>(rec.w4 + (list + p) * 4) = make_float4(wr[0], wr[1], wr[2], wr[3]);
        if (rec.dw4) {
            rec.dbase[list + p] = dbase;
            *reinterpret_cast<float4 *>(rec.dw4 + (list + p) * 4) = make_float4(dwr[0], dwr[1], dwr[2], dwr[3]);
        }
    }
}

// ---- 3. walk -------------------------------------------------------------------------------
template <int N>
__device__ __forceinline__ int row_bcast(int v)        // value of lane N of the caller's row of 16 lanes
{
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + N, 0xF, 0xF, true);
}
template <int N>
__device__ __forceinline__ float row_bcast(float v)
{
    return __builtin_bit_cast(float, row_bcast<N>(__builtin_bit_cast(int, v)));
}

// value of the partner lane for the level that pairs lanes differing in bit D (for D = 4 the partner
// is lane ^ 7: it differs in bit 2, which is all the reduction below needs)
template <int D>
__device__ __forceinline__ float partner(float v)
{
    const int iv = __builtin_bit_cast(int, v);
    if constexpr (D >= 16) return __shfl_xor(v, D, 64);
    else if constexpr (D == 8) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, 0x128, 0xF, 0xF, true));
    else if constexpr (D == 4) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, 0x141, 0xF, 0xF, true));
    else if constexpr (D == 2) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, 0x4E, 0xF, 0xF, true));
    else return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, 0xB1, 0xF, 0xF, true));
}

// p[0..N) hold, per lane, partial sums of N quantities.  Sums them over groups of LPS lanes while
// halving the number of quantities a lane carries at each level (lanes whose bit D is set keep the
// upper half); once one is left the remaining levels are plain sums.  Returns the total of quantity
// number quantity_of<LPS>(lane).
template <int D, int N>
__device__ __forceinline__ float reduce_levels(float (&p)[N], int lane)
{
    if constexpr (N > 1) {
        const bool up = (lane & D) != 0;
        float h[N / 2];
#pragma unroll
        for (int k = 0; k < N / 2; ++k) {
            const float keep = up ? p[k + N / 2] : p[k];
            const float send = up ? p[k] : p[k + N / 2];
            h[k] = keep + partner<D>(send);
        }
        if constexpr (D > 1) return reduce_levels<D / 2, N / 2>(h, lane);
        else return h[0];
    } else {
        float v = p[0] + partner<D>(p[0]);
        if constexpr (D > 1) {
            float one[1] = {v};
            return reduce_levels<D / 2, 1>(one, lane);
        } else {
            return v;
        }
    }
}
template <int LPS>
__device__ __forceinline__ int quantity_of(int lane)      // 16 quantities: the top four levels select
{
    return (lane / (LPS / 16)) & 15;
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
__device__ __forceinline__ void load_vec(const float *p, float (&v)[T])
{
    if constexpr (T == 8) {
        const float4 t = *reinterpret_cast<const float4 *>(p), u = *reinterpret_cast<const float4 *>(p + 4);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; v[4] = u.x; v[5] = u.y; v[6] = u.z; v[7] = u.w;
    } else if constexpr (T == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        static_assert(T == 1, "one, four or eight outputs per lane");
        v[0] = *p;
    }
}
template <int T>
__device__ __forceinline__ void store_vec(float *p, const float (&v)[T])
{
    if constexpr (T == 8) {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else if constexpr (T == 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        p[0] = v[0];
    }
}

// 4 waves per block, STREAMS streams per wave.  Per record: one gather of the sample's gy row
// (T floats per lane), T matrix-core instructions for the K window rows, T multiply-adds for the
// base term.  Sums are kept in two levels (the running sums are folded into a second set every 256
// records) so that a long run of samples in one cell does not lose accuracy to sequential fp32
// accumulation.
//
// DX: the same walk also produces dL/dx.  The K rows of the scale-folded table under the window
// slide along in registers with the accumulators (one row is loaded per step of the window), so a
// record costs another (K + 1) * T multiply-adds for  q_j = sum_s dw_s c[row+s][j] + dbase w_b[j]
// and T for gy . q; the per-lane partial dot products of 16 records are summed over the stream's lanes
// together (reduce_levels) and scattered to gx[sample][i] (gx_part[jt] when the layer has several
// output tiles; those are added up by gx_sum_kernel).
typedef float f32x4 __attribute__((ext_vector_type(4)));

// acc[s] += A[s] * b for s = 0..3, where A is the quadruple held by lanes 4*ABID .. 4*ABID+3 of the
// caller's group of 2^CBSZ blocks of four lanes (the whole wave for CBSZ = 4).
template <int CBSZ, int ABID>
__device__ __forceinline__ void rank1_update(f32x4 &acc, float a_quads, float b)
{
    acc = __builtin_amdgcn_mfma_f32_4x4x1f32(a_quads, b, acc, CBSZ, ABID, 0);
}

template <int STREAMS, int T, bool DX, bool FOLD>
__global__ __launch_bounds__(256) void backward_walk_kernel(SplineGeom g, WalkRecords rec,
                                                            const float *__restrict__ gy,
                                                            const float *__restrict__ cf,
                                                            const float *__restrict__ w_b,
                                                            float *__restrict__ part_c, float *__restrict__ part_b,
                                                            float *__restrict__ gx, int64_t B, int S, int n_chunks,
                                                            int n_jt, int blocks_per_chunk, int xcd_groups, int prezeroed, int n_seg,
                                                            float *__restrict__ carry)
{
    constexpr int LPS = 64 / STREAMS;
    constexpr int RPW = LPS / 4;                    // records whose weights fit one register of a stream
    constexpr int CBSZ = STREAMS == 1 ? 4 : (STREAMS == 2 ? 3 : 2);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane / LPS, q = lane % LPS, r16 = lane & 15;
    // Workgroups go to the 8 XCDs round-robin.  The XCDs form m = min(8, n_chunks) groups (m a power of
    // two); chunk c is handled by group c % m only, so that the gy rows a chunk's streams gather
    // (every input re-reads them) stay in the L2 of the XCDs of one group.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int grp = xcd % xcd_groups, n_sub = 8 / xcd_groups, sub_x = xcd / xcd_groups;
    const int bpc_sub = (blocks_per_chunk + n_sub - 1) / n_sub;
    const int c = grp + xcd_groups * (slot / bpc_sub);
    const int blk = (slot % bpc_sub) * n_sub + sub_x;
    const int ws = (blk * 4 + wave) * STREAMS + sub;
    if (c >= n_chunks || blk >= blocks_per_chunk || ws >= n_seg * n_jt * g.n_in) return;
    const int i = ws % g.n_in;
    const int jt = (ws / g.n_in) % n_jt;
    const int seg = ws / (g.n_in * n_jt);
    const int seg_len = S / n_seg;                  // a multiple of 16
    const int j = (jt * LPS + q) * T;
    const bool jok = j < g.n_out;
    const int jc = jok ? j : 0;
    const int64_t b0 = (int64_t)c * S;
    const int n_c = (int)((B - b0) < S ? (B - b0) : S);
    const int64_t list0 = ((int64_t)c * g.n_in + i) * S;
    const int64_t list = list0 + (int64_t)seg * seg_len;        // this segment's records
    // The segment owns the table rows from its first record's row up to the next segment's first
    // row; what its window holds beyond that at the end goes to the next segment's carry rows.
    const int r_next = seg + 1 < n_seg ? (rec.rt[list + seg_len] & 0xffff) : g.rows;
    const float *gyp = gy + b0 * g.n_out + jc;
    const bool store_c = jok && part_c != nullptr;
    float *out = part_c + ((int64_t)c * g.n_in + i) * g.rows * g.n_out + jc;
    const float *cfi = DX ? cf + (int64_t)i * g.slab_rows * g.n_out + jc : nullptr;
    float *gxo = DX ? gx + (int64_t)jt * B * g.n_in + b0 * g.n_in + i : nullptr;

    // a[r][s]: running sum of output j + r, window row cur + s; hi: the second level
    // (FOLD == false: chunks of at most 1024 samples, one level is accurate enough and the registers
    // of the second go to keeping more gy rows in flight)
    constexpr int TH = FOLD ? T : 1;
    f32x4 a[T], hi[TH];
    float ab[T], abh[TH], zero[T];
#pragma unroll
    for (int r = 0; r < T; ++r) {
        ab[r] = 0.0f; zero[r] = 0.0f;
        a[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
#pragma unroll
    for (int r = 0; r < TH; ++r) {
        abh[r] = 0.0f;
        hi[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    int cur = rec.rt[list] & 0xffff;         // first row of the window the accumulators stand on
    if (store_c && !prezeroed && seg == 0)
        for (int m = 0; m < cur; ++m) store_vec<T>(out + (int64_t)m * g.n_out, zero);

    // dL/dx: table rows cur .. cur+K-1 and the w_b row, zero in lanes past the last output
    float cw[kMaxK][T], wb[T];
    const float jmask = jok ? 1.0f : 0.0f;
    if constexpr (DX) {
#pragma unroll
        for (int r = 0; r < T; ++r) wb[r] = 0.0f;
        if (jok && w_b != nullptr && g.base_act != 0) load_vec<T>(w_b + (int64_t)i * g.n_out + j, wb);
    }

    // The window rows live in a ring: row m of the table is component m mod K of a[r] / hi[r] (and of
    // cw for dL/dx); the records carry their weights in the same arrangement.  retire() completes the
    // first row of the window: stores it (store == false: returns it in `gone` only), clears its
    // component and, for dL/dx, loads the table row that enters the window in its place.
    float gone[T];
    auto retire_slot = [&](auto sl, bool store, bool enter_next) {
        constexpr int SL = decltype(sl)::value;
#pragma unroll
        for (int r = 0; r < T; ++r) {
            gone[r] = a[r][SL];
            a[r][SL] = 0.0f;
            if constexpr (FOLD) {
                gone[r] += hi[r][SL];
                hi[r][SL] = 0.0f;
            }
        }
        if (store && store_c) store_vec<T>(out + (int64_t)cur * g.n_out, gone);
        if (DX && enter_next) {
            const int enter = cur + kMaxK < g.rows ? cur + kMaxK : g.rows - 1;     // clamped: unused past the end
            load_vec<T>(cfi + (int64_t)enter * g.n_out, cw[SL]);
#pragma unroll
            for (int r = 0; r < T; ++r) cw[SL][r] *= jmask;
        }
    };
    auto retire = [&](bool store, bool enter_next) {
        switch (cur & (kMaxK - 1)) {
        case 0: retire_slot(std::integral_constant<int, 0>{}, store, enter_next); break;
        case 1: retire_slot(std::integral_constant<int, 1>{}, store, enter_next); break;
        case 2: retire_slot(std::integral_constant<int, 2>{}, store, enter_next); break;
        default: retire_slot(std::integral_constant<int, 3>{}, store, enter_next); break;
        }
        ++cur;
    };
    auto reload_table_rows = [&]() {
        if constexpr (DX) {
#pragma unroll
            for (int s = 0; s < kMaxK; ++s) {
                // component s holds the row of the window that is congruent to s
                const int row = cur + ((s - cur) & (kMaxK - 1));
                load_vec<T>(cfi + (int64_t)row * g.n_out, cw[s]);
#pragma unroll
                for (int r = 0; r < T; ++r) cw[s][r] *= jmask;
            }
        }
    };

    // one batch of 16 records as the lanes hold it: row | sample and base value of record r16, the
    // weight quadruples of the stream's 16 records spread over STREAMS registers (lane q of register u
    // holds float number u * LPS + q of the batch's 64), the derivative record of r16
    struct Batch {
        int rt;
        float base;
        float wq[STREAMS];
        float dw[kMaxK];
        float dbase;
    };
    auto load_batch = [&](int bi) {
        Batch t;
        const int64_t at = list + (int64_t)bi * 16;
        t.rt = rec.rt[at + r16];
        t.base = rec.base[at + r16];
#pragma unroll
        for (int u = 0; u < STREAMS; ++u) t.wq[u] = rec.w4[at * 4 + u * LPS + q];
        if constexpr (DX) {
            const float4 d = *reinterpret_cast<const float4 *>(rec.dw4 + (at + r16) * 4);
            t.dw[0] = d.x; t.dw[1] = d.y; t.dw[2] = d.z; t.dw[3] = d.w;
            t.dbase = rec.dbase[at + r16];
        }
        return t;
    };

    reload_table_rows();

    // every record of the segment is walked, the padding behind the last sample of a ragged chunk
    // included (zero weights, sorted last)
    const int nb = seg_len / 16;
    Batch mine = load_batch(0);
    float gbuf[2][4][T];
    auto gather = [&](int tv_of_batch, auto h, float (&dst)[4][T]) {
        constexpr int H = decltype(h)::value;
        static_for<0, 4>([&](auto n) {
            constexpr int N = decltype(n)::value;
            const int t = row_bcast<H * 4 + N>(tv_of_batch);
            load_vec<T>(gyp + (int64_t)t * g.n_out, dst[N]);
        });
    };
    gather((int)((unsigned)mine.rt >> 16), std::integral_constant<int, 0>{}, gbuf[0]);
    for (int bi = 0; bi < nb; ++bi) {
        const Batch upcoming = load_batch(bi + 1 < nb ? bi + 1 : bi);
        const int rowv = mine.rt & 0xffff, tv = (int)((unsigned)mine.rt >> 16);
        float dot[16];
        bool quad_same = false;
        // The 16 records go in groups of four.  The gy rows of the next group (the first of the next
        // batch after the last) are requested before the current group is worked on.
        constexpr int GROUP = 4;
        auto group = [&](auto h) {
            constexpr int H = decltype(h)::value;
            auto &gr = gbuf[H & 1];
            if constexpr (H + 1 < 16 / GROUP) gather(tv, std::integral_constant<int, H + 1>{}, gbuf[(H + 1) & 1]);
            else gather((int)((unsigned)upcoming.rt >> 16), std::integral_constant<int, 0>{}, gbuf[0]);
            static_for<0, GROUP>([&](auto n) {
                constexpr int N = decltype(n)::value;
                constexpr int R = H * GROUP + N;
                const int row0 = row_bcast<R>(rowv);
                if (row0 - cur >= kMaxK) {
                    // the window jumps clear of its old position: write it out whole and start afresh
                    // (rows in between are zero: stored here, or already zero when the slab was pre-zeroed)
                    const int from = cur + kMaxK;
#pragma unroll
                    for (int s = 0; s < kMaxK; ++s) retire(true, false);
                    if (store_c && !prezeroed)
                        for (int m = from; m < row0; ++m) store_vec<T>(out + (int64_t)m * g.n_out, zero);
                    cur = row0;
                    if constexpr (DX) reload_table_rows();
                }
#pragma clang loop unroll(disable)
                while (cur < row0) retire(true, true);
                const float bs = row_bcast<R>(mine.base);
#pragma unroll
                for (int r = 0; r < T; ++r) {
                    rank1_update<CBSZ, R % RPW>(a[r], mine.wq[R / RPW], gr[N][r]);
                    ab[r] = fmaf(bs, gr[N][r], ab[r]);
                    asm volatile("" : "+v"(ab[r]));     // keep the base term with its record (see below)
                }
                if constexpr (DX) {
                    // Four consecutive records with the same window (the common case on small grids, where
                    // a cell holds many samples of the chunk) share the table rows: their
                    // q_j = sum_s dw_s c_s[j] + dbase w_b[j] are rank-1 updates again, one matrix-core
                    // instruction per window row and output register for all four (A = the four records'
                    // dw_s, broadcast from the lanes that hold them; B = the lane's table entry).
                    if constexpr (R % 4 == 0) quad_same = row_bcast<R>(rowv) == row_bcast<R + 3>(rowv);
                    if (!quad_same) {
                        const float d0 = row_bcast<R>(mine.dw[0]), d1 = row_bcast<R>(mine.dw[1]);
                        const float d2 = row_bcast<R>(mine.dw[2]), d3 = row_bcast<R>(mine.dw[3]);
                        const float db = row_bcast<R>(mine.dbase);
                        float acc = 0.0f;
#pragma unroll
                        for (int r = 0; r < T; ++r) {
                            float qv = d0 * cw[0][r];
                            qv = fmaf(d1, cw[1][r], qv);
                            qv = fmaf(d2, cw[2][r], qv);
                            qv = fmaf(d3, cw[3][r], qv);
                            qv = fmaf(db, wb[r], qv);
                            acc = fmaf(gr[N][r], qv, acc);
                        }
                        // pin the dot product here: left alone, the compiler sinks all sixteen of them below
                        // the last record and keeps a copy of the table rows per record alive until then
                        asm volatile("" : "+v"(acc));
                        dot[R] = acc;
                    }
                    if constexpr (R % 4 == 3) {
                        if (quad_same) {
                            float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                            for (int r = 0; r < T; ++r) {
                                f32x4 qv = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                                for (int s = 0; s < kMaxK; ++s) rank1_update<CBSZ, R / 4>(qv, mine.dw[s], cw[s][r]);
                                rank1_update<CBSZ, R / 4>(qv, mine.dbase, wb[r]);
#pragma unroll
                                for (int u = 0; u < 4; ++u) acc[u] = fmaf(gr[N - 3 + u][r], qv[u], acc[u]);
                            }
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                asm volatile("" : "+v"(acc[u]));
                                dot[R - 3 + u] = acc[u];
                            }
                        }
                    }
                }
            });
        };
        static_for<0, 16 / GROUP>(group);
        if constexpr (DX) {
            const float total = reduce_levels<LPS / 2, 16>(dot, lane);
            const int qn = quantity_of<LPS>(lane);
            const int t = __shfl(tv, (lane & ~15) | qn, 64);
            if ((lane % (LPS / 16)) == 0 && seg * seg_len + bi * 16 + qn < n_c) gxo[(int64_t)t * g.n_in] = total;
        }
        if constexpr (FOLD) {
            if ((bi & 15) == 15) {
#pragma unroll
                for (int r = 0; r < T; ++r) {
                    hi[r] += a[r];
                    a[r] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                    abh[r] += ab[r]; ab[r] = 0.0f;
                }
            }
        }
        mine = upcoming;
    }

    if (!store_c) return;
    // what the window still holds: rows below r_next belong to this segment, the others to the next
    // segment's carry rows (carry row s2 stands for table row r_next + s2)
    float *cr = carry + ((((int64_t)c * g.n_in + i) * n_seg + seg + 1) * kMaxK) * g.n_out + jc;
    const int last = cur + kMaxK;            // one past the window
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) {
        const int row = cur;
        retire(row < r_next, false);
        if (row >= r_next && seg + 1 < n_seg) store_vec<T>(cr + (int64_t)(row - r_next) * g.n_out, gone);
    }
    if (seg + 1 < n_seg)
        for (int s2 = (last > r_next ? last - r_next : 0); s2 < kMaxK; ++s2) store_vec<T>(cr + (int64_t)s2 * g.n_out, zero);
    if (!prezeroed)
        for (int m = last; m < r_next; ++m) store_vec<T>(out + (int64_t)m * g.n_out, zero);
    if (part_b) {
        float o[T];
#pragma unroll
        for (int r = 0; r < T; ++r) o[r] = FOLD ? ab[r] + abh[r < TH ? r : 0] : ab[r];
        store_vec<T>(part_b + (((int64_t)c * n_seg + seg) * g.n_in + i) * g.n_out + jc, o);
    }
}

// Adds the carry rows of segments 1 .. n_seg-1 to the partial slabs, in segment order.  One thread
// per (chunk, input, output).
__global__ __launch_bounds__(256) void walk_carry_kernel(SplineGeom g, const int *__restrict__ rt,
                                                         const float *__restrict__ carry, float *__restrict__ part_c,
                                                         int S, int n_chunks, int n_seg)
{
    const int64_t at = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (at >= (int64_t)n_chunks * g.n_in * g.n_out) return;
    const int j = (int)(at % g.n_out);
    const int64_t ci = at / g.n_out;               // chunk * n_in + input
    const int seg_len = S / n_seg;
    float *slab = part_c + ci * g.rows * g.n_out + j;
    for (int k = 1; k < n_seg; ++k) {
        const int rf = rt[ci * S + (int64_t)k * seg_len] & 0xffff;
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

WalkPlan plan_walk(const SplineGeom &g, int64_t B)
{
    WalkPlan p = {};
    if (g.rows < kMaxK || g.rows > 0xffff || B < 1) return p;
    if (g.n_out % 8 == 0 && g.n_out > 256) {
        p.T = 8;            // one tile covers 512 outputs: the per-record work is shared by twice as many
        p.streams = 1;
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
    //   - what keeps the gy rows of one chunk inside an XCD's L2 (about 2 MiB of it),
    //   - an eighth of the batch (one chunk per XCD at least),
    // then raised until the partial sums fit 2 GiB.  Few, long chunks keep the partial sums small;
    // the parallelism comes from cutting each sorted list into segments (below).
    auto pow2_floor = [](int64_t v) { int64_t q = 256; while (q * 2 <= v && q < 8192) q *= 2; return (int)q; };
    int S = pow2_floor((2ll << 20) / ((int64_t)g.n_out * 4));
    const int s_b8 = pow2_floor(B / 8);
    S = S < s_b8 ? S : s_b8;
    const int64_t slab = (int64_t)g.n_in * g.rows * g.n_out * (int64_t)sizeof(float);
    while (S < 8192 && ((B + S - 1) / S) * slab > (2ll << 30)) S *= 2;
    p.S = S;
    p.sbits = log2_exact(S);
    p.n_chunks = (int)((B + S - 1) / S);
    // segments per list: enough for about 2048 waves, at least 64 records each
    p.n_seg = 1;
    while (S / (p.n_seg * 2) >= 64 &&
           (int64_t)p.n_chunks * p.n_seg * p.n_jt * g.n_in < (int64_t)2048 * p.streams)
        p.n_seg *= 2;
    int bits = 0;
    while ((1 << bits) < g.rows - kMaxK + 1) ++bits;
    p.row_bits = bits < 1 ? 1 : bits;
    p.ok = (int64_t)p.n_chunks * slab <= (4ll << 30) ? 1 : 0;
    return p;
}

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
    const size_t n = (size_t)p.n_chunks * n_in * p.S;
    const size_t gxp = p.n_jt > 1 ? up256((size_t)p.n_jt * B * n_in * sizeof(float)) : 0;
    return up256((size_t)B * n_in * sizeof(float)) + 3 * up256(n * 4) + 2 * up256(n * 16) + gxp +
           walk_carry_bytes(p, n_in, n_out);
}

template <int STREAMS, int T>
static void walk_launch(bool dx, unsigned blocks, hipStream_t st, const SplineGeom &g, const WalkRecords &rec,
                        const float *gy, const float *cf, const float *w_b, float *part_c, float *part_b, float *gx,
                        int64_t B, const WalkPlan &p, int bpc, int m, int prezeroed, float *carry)
{
    auto kern = dx ? (p.S > 1024 ? backward_walk_kernel<STREAMS, T, true, true> : backward_walk_kernel<STREAMS, T, true, false>)
                   : (p.S > 1024 ? backward_walk_kernel<STREAMS, T, false, true> : backward_walk_kernel<STREAMS, T, false, false>);
    kern<<<blocks, 256, 0, st>>>(g, rec, gy, cf, w_b, part_c, part_b, gx, B, p.S, p.n_chunks, p.n_jt, bpc, m, prezeroed,
                                 p.n_seg, carry);
}

// gx == nullptr: parameter gradients only.  part_c == nullptr: dL/dx only.  cf is the scale-folded
// table ([n_in][slab_rows][n_out]); w_b may be null when the layer has no base term.
hipError_t launch_backward_walk(const SplineGeom &g, const WalkPlan &p, const float *x, const float *gy,
                                const float *cf, const float *w_b, void *scratch, float *gx, float *part_c,
                                float *part_b, int64_t B, hipStream_t st)
{
    const size_t n = (size_t)p.n_chunks * g.n_in * p.S;
    const bool dx = gx != nullptr;
    char *at = (char *)scratch;
    float *xT = (float *)at;            at += up256((size_t)B * g.n_in * sizeof(float));
    WalkRecords rec;
    rec.rt = (int *)at;                 at += up256(n * 4);
    rec.base = (float *)at;             at += up256(n * 4);
    rec.w4 = (float *)at;               at += up256(n * 16);
    rec.dbase = dx ? (float *)at : nullptr; at += up256(n * 4);
    rec.dw4 = dx ? (float *)at : nullptr;   at += up256(n * 16);
    float *gx_part = (float *)at;       at += p.n_jt > 1 ? up256((size_t)p.n_jt * B * g.n_in * sizeof(float)) : 0;
    float *carry = (float *)at;
    {
        dim3 grid((unsigned)((B + 63) / 64), (unsigned)((g.n_in + 63) / 64));
        prof::Timed tm("walk_transpose", st);
        transpose_kernel<<<grid, 256, 0, st>>>(x, xT, B, g.n_in);
    }
    {
        const size_t lds = (size_t)p.S * 12;
        // long chunks: 16 waves per sort (one workgroup per CU fits anyway), short ones 4
        auto kern = p.S >= 4096 ? cell_sort_kernel<16> : cell_sort_kernel<4>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        dim3 grid((unsigned)p.n_chunks, (unsigned)g.n_in);
        prof::Timed tm("walk_sort", st);
        kern<<<grid, p.S >= 4096 ? 1024 : 256, lds, st>>>(g, xT, B, p.S, p.sbits, p.row_bits, rec);
    }
    const int bpc = (p.n_seg * p.n_jt * g.n_in + 4 * p.streams - 1) / (4 * p.streams);
    int m = 1;
    while (m * 2 <= 8 && m * 2 <= p.n_chunks) m *= 2;
    const int bpc_sub = (bpc + 8 / m - 1) / (8 / m);
    const unsigned blocks = (unsigned)(8 * bpc_sub * ((p.n_chunks + m - 1) / m));
    float *gx_out = dx ? (p.n_jt > 1 ? gx_part : gx) : nullptr;
    // Sparse regime (far more rows than a chunk has samples): most rows of a chunk's partial slab
    // receive nothing.  The slab is zeroed with a streaming fill and the walk skips the gaps instead of
    // stepping through them row by row.
    const int prezeroed = (part_c != nullptr && g.rows > 2 * p.S) ? 1 : 0;
    if (prezeroed) {
        const int64_t n4 = (int64_t)p.n_chunks * g.n_in * g.rows * g.n_out;
        prof::Timed tm("walk_zero_fill", st);
        fill_zero_kernel<<<(unsigned)((n4 + 1023) / 1024), 256, 0, st>>>(part_c, n4);
    }
    {
        prof::Timed tm(dx ? "backward_walk" : "dparam_walk", st);
        if (p.T == 8 && p.streams == 1)
            walk_launch<1, 8>(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry);
        else if (p.T == 4 && p.streams == 1)
            walk_launch<1, 4>(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry);
        else if (p.T == 4 && p.streams == 2)
            walk_launch<2, 4>(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry);
        else if (p.T == 4 && p.streams == 4)
            walk_launch<4, 4>(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry);
        else if (p.T == 1 && p.streams == 4)
            walk_launch<4, 1>(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx_out, B, p, bpc, m, prezeroed, carry);
        else
            return hipErrorInvalidValue;
    }
    if (part_c != nullptr && p.n_seg > 1) {
        const int64_t nn = (int64_t)p.n_chunks * g.n_in * g.n_out;
        prof::Timed tm("walk_carry", st);
        walk_carry_kernel<<<(unsigned)((nn + 255) / 256), 256, 0, st>>>(g, rec.rt, carry, part_c, p.S, p.n_chunks,
                                                                       p.n_seg);
    }
    if (dx && p.n_jt > 1) {
        const int64_t nn = B * g.n_in;
        prof::Timed tm("walk_gx_sum", st);
        gx_sum_kernel<<<(unsigned)((nn + 255) / 256), 256, 0, st>>>(gx_part, gx, nn, p.n_jt);
    }
    return hipGetLastError();
}

}  // namespace kan
