// The walk kernel of kan_walk.hip and its launcher template.  Lives in a header so that every
// (streams per wave, outputs per lane) variant is compiled in a translation unit of its own
// (kan_walk_s*t*.hip): the kernel is large and the variants build in parallel that way.
#pragma once
#include <type_traits>
#include "kan_device.hpp"
#include "kan_launch.hpp"

namespace kan {

namespace {

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
    } else if constexpr (T == 2) {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
        static_assert(T == 1, "one, two, four or eight outputs per lane");
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
    } else if constexpr (T == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
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
                                                            float *__restrict__ carry, int chunk0, int shared, int L, int hk)
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
    // n_chunks counts the chunks of this launch, the first of which is chunk0 of the batch; the launch's
    // chunk number l uses partial slab l.  shared: a slab holds the sums of earlier launches, add to them.
    const int c_local = grp + xcd_groups * (slot / bpc_sub);
    const int c = chunk0 + c_local;
    const int blk = (slot % bpc_sub) * n_sub + sub_x;
    const int ws = (blk * 4 + wave) * STREAMS + sub;
    if (c_local >= n_chunks || blk >= blocks_per_chunk || ws >= n_seg * n_jt * g.n_in) return;
    const int i = ws % g.n_in;
    const int jt = (ws / g.n_in) % n_jt;
    const int seg = ws / (g.n_in * n_jt);
    // L entries per sorted list: S, or 2 S with two records per pair (hk); seg_len is a multiple of 16
    const int seg_len = L / n_seg;
    const int j = (jt * LPS + q) * T;
    const bool jok = j < g.n_out;
    const int jc = jok ? j : 0;
    const int64_t b0 = (int64_t)c * S;
    const int n_c = (int)((B - b0) < S ? (B - b0) : S);
    const int64_t list0 = ((int64_t)c * g.n_in + i) * L;
    const int n_live = hk ? 2 * n_c : n_c;          // records that belong to real samples (they sort first)
    // hk: 12 bits of sample index, bit 31 of a record (bit 12 after the shift) names the partial gx it adds to
    const int smp_mask = hk ? 0xfff : 0x1fff;
    const int64_t gx_second = (int64_t)n_jt * B * g.n_in;
    const int64_t list = list0 + (int64_t)seg * seg_len;        // this segment's records
    // The segment owns the table rows from its first record's row up to the next segment's first
    // row; what its window holds beyond that at the end goes to the next segment's carry rows.
    const int r_next = seg + 1 < n_seg ? (rec.rt[list + seg_len] & kRtRowMask) : g.rows;
    const float *gyp = gy + b0 * g.n_out + jc;
    const bool store_c = jok && part_c != nullptr;
    float *out = part_c + ((int64_t)c_local * g.n_in + i) * g.rows * g.n_out + jc;
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

    int cur = rec.rt[list] & kRtRowMask;     // first row of the window the accumulators stand on
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
        if (store && store_c) {
            float *dst = out + (int64_t)cur * g.n_out;
            if (shared) {
                // uniform.  Add to what earlier chunks left in the row.  Within a launch this wave is the
                // only writer of the row and launches follow each other on the stream, so the sum is the
                // same every run; the hardware add is used because it does not wait for the old value.
#pragma unroll
                for (int r = 0; r < T; ++r) unsafeAtomicAdd(dst + r, gone[r]);
            } else {
                store_vec<T>(dst, gone);
            }
        }
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
    gather((int)((unsigned)mine.rt >> kRtRowBits) & smp_mask, std::integral_constant<int, 0>{}, gbuf[0]);
    for (int bi = 0; bi < nb; ++bi) {
        const Batch upcoming = load_batch(bi + 1 < nb ? bi + 1 : bi);
        const int rowv = mine.rt & kRtRowMask, tvf = (int)((unsigned)mine.rt >> kRtRowBits);
        const int tv = tvf & smp_mask;
        float dot[16];
        bool quad_same = false;
        // The 16 records go in groups of four.  The gy rows of the next group (the first of the next
        // batch after the last) are requested before the current group is worked on.
        constexpr int GROUP = 4;
        auto group = [&](auto h) {
            constexpr int H = decltype(h)::value;
            auto &gr = gbuf[H & 1];
            if constexpr (H + 1 < 16 / GROUP) gather(tv, std::integral_constant<int, H + 1>{}, gbuf[(H + 1) & 1]);
            else gather((int)((unsigned)upcoming.rt >> kRtRowBits) & smp_mask, std::integral_constant<int, 0>{}, gbuf[0]);
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
            const int tf = __shfl(tvf, (lane & ~15) | qn, 64);
            const int t = tf & smp_mask;
            float *gxr = gxo + ((tf >> 12) & hk ? gx_second : 0);
            if ((lane % (LPS / 16)) == 0 && seg * seg_len + bi * 16 + qn < n_live) gxr[(int64_t)t * g.n_in] = total;
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

template <int STREAMS, int T>
void walk_launch(bool dx, unsigned blocks, hipStream_t st, const SplineGeom &g, const WalkRecords &rec,
                        const float *gy, const float *cf, const float *w_b, float *part_c, float *part_b, float *gx,
                        int64_t B, const WalkPlan &p, int bpc, int m, int prezeroed, float *carry, int chunk0,
                        int n_chunks)
{
    auto kern = dx ? (p.S > 1024 ? backward_walk_kernel<STREAMS, T, true, true> : backward_walk_kernel<STREAMS, T, true, false>)
                   : (p.S > 1024 ? backward_walk_kernel<STREAMS, T, false, true> : backward_walk_kernel<STREAMS, T, false, false>);
    // the first round of a shared run finds its slabs zero and stores like an unshared run
    kern<<<blocks, 256, 0, st>>>(g, rec, gy, cf, w_b, part_c, part_b, gx, B, p.S, n_chunks, p.n_jt, bpc, m, prezeroed,
                                 p.n_seg, carry, chunk0, (p.shared && chunk0 > 0) ? 1 : 0, p.L, p.hk);
}

}  // namespace

}  // namespace kan
