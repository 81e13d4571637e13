// Host-side launch functions of the kernels (one per kernel family).  Each
// enqueues on the given stream and returns the HIP launch status; none
// synchronises or allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "kan_device.hpp"

// Launch observer (kan_set_launch_observer in kan.h).  A Timed object calls the installed hooks on
// the host right before and right after one kernel launch is enqueued, and does nothing when none
// is installed.
namespace kanprof {
typedef void (*Hook)(const char *family, void *stream);
extern Hook g_before, g_after;
struct Timed {
    const char *family;
    hipStream_t st;
    Hook after;
    Timed(const char *f, hipStream_t s) : family(f), st(s), after(g_after)
    {
        if (Hook b = g_before) b(family, (void *)st);
    }
    ~Timed() { if (after) after(family, (void *)st); }
};
}  // namespace kanprof

namespace KAN_NS {

namespace prof = ::kanprof;

// Raises a kernel's dynamic LDS limit to `bytes` once per (kernel, device) instead of on every launch.
// `Tag` is any type unique to the kernel instantiation (each gets its own table).
template <typename Tag>
inline hipError_t ensure_dynamic_lds(const void *kern, int bytes)
{
    static int have[64] = {};      // bytes already granted, per device ordinal
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && __atomic_load_n(&have[dev], __ATOMIC_ACQUIRE) >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) __atomic_store_n(&have[dev], bytes, __ATOMIC_RELEASE);
    return e;
}

hipError_t launch_interval_index(const float *x, int32_t *idx, int64_t n, float lo, float inv_h,
                                 hipStream_t st);
hipError_t launch_fold_scale(const float *coef, const float *w_s, const float *w_b, float *cf, int n_in, int rows,
                             int n_out, hipStream_t st);

// generic (any shape) kernels
hipError_t launch_forward_generic(const SplineGeom &g, const float *x, const float *cf, const float *w_b,
                                  float *y, int64_t B, hipStream_t st);
hipError_t launch_dx_generic(const SplineGeom &g, const float *x, const float *cf, const float *w_b,
                             const float *gy, float *gx, int64_t B, hipStream_t st);
int dparam_generic_row_blocks(int rows);     // base-term partial slices per chunk
hipError_t launch_dparam_generic(const SplineGeom &g, const float *x, const float *gy, float *part_c,
                                 float *part_b, int64_t B, int n_chunks, int64_t chunk_len, hipStream_t st);
// tail_scratch: bytes of scratch that follow the first partial slab when there is only one (with two
// or more, the second slab serves); 0 = none
size_t dparam_reduce_tail_bytes(int n_in, int n_out);
hipError_t launch_dparam_reduce(float *part_c, const float *part_b, const float *coef, const float *w_s,
                                float *gcoef, float *gw_s, float *gw_b, int n_in, int rows, int n_out,
                                int n_chunks, int n_slices_b, hipStream_t st, size_t tail_scratch = 0);

// narrow layers (n_out <= 16)
int narrow_applicable(const SplineGeom &g);
hipError_t launch_forward_narrow(const SplineGeom &g, const float *x, const float *cf, const float *w_b, float *y,
                                 int64_t B, hipStream_t st);
hipError_t launch_dx_narrow(const SplineGeom &g, const float *x, const float *cf, const float *w_b, const float *gy,
                            float *gx, int64_t B, hipStream_t st);

// layers of 17 .. 64 outputs: four samples per wave, one per DPP row (0: not applicable)
int forward_rows_plan(const SplineGeom &g);
hipError_t launch_forward_rows(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                               hipStream_t st);

// LDS-staged kernels (small grids); *_plan returns 0 when the shape does not qualify
int forward_lds_plan(const SplineGeom &g);
hipError_t launch_forward_lds(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                              hipStream_t st);

// LDS-staged kernel for long tables (narrow output tile, many samples per workgroup); the plan
// returns 0 when the shape does not qualify
int forward_lds_rows_plan(const SplineGeom &g, int64_t B);
hipError_t launch_forward_lds_rows(const SplineGeom &g, const float *x, const float *cf, float *y, int64_t B,
                                   hipStream_t st);

// Sorted pair records of the walk, one per (sample, input) pair, as a structure of arrays indexed
// [chunk][input][rank in the chunk's sorted order]: first row of the K-wide window (clamped into the
// table; kRtRowBits bits) | the sample's index inside its chunk << kRtRowBits (chunks hold at most
// 2^13 samples; 2^12 for degrees 4 and 5, where bit 31 says which of a pair's two records this is); the base value; the K window weights (16-byte
// aligned quadruples); and the same for the x-derivatives (null when dL/dx is not wanted).
constexpr int kRtRowBits = 19;
constexpr int kRtRowMask = (1 << kRtRowBits) - 1;
struct WalkRecords {
    int *rt;
    float *base;
    float *w4;
    float *dbase;
    float *dw4;
};

hipError_t launch_sorted_records(const SplineGeom &g, const float *x, float *xT, int64_t B, int S, int row_bits,
                                 const WalkRecords &rec, hipStream_t st);

// Chunk-sorted walk (large grids, narrow layers).  plan_walk().ok == 0: shape not covered.
struct WalkPlan {
    int ok;
    int S, sbits;        // samples per chunk (power of two) and its log2
    int n_chunks;
    int n_seg;           // segments each sorted list is cut into (one stream each), a power of two
    int streams, T;      // streams per wave, outputs per lane
    int n_jt;            // output tiles of (64 / streams) * T outputs
    int row_bits;        // bits of the largest window row (sort key width)
    int shared;          // 1: fewer partial slabs than chunks; the chunks are walked in rounds of n_slabs
    int n_slabs;         // partial slabs the walk writes: n_chunks, or what fits the budget when shared
    int hk;              // 1: degrees 4 and 5.  A pair's window of six rows is walked as two records of four
                         // rows (rows 0..3 with the base term, rows 4..5), so a sorted list has L = 2 S entries
                         // and dL/dx is the sum of two partial results per output tile
    int L;               // entries of one sorted list: S, or 2 S when hk
};
// allow_shared: tables whose per-chunk partial slabs would not fit the budget are still planned, with the
// chunks taking turns on the slabs that fit (ok stays 0 for them otherwise).
WalkPlan plan_walk(const SplineGeom &g, int64_t B, bool allow_shared = false, bool high_degree = false);
size_t walk_scratch_bytes(const WalkPlan &p, int64_t B, int n_in, int n_out);
hipError_t launch_backward_walk(const SplineGeom &g, const WalkPlan &p, const float *x, const float *gy,
                                const float *cf, const float *w_b, void *scratch, float *gx, float *part_c,
                                float *part_b, int64_t B, hipStream_t st);

// How the batch is cut into chunks for the parameter-gradient reduction: chunks of about 1024
// samples, at most 64 of them, and no more than fit a 512 MiB budget of partial sums.
struct ChunkPlan { int n_chunks; int64_t chunk_len; };
inline ChunkPlan plan_chunks(int64_t B, int n_in, int rows, int n_out)
{
    int64_t slab = (int64_t)n_in * rows * n_out * (int64_t)sizeof(float);
    int64_t by_budget = (512ll << 20) / (slab > 0 ? slab : 1);
    int64_t n = (B + 1023) / 1024;
    if (n > 64) n = 64;
    if (n > by_budget) n = by_budget;
    if (n < 1) n = 1;
    ChunkPlan p;
    p.chunk_len = (B + n - 1) / n;
    if (p.chunk_len < 1) p.chunk_len = 1;
    p.n_chunks = (int)((B + p.chunk_len - 1) / p.chunk_len);
    if (p.n_chunks < 1) p.n_chunks = 1;
    return p;
}

}  // namespace KAN_NS
