// C ABI of the bounded-grid KAN layer: argument checks, workspace layout and
// kernel dispatch.  See include/kan.h for the contract.
#include <mutex>
#include "kan.h"
#include "kan_launch.hpp"
#include "kan_highk.hpp"

using namespace kan;

namespace kanprof {
Hook g_before = nullptr, g_after = nullptr;
}

extern "C" int kan_set_launch_observer(kan_launch_hook before, kan_launch_hook after)
{
    kanprof::g_before = before;
    kanprof::g_after = after;
    return KAN_OK;
}

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// every float array is read and written with 16-byte accesses where the widths allow
inline bool misaligned(const void *p) { return p && ((uintptr_t)p % 16) != 0; }

int check_desc(const kan_layer_desc *d)
{
    if (!d) return KAN_ERR_INVALID_ARG;
    if (d->n_in <= 0 || d->n_out <= 0 || d->G <= 0) return KAN_ERR_INVALID_ARG;
    if (!(d->grid_hi > d->grid_lo)) return KAN_ERR_INVALID_ARG;
    if (d->k < 1 || d->k > 5) return KAN_ERR_UNSUPPORTED;
    if (d->n_in > 65535) return KAN_ERR_UNSUPPORTED;          // inputs index a 16-bit launch dimension
    // float offsets inside one input's table are 32-bit
    if (((int64_t)d->G + d->k + 1) * (int64_t)d->n_out >= (1ll << 31)) return KAN_ERR_UNSUPPORTED;
    if (d->base_act != KAN_BASE_NONE && d->base_act != KAN_BASE_SILU) return KAN_ERR_UNSUPPORTED;
    return KAN_OK;
}

SplineGeom geom_of(const kan_layer_desc *d)
{
    SplineGeom g;
    g.n_in = d->n_in;
    g.n_out = d->n_out;
    g.rows = d->G + d->k;
    g.slab_rows = g.rows + 1;
    g.k = d->k;
    g.lo = d->grid_lo;
    g.inv_h = (float)d->G / (d->grid_hi - d->grid_lo);
    g.cell_base = nullptr;
    g.base_act = d->base_act;
    return g;
}

// degrees 4 and 5 run on the generic kernels built for a window of 6 rows
bool high_degree(const kan_layer_desc *d) { return d->k > 3; }

HighKLayer highk_of(const kan_layer_desc *d)
{
    HighKLayer l = {};
    l.n_in = d->n_in; l.n_out = d->n_out; l.rows = d->G + d->k; l.k = d->k;
    l.lo = d->grid_lo; l.inv_h = (float)d->G / (d->grid_hi - d->grid_lo);
    l.base_act = d->base_act;
    return l;
}

// scale-folded table: G + k coefficient rows plus the w_b row per input
size_t folded_bytes(const kan_layer_desc *d)
{
    return align_up((size_t)d->n_in * (size_t)(d->G + d->k + 1) * (size_t)d->n_out * sizeof(float));
}

size_t edge_bytes(const kan_layer_desc *d)
{
    return align_up((size_t)d->n_in * (size_t)d->n_out * sizeof(float));
}

// which kernel takes the parameter gradients and how its scratch is cut
struct BackwardPlan {
    bool walk;
    WalkPlan wp;
    ChunkPlan cp;
    size_t rec_bytes;       // transposed x + sorted records of the walk (0 for the generic kernel)
    int b_slices_per_chunk; // base-term partial slices each chunk writes
    int n_slabs;            // partial slabs of the table gradient (one per chunk, or one shared by all)
    size_t tail_bytes;      // scratch behind a single shared slab for the row-slice sums of gw_s
};

BackwardPlan backward_plan(const kan_layer_desc *d, int64_t B)
{
    SplineGeom g = geom_of(d);
    BackwardPlan bp;
    // degrees 4 and 5 walk two four-row records per pair
    bp.wp = plan_walk(g, B, true, high_degree(d));
    bp.walk = bp.wp.ok != 0;
    bp.tail_bytes = 0;
    if (bp.walk) {
        bp.n_slabs = bp.wp.n_slabs;
        if (bp.wp.shared) bp.tail_bytes = align_up(dparam_reduce_tail_bytes(g.n_in, g.n_out));
        bp.cp.n_chunks = bp.wp.n_chunks;
        bp.cp.chunk_len = bp.wp.S;
        bp.rec_bytes = align_up(walk_scratch_bytes(bp.wp, B, g.n_in, g.n_out));
        bp.b_slices_per_chunk = bp.wp.n_seg;
    } else {
        bp.cp = plan_chunks(B, g.n_in, g.rows, g.n_out);
        bp.n_slabs = bp.cp.n_chunks;
        bp.rec_bytes = 0;
        bp.b_slices_per_chunk = high_degree(d) ? highk_row_blocks(g.rows) : dparam_generic_row_blocks(g.rows);
    }
    return bp;
}

}  // namespace

extern "C" const char *kan_strerror(int status)
{
    switch (status) {
    case KAN_OK: return "ok";
    case KAN_ERR_INVALID_ARG: return "invalid argument";
    case KAN_ERR_UNSUPPORTED: return "unsupported configuration";
    case KAN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KAN_ERR_RANGE: return "input spans more groups than max_groups";
    case KAN_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

extern "C" size_t kan_workspace_bytes(const kan_layer_desc *desc, int64_t B, int pass)
{
    if (check_desc(desc) != KAN_OK || B < 0) return 0;
    if (pass == KAN_PASS_FORWARD) return folded_bytes(desc);
    if (pass != KAN_PASS_BACKWARD) return 0;
    const BackwardPlan bp = backward_plan(desc, B);
    return folded_bytes(desc) + bp.rec_bytes + (size_t)bp.n_slabs * folded_bytes(desc) + bp.tail_bytes +
           (size_t)bp.cp.n_chunks * bp.b_slices_per_chunk * edge_bytes(desc);
}

// Forward pass with the scratch space given explicitly; shared by kan_forward and kan_forward_static.
static int forward_impl(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                        const float *w_s, const float *w_b, float *y, void *ws, size_t ws_bytes,
                        void *stream)
{
    int rc = check_desc(desc);
    if (rc != KAN_OK) return rc;
    if (B < 0) return KAN_ERR_INVALID_ARG;
    if (B == 0) return KAN_OK;
    if (!x || !coef || !w_s || !y) return KAN_ERR_INVALID_ARG;
    if (desc->base_act != KAN_BASE_NONE && !w_b) return KAN_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(coef) || misaligned(w_s) || misaligned(w_b) || misaligned(y)) return KAN_ERR_INVALID_ARG;
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < kan_workspace_bytes(desc, B, KAN_PASS_FORWARD))
        return KAN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    SplineGeom g = geom_of(desc);
    float *cf = (float *)ws;
    if (high_degree(desc))
        return highk_forward(highk_of(desc), x, coef, w_s, w_b, cf, y, B, st) == hipSuccess ? KAN_OK : KAN_ERR_HIP;
    if (launch_fold_scale(coef, w_s, g.base_act ? w_b : nullptr, cf, g.n_in, g.rows, g.n_out, st) != hipSuccess) return KAN_ERR_HIP;
    hipError_t e = narrow_applicable(g)    ? launch_forward_narrow(g, x, cf, w_b, y, B, st)
                   : (g.n_out <= 64 && forward_lds_rows_plan(g, B)) ? launch_forward_lds_rows(g, x, cf, y, B, st)
                   : forward_rows_plan(g) ? launch_forward_rows(g, x, cf, y, B, st)
                   : forward_lds_plan(g)  ? launch_forward_lds(g, x, cf, y, B, st)
                   : forward_lds_rows_plan(g, B) ? launch_forward_lds_rows(g, x, cf, y, B, st)
                                         : launch_forward_generic(g, x, cf, w_b, y, B, st);
    return e == hipSuccess ? KAN_OK : KAN_ERR_HIP;
}

extern "C" int kan_forward(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                           const float *w_s, const float *w_b, float *y, void *ws, size_t ws_bytes,
                           void *stream)
{
    return forward_impl(desc, B, x, coef, w_s, w_b, y, ws, ws_bytes, stream);
}

// ---- forward pass for callers that cannot allocate -------------------------------------------
// The scratch of kan_forward (the scale-folded table) lives in a device array of fixed size that is
// part of the library's code object: every GPU the library runs on holds one copy at an address of
// its own, found once per device with hipGetSymbolAddress.  In host code the array's name is only
// a handle for that query, never a device address.
static __device__ __align__(256) unsigned char scratch[KAN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices];      // per device; nullptr until the first call on that device

// device address of `scratch` on the current device (nullptr: the query failed)
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}
}  // namespace

extern "C" size_t kan_static_scratch_bytes(void) { return KAN_STATIC_SCRATCH_BYTES; }

extern "C" int kan_forward_static(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                                  const float *w_s, const float *w_b, float *y, void *stream)
{
    int rc = check_desc(desc);
    if (rc != KAN_OK) return rc;
    if (B < 0) return KAN_ERR_INVALID_ARG;
    if (B == 0) return KAN_OK;
    if (kan_workspace_bytes(desc, B, KAN_PASS_FORWARD) > (size_t)KAN_STATIC_SCRATCH_BYTES) return KAN_ERR_WORKSPACE;
    void *ws = static_scratch();
    if (!ws) return KAN_ERR_HIP;
    return forward_impl(desc, B, x, coef, w_s, w_b, y, ws, KAN_STATIC_SCRATCH_BYTES, stream);
}

// Backward pass; `folded` (may be null) is the scale-folded table a forward pass left in its workspace.
static int backward_impl(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                         const float *w_s, const float *w_b, const float *gy, const float *folded, float *gx,
                         float *gcoef, float *gw_s, float *gw_b, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != KAN_OK) return rc;
    if (B < 0) return KAN_ERR_INVALID_ARG;
    if (B == 0) return KAN_OK;
    if (!x || !coef || !w_s || !gy) return KAN_ERR_INVALID_ARG;
    if (desc->base_act != KAN_BASE_NONE && !w_b) return KAN_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(coef) || misaligned(w_s) || misaligned(w_b) || misaligned(gy) || misaligned(gx) ||
        misaligned(gcoef) || misaligned(gw_s) || misaligned(gw_b))
        return KAN_ERR_INVALID_ARG;
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < kan_workspace_bytes(desc, B, KAN_PASS_BACKWARD))
        return KAN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    SplineGeom g = geom_of(desc);
    float *cf = (float *)ws;
    const BackwardPlan bp = backward_plan(desc, B);
    if (misaligned(folded)) return KAN_ERR_INVALID_ARG;
    if (high_degree(desc) && !bp.walk) {
        float *part_c = (float *)((char *)ws + folded_bytes(desc));
        float *part_b = (float *)((char *)part_c + (size_t)bp.n_slabs * folded_bytes(desc));
        return highk_backward(highk_of(desc), x, coef, w_s, w_b, gy, cf, gx, gcoef, gw_s, gw_b, part_c, part_b,
                              bp.cp.n_chunks, bp.cp.chunk_len, B, st) == hipSuccess
                   ? KAN_OK
                   : KAN_ERR_HIP;
    }
    const bool want_params = gcoef || gw_s || gw_b;
    // the chunk-sorted walk takes dL/dx together with the parameter gradients (one pass over gy)
    const bool fused_dx = gx && bp.walk;
    const float *table = folded ? folded : cf;        // the table dL/dx reads
    if (gx) {
        if (!folded &&
            launch_fold_scale(coef, w_s, g.base_act ? w_b : nullptr, cf, g.n_in, g.rows, g.n_out, st) != hipSuccess)
            return KAN_ERR_HIP;
        if (!fused_dx) {
            hipError_t e = narrow_applicable(g) ? launch_dx_narrow(g, x, table, w_b, gy, gx, B, st)
                                                : launch_dx_generic(g, x, table, w_b, gy, gx, B, st);
            if (e != hipSuccess) return KAN_ERR_HIP;
        }
    }
    const bool want_b = gw_b && desc->base_act != KAN_BASE_NONE;
    if (want_params || fused_dx) {
        const ChunkPlan cp = bp.cp;
        char *at = (char *)ws + folded_bytes(desc);
        void *walk_scratch = at;
        at += bp.rec_bytes;
        float *part_c = (float *)at;
        float *part_b = (float *)((char *)part_c + (size_t)bp.n_slabs * folded_bytes(desc) + bp.tail_bytes);
        // partial slabs are laid out back to back with the unpadded slab size
        hipError_t e = bp.walk ? launch_backward_walk(g, bp.wp, x, gy, table, w_b, walk_scratch, fused_dx ? gx : nullptr,
                                                      want_params ? part_c : nullptr, want_b ? part_b : nullptr, B, st)
                               : launch_dparam_generic(g, x, gy, part_c, want_b ? part_b : nullptr, B, cp.n_chunks,
                                                       cp.chunk_len, st);
        if (e != hipSuccess) return KAN_ERR_HIP;
        if (want_params &&
            launch_dparam_reduce(part_c, want_b ? part_b : nullptr, coef, w_s, gcoef, gw_s, gw_b, g.n_in, g.rows,
                                 g.n_out, bp.n_slabs, cp.n_chunks * bp.b_slices_per_chunk, st,
                                 // a shared slab is followed by the folded table's spare row and the tail scratch
                                 bp.tail_bytes ? bp.tail_bytes + (folded_bytes(desc) - (size_t)g.n_in * g.rows * g.n_out * sizeof(float)) : 0) != hipSuccess)
            return KAN_ERR_HIP;
    }
    return KAN_OK;
}

extern "C" int kan_backward(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                            const float *w_s, const float *w_b, const float *gy, float *gx, float *gcoef,
                            float *gw_s, float *gw_b, void *ws, size_t ws_bytes, void *stream)
{
    return backward_impl(desc, B, x, coef, w_s, w_b, gy, nullptr, gx, gcoef, gw_s, gw_b, ws, ws_bytes, stream);
}

extern "C" int kan_backward_saved(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                                  const float *w_s, const float *w_b, const float *gy, const void *forward_ws,
                                  float *gx, float *gcoef, float *gw_s, float *gw_b, void *ws, size_t ws_bytes,
                                  void *stream)
{
    if (!forward_ws || ((uintptr_t)forward_ws % kAlign) != 0) return KAN_ERR_WORKSPACE;
    if (forward_ws == ws) return KAN_ERR_INVALID_ARG;          // the backward scratch would overwrite the table
    return backward_impl(desc, B, x, coef, w_s, w_b, gy, (const float *)forward_ws, gx, gcoef, gw_s, gw_b, ws,
                         ws_bytes, stream);
}

extern "C" int kan_interval_index(const kan_layer_desc *desc, int64_t n, const float *x, int32_t *idx,
                                  void *stream)
{
    int rc = check_desc(desc);
    if (rc != KAN_OK) return rc;
    if (n < 0) return KAN_ERR_INVALID_ARG;
    if (n == 0) return KAN_OK;
    if (!x || !idx) return KAN_ERR_INVALID_ARG;
    SplineGeom g = geom_of(desc);
    if (launch_interval_index(x, idx, n, g.lo, g.inv_h, (hipStream_t)stream) != hipSuccess) return KAN_ERR_HIP;
    return KAN_OK;
}
