// C ABI of the UKAN layer: workspace layout, the single read-back of the group span, and
// the sequence of kernels (range -> CG forward -> spline kernels -> CG backward).
// See include/kan.h for the contract.
#include <initializer_list>
#include "kan.h"
#include "kan_launch.hpp"
#include "kan_highk.hpp"
#include "ukan_launch.hpp"

using namespace kan;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int check_desc(const ukan_layer_desc *d)
{
    if (!d) return KAN_ERR_INVALID_ARG;
    if (d->n_in <= 0 || d->n_out <= 0 || !(d->h > 0.0f)) return KAN_ERR_INVALID_ARG;
    if (d->d_pe <= 0 || d->d_feat < 0 || d->d_hidden <= 0) return KAN_ERR_INVALID_ARG;
    if (d->k < 1 || d->k > 5) return KAN_ERR_UNSUPPORTED;
    if (d->n_in > 65535) return KAN_ERR_UNSUPPORTED;          // inputs index a 16-bit launch dimension
    if (d->d_pe % 2 != 0) return KAN_ERR_UNSUPPORTED;         // sin/cos pairs
    if (d->base_act != KAN_BASE_NONE && d->base_act != KAN_BASE_SILU) return KAN_ERR_UNSUPPORTED;
    return KAN_OK;
}

// the walk is planned for the largest table the workspace allows, so that the chunking (and with it
// the workspace layout) does not depend on the data
WalkPlan walk_for(const ukan_layer_desc *d, int64_t B, int32_t max_groups)
{
    SplineGeom g = {};
    g.n_in = d->n_in; g.n_out = d->n_out; g.rows = max_groups * (d->k + 1); g.slab_rows = g.rows; g.k = d->k;
    return plan_walk(g, B, false, d->k > 3);     // degrees 4 and 5: two four-row records per pair
}

// degrees 4 and 5 run the kernels built for a window of six rows
bool high_degree(const ukan_layer_desc *d) { return d->k > 3; }

HighKLayer highk_of(const SplineGeom &g)
{
    HighKLayer l = {};
    l.n_in = g.n_in; l.n_out = g.n_out; l.rows = g.rows; l.k = g.k; l.lo = g.lo; l.inv_h = g.inv_h;
    l.base_act = g.base_act; l.slab_rows = g.slab_rows; l.cell_base = g.cell_base;
    return l;
}

int row_blocks_for(const ukan_layer_desc *d, int rows)
{
    return high_degree(d) ? highk_row_blocks(rows) : dparam_generic_row_blocks(rows);
}

// base-term partial slices each chunk writes
int b_slices_for(const ukan_layer_desc *d, int64_t B, int32_t max_groups)
{
    const WalkPlan wp = walk_for(d, B, max_groups);
    return wp.ok ? wp.n_seg : row_blocks_for(d, max_groups * (d->k + 1));
}

// scratch of the walk's pre-pass (transposed x + sorted records)
size_t record_bytes_for(const ukan_layer_desc *d, int64_t B, int32_t max_groups)
{
    const WalkPlan wp = walk_for(d, B, max_groups);
    return wp.ok ? walk_scratch_bytes(wp, B, d->n_in, d->n_out) : 0;
}

ChunkPlan chunks_for(const ukan_layer_desc *d, int64_t B, int32_t max_groups)
{
    const WalkPlan wp = walk_for(d, B, max_groups);
    if (wp.ok) {
        ChunkPlan cp;
        cp.n_chunks = wp.n_chunks; cp.chunk_len = wp.S;
        return cp;
    }
    return plan_chunks(B, d->n_in, max_groups * (d->k + 1), d->n_out);
}

// Offsets (bytes) of every scratch region for `n_g` generator rows per input.
struct Layout {
    size_t cmin, cmax, g_first, n_groups, cell_base, summary;
    size_t hid, cf;                                   // forward
    size_t z, pre, raw, rec, part_c, part_b, gout, gpre, split;   // backward only
    size_t total;
};

int split_slices(int64_t rows) { int64_t s = (rows + 511) / 512; return (int)(s < 1 ? 1 : (s > 64 ? 64 : s)); }

Layout make_layout(const ukan_layer_desc *d, int64_t B, int64_t n_g, int n_chunks, size_t rec_bytes, int b_slices,
                   int pass)
{
    const size_t K = (size_t)d->k + 1, n_in = (size_t)d->n_in, n_out = (size_t)d->n_out;
    const size_t rows = n_in * (size_t)n_g, n_o = K * n_out, dz = (size_t)d->d_feat + d->d_pe, dh = (size_t)d->d_hidden;
    const size_t table = align_up(rows * n_o * sizeof(float));
    Layout L;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t here = at; at += align_up(bytes); return here; };
    L.cmin = take(n_in * 4); L.cmax = take(n_in * 4); L.g_first = take(n_in * 4);
    L.n_groups = take(n_in * 4); L.cell_base = take(n_in * 4); L.summary = take(256);
    L.hid = take(rows * dh * 4);
    L.cf = take(table);
    L.z = L.pre = L.raw = L.rec = L.part_c = L.part_b = L.gout = L.gpre = L.split = 0;
    if (pass == KAN_PASS_BACKWARD) {
        L.z = take(rows * dz * 4);
        L.pre = take(rows * dh * 4);
        L.raw = take(table);
        L.rec = take(rec_bytes);
        L.part_c = take((size_t)n_chunks * table);
        L.part_b = take((size_t)n_chunks * b_slices * n_in * n_out * 4);
        L.gout = take(table);
        L.gpre = take(rows * dh * 4);
        size_t s1 = (size_t)split_slices((int64_t)rows) * dh * n_o * 4;      // gW2 partials
        size_t s2 = (size_t)split_slices((int64_t)rows) * dz * dh * 4;       // gW1 partials
        size_t s3 = (size_t)colsum_slices((int64_t)rows) * (n_o > dh ? n_o : dh) * 4;
        size_t s = s1 > s2 ? s1 : s2;
        L.split = take(s > s3 ? s : s3);
    }
    L.total = at;
    return L;
}

// What the forward pass hands to the backward pass (ukan_cg_forward_saved): everything steps 1-2
// produce.  Offsets (bytes) into the caller's `saved` buffer for n_g generator rows per input.
struct SavedLayout { size_t g_first, cell_base, hid, cf, z, pre, raw, total; };

SavedLayout saved_layout(const ukan_layer_desc *d, int64_t n_g)
{
    const size_t K = (size_t)d->k + 1, n_in = (size_t)d->n_in, rows = n_in * (size_t)n_g;
    const size_t table = align_up(rows * K * (size_t)d->n_out * sizeof(float));
    const size_t dz = (size_t)d->d_feat + d->d_pe, dh = (size_t)d->d_hidden;
    SavedLayout S;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t here = at; at += align_up(bytes); return here; };
    S.g_first = take(n_in * 4); S.cell_base = take(n_in * 4);
    S.hid = take(rows * dh * 4); S.cf = take(table);
    S.z = take(rows * dz * 4); S.pre = take(rows * dh * 4); S.raw = take(table);
    S.total = at;
    return S;
}

// The products of steps 1-2, wherever they live (the workspace, or the caller's saved buffer).
struct Prepared {
    SplineGeom g;
    Layout L;          // scratch regions of the workspace
    int n_g;
    ChunkPlan cp;
    int32_t *g_first, *cell_base;
    float *hid, *cf, *z, *pre, *raw;     // z, pre, raw: null unless kept for the backward pass
};

void spline_geom(const ukan_layer_desc *d, int span, const int32_t *cell_base, SplineGeom *g)
{
    g->n_in = d->n_in; g->n_out = d->n_out;
    g->rows = span * (d->k + 1); g->slab_rows = g->rows; g->k = d->k;
    g->lo = 0.0f; g->inv_h = 1.0f / d->h;
    g->cell_base = cell_base;
    g->base_act = d->base_act;
}

// steps 1-2 of the pass: group range, read-back, CG forward into the table(s)
// With `saved` the products go to the caller's buffer (laid out for the span found) and z, pre and
// the unscaled table are kept whatever the pass.
// With provided_span > 0 nothing is read back: the table is built for that many groups per input and
// *overflow (device) says whether the batch needed more.
int prepare(const ukan_layer_desc *d, int64_t B, const float *x, const ukan_params *p, int32_t max_groups,
            char *ws, int pass, hipStream_t st, Prepared *out, char *saved = nullptr, int32_t provided_span = 0,
            int32_t *overflow = nullptr)
{
    const int K = d->k + 1;
    const float inv_h = 1.0f / d->h;
    out->cp = chunks_for(d, B, max_groups);
    Layout L0 = make_layout(d, B, max_groups, out->cp.n_chunks, record_bytes_for(d, B, max_groups), b_slices_for(d, B, max_groups), pass);     // meta offsets do not depend on n_g
    int32_t *cmin = (int32_t *)(ws + L0.cmin), *cmax = (int32_t *)(ws + L0.cmax);
    int32_t *n_groups = (int32_t *)(ws + L0.n_groups), *summary = (int32_t *)(ws + L0.summary);
    // the saved layout starts with g_first and cell_base at offsets that do not depend on the span
    const SavedLayout S0 = saved_layout(d, max_groups);
    int32_t *g_first = (int32_t *)(saved ? saved + S0.g_first : ws + L0.g_first);
    int32_t *cell_base = (int32_t *)(saved ? saved + S0.cell_base : ws + L0.cell_base);
    if (launch_range(x, B, d->n_in, inv_h, K, cmin, cmax, g_first, n_groups, cell_base, summary, st) != hipSuccess)
        return KAN_ERR_HIP;
    int32_t span = provided_span;
    if (provided_span > 0) {
        if (launch_span_check(summary, provided_span, overflow, st) != hipSuccess) return KAN_ERR_HIP;
    } else {
        if (hipMemcpyAsync(&span, summary, sizeof(span), hipMemcpyDeviceToHost, st) != hipSuccess) return KAN_ERR_HIP;
        if (hipStreamSynchronize(st) != hipSuccess) return KAN_ERR_HIP;
    }
    if (span < 2 || span > max_groups) return KAN_ERR_RANGE;
    out->n_g = span;
    out->L = make_layout(d, B, span, out->cp.n_chunks, record_bytes_for(d, B, max_groups), b_slices_for(d, B, max_groups), pass);
    const Layout &L = out->L;
    const int64_t rows = (int64_t)d->n_in * span;
    const int64_t n_o = (int64_t)K * d->n_out;

    const bool bwd = pass == KAN_PASS_BACKWARD;
    out->g_first = g_first; out->cell_base = cell_base;
    if (saved) {
        const SavedLayout S = saved_layout(d, span);
        out->hid = (float *)(saved + S.hid); out->cf = (float *)(saved + S.cf);
        out->z = (float *)(saved + S.z); out->pre = (float *)(saved + S.pre); out->raw = (float *)(saved + S.raw);
    } else {
        out->hid = (float *)(ws + L.hid); out->cf = (float *)(ws + L.cf);
        out->z = bwd ? (float *)(ws + L.z) : nullptr;
        out->pre = bwd ? (float *)(ws + L.pre) : nullptr;
        out->raw = bwd ? (float *)(ws + L.raw) : nullptr;
    }
    float *hid = out->hid;
    if (launch_cg_hidden(p->E, p->W1, p->b1, g_first, out->z, out->pre, hid, d->n_in, span, d->d_pe, d->d_feat,
                         d->d_hidden, st) != hipSuccess)
        return KAN_ERR_HIP;
    GemmArgs a = {};
    a.A = hid; a.a_rs = d->d_hidden; a.a_cs = 1;
    a.B = p->W2; a.b_rs = n_o; a.b_cs = 1;
    a.C = out->cf; a.ldc = n_o;
    a.M = rows; a.N = n_o; a.K = d->d_hidden;
    a.k_slice = d->d_hidden; a.c_slice = 0;
    a.bias = p->b2; a.scale = p->scale; a.C2 = out->raw;
    a.rows_per_input = span; a.n_out = d->n_out;
    if (launch_gemm(a, EPI_CG_OUT, 1, "cg_output_gemm", st) != hipSuccess) return KAN_ERR_HIP;

    spline_geom(d, span, cell_base, &out->g);
    return KAN_OK;
}

int check_common(const ukan_layer_desc *d, int64_t B, const float *x, const ukan_params *p, int32_t max_groups,
                 void *ws, size_t ws_bytes, int pass)
{
    int rc = check_desc(d);
    if (rc != KAN_OK) return rc;
    if (B < 0 || max_groups < 2) return KAN_ERR_INVALID_ARG;
    if (B == 0) return KAN_OK;
    if (!x || !p || !p->E || !p->W1 || !p->b1 || !p->W2 || !p->b2 || !p->scale) return KAN_ERR_INVALID_ARG;
    if (d->base_act != KAN_BASE_NONE && !p->w_b) return KAN_ERR_INVALID_ARG;
    for (const void *q : {(const void *)x, (const void *)p->E, (const void *)p->W1, (const void *)p->b1,
                          (const void *)p->W2, (const void *)p->b2, (const void *)p->scale, (const void *)p->w_b})
        if (q && ((uintptr_t)q % 16) != 0) return KAN_ERR_INVALID_ARG;
    size_t need = ukan_workspace_bytes(d, B, max_groups, pass);
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || need == 0 || ws_bytes < need) return KAN_ERR_WORKSPACE;
    return KAN_OK;
}

}  // namespace

extern "C" size_t ukan_workspace_bytes(const ukan_layer_desc *desc, int64_t B, int32_t max_groups, int pass)
{
    if (check_desc(desc) != KAN_OK || B < 0 || max_groups < 2) return 0;
    if (pass != KAN_PASS_FORWARD && pass != KAN_PASS_BACKWARD) return 0;
    ChunkPlan cp = chunks_for(desc, B, max_groups);
    return make_layout(desc, B, max_groups, cp.n_chunks, record_bytes_for(desc, B, max_groups),
                       b_slices_for(desc, B, max_groups), pass).total;
}

namespace {
int forward_impl(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p, float *y,
                 int32_t max_groups, void *ws, size_t ws_bytes, void *stream, char *saved, int32_t *span,
                 int32_t provided_span = 0, int32_t *overflow = nullptr)
{
    int rc = check_common(desc, B, x, p, max_groups, ws, ws_bytes, KAN_PASS_FORWARD);
    if (rc != KAN_OK || B == 0) return rc;
    if (!y || ((uintptr_t)y % 16) != 0) return KAN_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    Prepared pr;
    rc = prepare(desc, B, x, p, max_groups, (char *)ws, KAN_PASS_FORWARD, st, &pr, saved, provided_span, overflow);
    if (rc != KAN_OK) return rc;
    if (span) *span = pr.n_g;
    hipError_t e = high_degree(desc)                  ? highk_table_forward(highk_of(pr.g), x, pr.cf, p->w_b, y, B, st)
                   : narrow_applicable(pr.g)        ? launch_forward_narrow(pr.g, x, pr.cf, p->w_b, y, B, st)
                   : forward_lds_rows_plan(pr.g, B) ? launch_forward_lds_rows(pr.g, x, pr.cf, y, B, st)
                                                    : launch_forward_generic(pr.g, x, pr.cf, p->w_b, y, B, st);
    if (e != hipSuccess) return KAN_ERR_HIP;
    return KAN_OK;
}

int backward_body(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p, const float *gy,
                  float *gx, const ukan_grads *g, int32_t max_groups, char *w, const Prepared &pr, hipStream_t st);

int check_backward_args(const float *gy, const float *gx, const ukan_grads *g)
{
    if (!gy || ((uintptr_t)gy % 16) != 0 || ((uintptr_t)gx % 16) != 0) return KAN_ERR_INVALID_ARG;
    if (g)
        for (const void *q : {(const void *)g->gE, (const void *)g->gW1, (const void *)g->gb1, (const void *)g->gW2,
                              (const void *)g->gb2, (const void *)g->gscale, (const void *)g->gw_b})
            if (q && ((uintptr_t)q % 16) != 0) return KAN_ERR_INVALID_ARG;
    return KAN_OK;
}
}  // namespace

extern "C" int ukan_cg_forward(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                               float *y, int32_t max_groups, void *ws, size_t ws_bytes, void *stream)
{
    return forward_impl(desc, B, x, p, y, max_groups, ws, ws_bytes, stream, nullptr, nullptr);
}

extern "C" size_t ukan_saved_bytes(const ukan_layer_desc *desc, int32_t max_groups)
{
    if (check_desc(desc) != KAN_OK || max_groups < 2) return 0;
    return saved_layout(desc, max_groups).total;
}

extern "C" int ukan_cg_forward_saved(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                                     float *y, int32_t max_groups, void *saved, size_t saved_bytes, int32_t *span,
                                     void *ws, size_t ws_bytes, void *stream)
{
    if (!span) return KAN_ERR_INVALID_ARG;
    *span = 0;
    const size_t need = ukan_saved_bytes(desc, max_groups);
    if (need == 0) return check_desc(desc) != KAN_OK ? check_desc(desc) : KAN_ERR_INVALID_ARG;
    if (B > 0 && (!saved || ((uintptr_t)saved % kAlign) != 0 || saved_bytes < need)) return KAN_ERR_WORKSPACE;
    return forward_impl(desc, B, x, p, y, max_groups, ws, ws_bytes, stream, (char *)saved, span);
}

extern "C" int ukan_cg_forward_saved_async(const ukan_layer_desc *desc, int64_t B, const float *x,
                                           const ukan_params *p, float *y, int32_t max_groups, int32_t n_groups,
                                           void *saved, size_t saved_bytes, int32_t *overflow, void *ws,
                                           size_t ws_bytes, void *stream)
{
    const size_t need = ukan_saved_bytes(desc, max_groups);
    if (need == 0) return check_desc(desc) != KAN_OK ? check_desc(desc) : KAN_ERR_INVALID_ARG;
    if (n_groups < 2 || n_groups > max_groups) return KAN_ERR_RANGE;
    if (B > 0 && (!overflow || ((uintptr_t)overflow % 4) != 0)) return KAN_ERR_INVALID_ARG;
    if (B > 0 && (!saved || ((uintptr_t)saved % kAlign) != 0 || saved_bytes < need)) return KAN_ERR_WORKSPACE;
    return forward_impl(desc, B, x, p, y, max_groups, ws, ws_bytes, stream, (char *)saved, nullptr, n_groups, overflow);
}

extern "C" int ukan_cg_backward_saved(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                                      const float *gy, float *gx, const ukan_grads *g, int32_t max_groups,
                                      const void *saved, size_t saved_bytes, int32_t span, void *ws, size_t ws_bytes,
                                      void *stream)
{
    int rc = check_common(desc, B, x, p, max_groups, ws, ws_bytes, KAN_PASS_BACKWARD);
    if (rc != KAN_OK || B == 0) return rc;
    rc = check_backward_args(gy, gx, g);
    if (rc != KAN_OK) return rc;
    if (span < 2 || span > max_groups) return KAN_ERR_RANGE;
    if (!saved || ((uintptr_t)saved % kAlign) != 0 || saved_bytes < ukan_saved_bytes(desc, max_groups))
        return KAN_ERR_WORKSPACE;
    char *sv = (char *)saved;      // read only below
    Prepared pr;
    pr.n_g = span;
    pr.cp = chunks_for(desc, B, max_groups);
    pr.L = make_layout(desc, B, span, pr.cp.n_chunks, record_bytes_for(desc, B, max_groups),
                       b_slices_for(desc, B, max_groups), KAN_PASS_BACKWARD);
    const SavedLayout S = saved_layout(desc, span);
    pr.g_first = (int32_t *)(sv + S.g_first); pr.cell_base = (int32_t *)(sv + S.cell_base);
    pr.hid = (float *)(sv + S.hid); pr.cf = (float *)(sv + S.cf);
    pr.z = (float *)(sv + S.z); pr.pre = (float *)(sv + S.pre); pr.raw = (float *)(sv + S.raw);
    spline_geom(desc, span, pr.cell_base, &pr.g);
    return backward_body(desc, B, x, p, gy, gx, g, max_groups, (char *)ws, pr, (hipStream_t)stream);
}

extern "C" int ukan_cg_backward(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                                const float *gy, float *gx, const ukan_grads *g, int32_t max_groups, void *ws,
                                size_t ws_bytes, void *stream)
{
    int rc = check_common(desc, B, x, p, max_groups, ws, ws_bytes, KAN_PASS_BACKWARD);
    if (rc != KAN_OK || B == 0) return rc;
    rc = check_backward_args(gy, gx, g);
    if (rc != KAN_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    Prepared pr;
    rc = prepare(desc, B, x, p, max_groups, (char *)ws, KAN_PASS_BACKWARD, st, &pr);
    if (rc != KAN_OK) return rc;
    return backward_body(desc, B, x, p, gy, gx, g, max_groups, (char *)ws, pr, st);
}

namespace {
// steps after the coefficient table exists: dL/dx, the table gradient, and its way back through the CG
int backward_body(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p, const float *gy,
                  float *gx, const ukan_grads *g, int32_t max_groups, char *w, const Prepared &pr, hipStream_t st)
{
    const Layout &L = pr.L;
    const int K = desc->k + 1, dh = desc->d_hidden, dz = desc->d_feat + desc->d_pe;
    const int64_t rows = (int64_t)desc->n_in * pr.n_g, n_o = (int64_t)K * desc->n_out;

    const bool narrow = narrow_applicable(pr.g) != 0;
    const WalkPlan wp = walk_for(desc, B, max_groups);
    const bool fused_dx = gx && wp.ok;      // dL/dx rides along with the table gradient
    if (gx && !fused_dx) {
        hipError_t e = high_degree(desc) ? highk_table_dx(highk_of(pr.g), x, pr.cf, p->w_b, gy, gx, B, st)
                       : narrow          ? launch_dx_narrow(pr.g, x, pr.cf, p->w_b, gy, gx, B, st)
                                         : launch_dx_generic(pr.g, x, pr.cf, p->w_b, gy, gx, B, st);
        if (e != hipSuccess) return KAN_ERR_HIP;
    }

    const bool cg_grads = g && (g->gE || g->gW1 || g->gb1 || g->gW2 || g->gb2);
    const bool want_b = g && g->gw_b && desc->base_act != KAN_BASE_NONE;
    const bool want_params = cg_grads || (g && (g->gscale || g->gw_b));
    if (!want_params && !fused_dx) return KAN_OK;

    // table gradient: partial sums per batch chunk, then  gout = scale * sum,  gscale = sum_m raw * sum
    float *part_c = (float *)(w + L.part_c), *part_b = (float *)(w + L.part_b);
    float *gout = (float *)(w + L.gout);
    int b_slices;
    if (wp.ok) {
        if (launch_backward_walk(pr.g, wp, x, gy, pr.cf, p->w_b, w + L.rec, fused_dx ? gx : nullptr,
                                 want_params ? part_c : nullptr, want_b ? part_b : nullptr, B, st) != hipSuccess)
            return KAN_ERR_HIP;
        b_slices = pr.cp.n_chunks * wp.n_seg;
    } else {
        hipError_t e = high_degree(desc)
                           ? highk_table_dparam(highk_of(pr.g), x, gy, part_c, want_b ? part_b : nullptr, B,
                                                pr.cp.n_chunks, pr.cp.chunk_len, st)
                           : launch_dparam_generic(pr.g, x, gy, part_c, want_b ? part_b : nullptr, B, pr.cp.n_chunks,
                                                   pr.cp.chunk_len, st);
        if (e != hipSuccess) return KAN_ERR_HIP;
        b_slices = pr.cp.n_chunks * row_blocks_for(desc, pr.g.rows);
    }
    if (!want_params) return KAN_OK;
    if (launch_dparam_reduce(part_c, want_b ? part_b : nullptr, pr.raw, p->scale,
                             cg_grads ? gout : nullptr, g->gscale, g->gw_b, desc->n_in, pr.g.rows, desc->n_out,
                             pr.cp.n_chunks, b_slices, st) != hipSuccess)
        return KAN_ERR_HIP;
    if (!cg_grads) return KAN_OK;

    float *split = (float *)(w + L.split);
    const float *hid = pr.hid;
    float *gpre = (float *)(w + L.gpre);
    const int slices = split_slices(rows);
    int64_t k_slice = (rows + slices - 1) / slices;
    k_slice = (k_slice + 15) / 16 * 16;

    if (g->gb2 && launch_colsum(gout, split, g->gb2, rows, (int)n_o, st) != hipSuccess) return KAN_ERR_HIP;
    if (g->gW2) {       // gW2[c][o] = sum_rows hid[row][c] * gout[row][o]
        GemmArgs a = {};
        a.A = hid; a.a_rs = 1; a.a_cs = dh;
        a.B = gout; a.b_rs = n_o; a.b_cs = 1;
        a.C = split; a.ldc = n_o; a.M = dh; a.N = n_o; a.K = rows;
        a.k_slice = k_slice; a.c_slice = (int64_t)dh * n_o;
        const int used = (int)((rows + k_slice - 1) / k_slice);
        if (launch_gemm(a, EPI_PLAIN, used, "cg_gW2_gemm", st) != hipSuccess) return KAN_ERR_HIP;
        if (launch_slice_sum(split, g->gW2, (int64_t)dh * n_o, used, st) != hipSuccess) return KAN_ERR_HIP;
    }
    if (g->gE || g->gW1 || g->gb1) {
        GemmArgs a = {};    // gpre[row][c] = (sum_o gout[row][o] * W2[c][o]) * silu'(pre[row][c])
        a.A = gout; a.a_rs = n_o; a.a_cs = 1;
        a.B = p->W2; a.b_rs = 1; a.b_cs = n_o;
        a.C = gpre; a.ldc = dh; a.M = rows; a.N = dh; a.K = n_o;
        a.k_slice = n_o; a.c_slice = 0;
        a.aux = pr.pre;
        if (launch_gemm(a, EPI_SILU_GRAD, 1, "cg_ghid_gemm", st) != hipSuccess) return KAN_ERR_HIP;
        if (g->gb1 && launch_colsum(gpre, split, g->gb1, rows, dh, st) != hipSuccess) return KAN_ERR_HIP;
        if (g->gW1) {   // gW1[p][c] = sum_rows z[row][p] * gpre[row][c]
            GemmArgs b = {};
            b.A = pr.z; b.a_rs = 1; b.a_cs = dz;
            b.B = gpre; b.b_rs = dh; b.b_cs = 1;
            b.C = split; b.ldc = dh; b.M = dz; b.N = dh; b.K = rows;
            b.k_slice = k_slice; b.c_slice = (int64_t)dz * dh;
            const int used = (int)((rows + k_slice - 1) / k_slice);
            if (launch_gemm(b, EPI_PLAIN, used, "cg_gW1_gemm", st) != hipSuccess) return KAN_ERR_HIP;
            if (launch_slice_sum(split, g->gW1, (int64_t)dz * dh, used, st) != hipSuccess) return KAN_ERR_HIP;
        }
        if (g->gE && desc->d_feat > 0 &&
            launch_embed_grad(p->W1, gpre, g->gE, desc->n_in, pr.n_g, desc->d_feat, dh, st) != hipSuccess)
            return KAN_ERR_HIP;
    }
    return KAN_OK;
}
}  // namespace

namespace {
inline int64_t floordiv64(int64_t a, int64_t b) { int64_t q = a / b; return (a % b != 0 && ((a < 0) != (b < 0))) ? q - 1 : q; }

// groups the export needs: global coefficients cell_lo - K .. cell_hi - 1
struct ExportPlan { int64_t g_first, n_g; size_t gf_off, hid_off, table_off, total; };
bool export_plan(const ukan_layer_desc *d, int64_t cell_lo, int64_t cell_hi, ExportPlan *e)
{
    const int64_t K = d->k + 1;
    if (cell_hi < cell_lo || cell_lo < -(1ll << 30) || cell_hi > (1ll << 30)) return false;
    e->g_first = floordiv64(cell_lo - K, K);
    e->n_g = floordiv64(cell_hi - 1, K) - e->g_first + 1;
    if (e->n_g < 1 || e->n_g > (1 << 20)) return false;
    const size_t rows = (size_t)d->n_in * (size_t)e->n_g;
    size_t at = 0;
    e->gf_off = at;    at += align_up((size_t)d->n_in * 4);
    e->hid_off = at;   at += align_up(rows * d->d_hidden * 4);
    e->table_off = at; at += align_up(rows * K * d->n_out * 4);
    e->total = at;
    return true;
}
}  // namespace

extern "C" size_t ukan_materialize_workspace_bytes(const ukan_layer_desc *desc, int64_t cell_lo, int64_t cell_hi)
{
    ExportPlan e;
    if (check_desc(desc) != KAN_OK || !export_plan(desc, cell_lo, cell_hi, &e)) return 0;
    return e.total;
}

extern "C" int ukan_materialize(const ukan_layer_desc *desc, const ukan_params *p, int64_t cell_lo, int64_t cell_hi,
                                float *coef, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != KAN_OK) return rc;
    ExportPlan e;
    if (!export_plan(desc, cell_lo, cell_hi, &e)) return KAN_ERR_INVALID_ARG;
    if (!p || !p->E || !p->W1 || !p->b1 || !p->W2 || !p->b2 || !p->scale || !coef) return KAN_ERR_INVALID_ARG;
    if (((uintptr_t)coef % 16) != 0) return KAN_ERR_INVALID_ARG;
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < e.total) return KAN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *w = (char *)ws;
    const int K = desc->k + 1;
    int32_t *g_first = (int32_t *)(w + e.gf_off);
    float *hid = (float *)(w + e.hid_off), *table = (float *)(w + e.table_off);
    if (launch_fill_int(g_first, (int32_t)e.g_first, desc->n_in, st) != hipSuccess) return KAN_ERR_HIP;
    if (launch_cg_hidden(p->E, p->W1, p->b1, g_first, nullptr, nullptr, hid, desc->n_in, (int)e.n_g, desc->d_pe,
                         desc->d_feat, desc->d_hidden, st) != hipSuccess)
        return KAN_ERR_HIP;
    const int64_t n_o = (int64_t)K * desc->n_out;
    GemmArgs a = {};
    a.A = hid; a.a_rs = desc->d_hidden; a.a_cs = 1;
    a.B = p->W2; a.b_rs = n_o; a.b_cs = 1;
    a.C = table; a.ldc = n_o;
    a.M = (int64_t)desc->n_in * e.n_g; a.N = n_o; a.K = desc->d_hidden;
    a.k_slice = desc->d_hidden; a.c_slice = 0;
    a.bias = p->b2; a.scale = p->scale; a.C2 = nullptr;
    a.rows_per_input = e.n_g; a.n_out = desc->n_out;
    if (launch_gemm(a, EPI_CG_OUT, 1, "cg_output_gemm", st) != hipSuccess) return KAN_ERR_HIP;
    // table row r of an input is global coefficient g_first*K + r; coef row m is global coefficient cell_lo - K + m
    const int shift = (int)(cell_lo - K - e.g_first * K);
    const int coef_rows = (int)(cell_hi - cell_lo + 1) + desc->k;
    if (launch_table_rows(table, coef, desc->n_in, (int)(e.n_g * K), coef_rows, shift, desc->n_out, st) != hipSuccess)
        return KAN_ERR_HIP;
    return KAN_OK;
}

extern "C" int ukan_group_index(const ukan_layer_desc *desc, int64_t n, const float *x, int32_t *cell,
                                int32_t *group, int32_t *offset, void *stream)
{
    int rc = check_desc(desc);
    if (rc != KAN_OK) return rc;
    if (n < 0) return KAN_ERR_INVALID_ARG;
    if (n == 0) return KAN_OK;
    if (!x) return KAN_ERR_INVALID_ARG;
    if (launch_group_index(x, cell, group, offset, n, 1.0f / desc->h, desc->k + 1, (hipStream_t)stream) != hipSuccess)
        return KAN_ERR_HIP;
    return KAN_OK;
}
