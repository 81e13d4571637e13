// The generic kernels and the row-stream forward kernel once more, for spline degrees 4 and 5 (window of
// 6 rows).  Everything in kan_generic.hip and kan_rows.hip is written against kMaxK; this translation unit
// compiles them with kMaxK = 6 in a namespace of its own and exposes them through kan_highk.hpp.
#define KAN_MAXK 6
#define KAN_NS kan_k5
#include "kan_generic.hip"
#include "kan_rows.hip"
#include "kan_highk.hpp"

namespace kan {

namespace {
kan_k5::SplineGeom geom_of(const HighKLayer &l)
{
    kan_k5::SplineGeom g;
    g.n_in = l.n_in; g.n_out = l.n_out; g.rows = l.rows; g.slab_rows = l.slab_rows ? l.slab_rows : l.rows + 1; g.k = l.k;
    g.lo = l.lo; g.inv_h = l.inv_h; g.cell_base = l.cell_base; g.base_act = l.base_act;
    return g;
}
}  // namespace

hipError_t highk_table_forward(const HighKLayer &l, const float *x, const float *table, const float *w_b, float *y,
                               int64_t B, hipStream_t st)
{
    return kan_k5::launch_forward_generic(geom_of(l), x, table, w_b, y, B, st);
}

hipError_t highk_table_dx(const HighKLayer &l, const float *x, const float *table, const float *w_b, const float *gy,
                          float *gx, int64_t B, hipStream_t st)
{
    return kan_k5::launch_dx_generic(geom_of(l), x, table, w_b, gy, gx, B, st);
}

hipError_t highk_table_dparam(const HighKLayer &l, const float *x, const float *gy, float *part_c, float *part_b,
                              int64_t B, int n_chunks, int64_t chunk_len, hipStream_t st)
{
    return kan_k5::launch_dparam_generic(geom_of(l), x, gy, part_c, part_b, B, n_chunks, chunk_len, st);
}

int highk_row_blocks(int rows) { return kan_k5::dparam_generic_row_blocks(rows); }

hipError_t highk_forward(const HighKLayer &l, const float *x, const float *coef, const float *w_s, const float *w_b,
                         float *cf, float *y, int64_t B, hipStream_t st)
{
    const kan_k5::SplineGeom g = geom_of(l);
    hipError_t e = kan_k5::launch_fold_scale(coef, w_s, g.base_act ? w_b : nullptr, cf, g.n_in, g.rows, g.n_out, st);
    if (e != hipSuccess) return e;
    if (kan_k5::forward_rows_plan(g)) return kan_k5::launch_forward_rows(g, x, cf, y, B, st);
    if (kan_k5::forward_lds_plan(g)) return kan_k5::launch_forward_lds(g, x, cf, y, B, st);
    return kan_k5::launch_forward_generic(g, x, cf, w_b, y, B, st);
}

hipError_t highk_backward(const HighKLayer &l, const float *x, const float *coef, const float *w_s, const float *w_b,
                          const float *gy, float *cf, float *gx, float *gcoef, float *gw_s, float *gw_b,
                          float *part_c, float *part_b, int n_chunks, int64_t chunk_len, int64_t B, hipStream_t st)
{
    const kan_k5::SplineGeom g = geom_of(l);
    hipError_t e;
    if (gx) {
        e = kan_k5::launch_fold_scale(coef, w_s, g.base_act ? w_b : nullptr, cf, g.n_in, g.rows, g.n_out, st);
        if (e != hipSuccess) return e;
        e = kan_k5::launch_dx_generic(g, x, cf, w_b, gy, gx, B, st);
        if (e != hipSuccess) return e;
    }
    if (gcoef || gw_s || gw_b) {
        const bool want_b = gw_b && g.base_act;
        e = kan_k5::launch_dparam_generic(g, x, gy, part_c, want_b ? part_b : nullptr, B, n_chunks, chunk_len, st);
        if (e != hipSuccess) return e;
        e = kan_k5::launch_dparam_reduce(part_c, want_b ? part_b : nullptr, coef, w_s, gcoef, gw_s, gw_b, g.n_in, g.rows,
                                         g.n_out, n_chunks, n_chunks * kan_k5::dparam_generic_row_blocks(g.rows), st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace kan
