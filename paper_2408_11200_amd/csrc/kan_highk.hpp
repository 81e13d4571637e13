// Degrees 4 and 5: the generic kernels compiled for a window of 6 rows (kan_generic_k5.hip).  Plain
// argument types only, so that callers built for the default window can use it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kan {

struct HighKLayer {
    int n_in, n_out, rows, k;       // rows = G + k
    float lo, inv_h;
    int base_act;
    // optional (zero-initialise the struct): a table of slab_rows rows per input (0: rows + 1, the last one w_b) whose
    // first row is cell cell_base[i] of input i (device pointer; null: cell 0)
    int slab_rows;
    const int *cell_base;
};

int highk_row_blocks(int rows);     // base-term partial slices per chunk
// y = layer(x); cf: scratch for the scale-folded table ((rows + 1) rows per input)
hipError_t highk_forward(const HighKLayer &l, const float *x, const float *coef, const float *w_s, const float *w_b,
                         float *cf, float *y, int64_t B, hipStream_t st);
// any of gx / (gcoef, gw_s, gw_b) may be null; part_c: n_chunks tables of rows rows, part_b: n_chunks *
// highk_row_blocks(rows) edge slices
hipError_t highk_backward(const HighKLayer &l, const float *x, const float *coef, const float *w_s, const float *w_b,
                          const float *gy, float *cf, float *gx, float *gcoef, float *gw_s, float *gw_b,
                          float *part_c, float *part_b, int n_chunks, int64_t chunk_len, int64_t B, hipStream_t st);

// The generic kernels on an existing table (UKAN layers of degree 4 and 5): forward, dL/dx, and the per-chunk
// partial sums of the table gradient (part_c: n_chunks tables of rows rows, part_b: n_chunks * highk_row_blocks(rows)
// edge slices or null).  w_b may be null.
hipError_t highk_table_forward(const HighKLayer &l, const float *x, const float *table, const float *w_b, float *y,
                               int64_t B, hipStream_t st);
hipError_t highk_table_dx(const HighKLayer &l, const float *x, const float *table, const float *w_b, const float *gy,
                          float *gx, int64_t B, hipStream_t st);
hipError_t highk_table_dparam(const HighKLayer &l, const float *x, const float *gy, float *part_c, float *part_b,
                              int64_t B, int n_chunks, int64_t chunk_len, hipStream_t st);

// Sorted records of the walk for degrees 4 and 5 (kan_walk_k5.hip): per (chunk of S samples, input) a list of
// 2 S records in the four-row format of the walk, two per pair (rows 0..3 of its six-row window with the base
// term; rows 4..5), sorted by first row.  xT is the transposed input [n_in][B]; rt / base / w4 (and dbase / dw4
// when not null) are the record arrays, [chunk][input][2 S].  S: a power of two, 256 .. 4096.
hipError_t highk_sorted_records(const HighKLayer &l, const float *xT, int64_t B, int S, int row_bits, int *rt,
                                float *base, float *w4, float *dbase, float *dw4, hipStream_t st);

}  // namespace kan
