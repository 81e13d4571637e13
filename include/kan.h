/*
 * kan.h - C ABI of the MI355X (gfx950) B-spline KAN / UKAN layer library.
 *
 * The library computes, on one GPU and in fp32, the forward and backward pass
 * of one Kolmogorov-Arnold layer in its local B-spline form, and of the UKAN
 * variant whose coefficients come from a coefficient-generator (CG) MLP.
 * Citations name sections / equations of arXiv 2408.11200.
 *
 * Conventions that hold for every entry point
 *   - Every pointer argument is DEVICE memory owned by the caller unless it is
 *     a descriptor / parameter struct, which is HOST memory read during the
 *     call.  The library allocates nothing, links nothing but the HIP runtime
 *     and keeps no state between calls (the two exceptions, the launch observer
 *     and the built-in array of kan_forward_static, say so where they are
 *     declared); scratch space comes in through (ws, ws_bytes) and must be at
 *     least what the matching *_workspace_bytes call returns (256-byte aligned).
 *   - `stream` is a hipStream_t passed as void*.  All work is enqueued on it.
 *     kan_* calls never synchronise; ukan_cg_forward, ukan_cg_backward and
 *     ukan_cg_forward_saved synchronise the stream once to read back the group
 *     span (4 bytes), see below; the other ukan_* calls do not.
 *   - Every float array must be 16-byte aligned (KAN_ERR_INVALID_ARG otherwise).
 *   - Row-major layouts:  x[B][n_in]  y,gy[B][n_out]  gx[B][n_in]
 *       coef,gcoef[n_in][G+k][n_out]   w_s,w_b,gw_s,gw_b[n_in][n_out]
 *   - Return value: KAN_OK or a negative kan_status; nothing is thrown.  B == 0
 *     succeeds and touches nothing.  Gradient outputs are overwritten, not
 *     accumulated; any gradient output pointer may be NULL to skip it.
 *   - Inputs are expected finite.  A non-finite x gets a zero spline term and
 *     propagates through the base term only.
 *
 * Grid convention: G cells on [grid_lo, grid_hi), degree k, k extra knots on
 * each side, G + k coefficients per edge.  The cell width enters as the fp32
 * number inv_h = (float)G / (grid_hi - grid_lo), computed once on the host.
 * Interval index (section "Algorithm", text after Eq. "matrixform"):
 *   idx = floorf((x - grid_lo) * inv_h)   with separately rounded fp32 subtract
 *   and multiply.  Cells -k..-1 and G..G+k-1 are padding cells (part of the
 *   window falls off the coefficient array and contributes zero); beyond them
 *   the spline and its derivative are zero.
 */
#ifndef KAN_H
#define KAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kan_status {
    KAN_OK = 0,
    KAN_ERR_INVALID_ARG = -1, /* null or misaligned pointer, non-positive size, grid_hi <= grid_lo, h <= 0 */
    KAN_ERR_UNSUPPORTED = -2, /* k outside 1..5, n_in above 65535, unknown base_act, odd d_pe */
    KAN_ERR_WORKSPACE = -3,   /* ws is NULL / misaligned / smaller than *_workspace_bytes     */
    KAN_ERR_RANGE = -4,       /* UKAN: some input spans more groups than max_groups           */
    KAN_ERR_HIP = -5          /* a HIP runtime call or kernel launch failed                   */
} kan_status;

enum { KAN_BASE_NONE = 0, KAN_BASE_SILU = 1 };
enum { KAN_PASS_FORWARD = 0, KAN_PASS_BACKWARD = 1 };

/* One bounded-grid layer (Eqs. "activation", "kanphi", "kanspline"): widths n_l, n_{l+1},
   grid size G (cells), degree k (1..5), grid range.  base_act selects b(x) of Eq. "kanphi". */
typedef struct kan_layer_desc {
    int32_t n_in, n_out;
    int32_t G, k;
    float grid_lo, grid_hi;
    int32_t base_act;
} kan_layer_desc;

/* One UKAN layer (section "Algorithm", CG paragraph): unbounded grid t_j = j*h, degree k (1..5),
   groups of K = k+1 cells; CG input = [feature embedding (d_feat) ; sinusoidal PE of the group
   index (d_pe)], one hidden layer of d_hidden units with SiLU, K*n_out outputs.           */
typedef struct ukan_layer_desc {
    int32_t n_in, n_out;
    int32_t k;
    float h;
    int32_t d_pe, d_feat, d_hidden;
    int32_t base_act;
} ukan_layer_desc;

/* CG parameters (device pointers).  E[n_in][d_feat]; W1[d_feat+d_pe][d_hidden] (embedding rows
   first); b1[d_hidden]; W2[d_hidden][K*n_out] with output index q*n_out + j; b2[K*n_out];
   scale[n_in][n_out] multiplies the generated coefficients; w_b[n_in][n_out] is read only when
   base_act != 0 (may be NULL otherwise). */
typedef struct ukan_params {
    const float *E, *W1, *b1, *W2, *b2, *scale, *w_b;
} ukan_params;

/* Gradients of the above, same shapes; any member may be NULL. */
typedef struct ukan_grads {
    float *gE, *gW1, *gb1, *gW2, *gb2, *gscale, *gw_b;
} ukan_grads;

/* Human-readable name of a status code (static string). */
const char *kan_strerror(int status);

/* Scratch bytes needed by kan_forward (pass = KAN_PASS_FORWARD) or kan_backward for batch B.
   Returns 0 for an invalid descriptor.  Forward: the scale-folded table.  Backward: that, the transposed input, two
   sorted record arrays (44 bytes per (sample, input) pair) and the per-chunk partial gradient tables: a small multiple
   of B * n_in * 48 bytes + at most 2 GiB of partial tables (more only when a single table exceeds that). */
size_t kan_workspace_bytes(const kan_layer_desc *desc, int64_t B, int pass);

/* Forward pass of one layer, Eqs. "activation" + "kanphi" + "matrixform":
     y[b][j] = sum_i ( w_s[i][j] * sum_{s=0..k} coef[i][idx+s][j] * N_s(u) + w_b[i][j] * silu(x[b][i]) )
   with idx, u the cell and local coordinate of x[b][i] and N_s the k+1 non-zero Cox-de Boor
   basis values of that cell.  w_b may be NULL when base_act == KAN_BASE_NONE.  Writes y. */
int kan_forward(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                const float *w_s, const float *w_b, float *y, void *ws, size_t ws_bytes,
                void *stream);

/* Backward pass of the same layer given gy = dL/dy:
     gx[b][i]       = sum_j gy[b][j] ( w_s[i][j] sum_s coef[i][idx+s][j] dN_s/dx + w_b[i][j] silu'(x[b][i]) )
     gcoef[i][m][j] = w_s[i][j] sum_b gy[b][j] N_{m-idx(b,i)}(u(b,i))
     gw_s[i][j]     = sum_b gy[b][j] spline_ij(x[b][i])
     gw_b[i][j]     = sum_b gy[b][j] silu(x[b][i])
   The batch reduction runs in a fixed order (no atomics whose order could vary): repeated
   calls give bit-identical gradients. */
int kan_backward(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                 const float *w_s, const float *w_b, const float *gy, float *gx, float *gcoef,
                 float *gw_s, float *gw_b, void *ws, size_t ws_bytes, void *stream);

/* kan_backward for a training step that has just run kan_forward on the same layer: forward_ws is the
   workspace that kan_forward call was given (it holds the scale-folded table, the first
   kan_workspace_bytes(desc, B, KAN_PASS_FORWARD) bytes), untouched since, with coef, w_s and w_b unchanged;
   the backward pass then reads the table from there instead of folding it again.  forward_ws must not be
   the same buffer as ws (KAN_ERR_INVALID_ARG); NULL or misaligned gives KAN_ERR_WORKSPACE.  The library
   cannot check that the table is current.  Results are bit-identical to kan_backward. */
int kan_backward_saved(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                       const float *w_s, const float *w_b, const float *gy, const void *forward_ws,
                       float *gx, float *gcoef, float *gw_s, float *gw_b, void *ws, size_t ws_bytes,
                       void *stream);

/* kan_forward for callers that cannot allocate device memory (code running under HIP graph capture, tight
   serving loops, harnesses that forbid hipMalloc): same arguments and result as kan_forward, but the scratch
   space is a fixed array of KAN_STATIC_SCRATCH_BYTES that is part of the library's device code, so there is
   no (ws, ws_bytes) to provide and the call allocates nothing.  Each GPU holds its own copy of the array
   from the first call on it until the process ends.  Returns KAN_ERR_WORKSPACE when
   kan_workspace_bytes(desc, B, KAN_PASS_FORWARD) exceeds KAN_STATIC_SCRATCH_BYTES (y is not written),
   KAN_ERR_HIP when the array's address cannot be obtained.  All calls on one GPU share the array: calls that
   may overlap in time on the same GPU (different streams or threads) race on it; calls on one stream do not.
   kan_static_scratch_bytes() returns the limit. */
#define KAN_STATIC_SCRATCH_BYTES (32u << 20)
size_t kan_static_scratch_bytes(void);
int kan_forward_static(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                       const float *w_s, const float *w_b, float *y, void *stream);

/* Parity aid: idx[p] = interval index of x[p] for p < n (the integer the forward pass uses
   before any clamping), saturated to +-2^30. */
int kan_interval_index(const kan_layer_desc *desc, int64_t n, const float *x, int32_t *idx,
                       void *stream);

/* ---- launch observer ---------------------------------------------------------------------- */

/* Two optional host callbacks, process-wide: `before` is called on the calling thread right before
   each kernel launch of the library is enqueued and `after` right after it, with a static string
   naming the kernel family and the launch stream.  Either may be NULL; (NULL, NULL), the initial
   state, switches the observer off.  The two pointers are the only state the library keeps besides
   the array of kan_forward_static.  Meant for measurement (the benchmark library of kan_bench.h
   records a HIP event in each); do not change the observer while another thread is inside a call. */
typedef void (*kan_launch_hook)(const char *family, void *stream);
int kan_set_launch_observer(kan_launch_hook before, kan_launch_hook after);

/* ---- UKAN ------------------------------------------------------------------------------ */

/* Scratch bytes for ukan_cg_forward / ukan_cg_backward.  max_groups bounds, per input, the
   number of consecutive groups (g_min-1 .. g_max) the coefficient table may hold. */
size_t ukan_workspace_bytes(const ukan_layer_desc *desc, int64_t B, int32_t max_groups, int pass);

/* UKAN forward (section "Algorithm": cell i(x) = floor(x/h), group g = floor(i/K), offset
   r = i mod K, window = entries r..r+K-1 of [C_{g-1};C_g]):
     1. per input, the range of groups the batch touches (device reduction over x);
     2. CG forward for exactly those (input, group) rows -> coefficient table in ws;
     3. local B-spline evaluation on the table, as kan_forward with scale in the role of w_s.
   Synchronises `stream` once after step 1 to read the widest group span; returns
   KAN_ERR_RANGE if it exceeds max_groups (y is then not written). */
int ukan_cg_forward(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                    float *y, int32_t max_groups, void *ws, size_t ws_bytes, void *stream);

/* UKAN backward given gy: gx (through the local coordinate only; the group index is piecewise
   constant), and the gradients of every CG parameter, of scale and of w_b.  Recomputes steps 1-2
   of the forward pass; same synchronisation and error behaviour.  A training step that has run the
   forward pass on the same x and parameters should use the *_saved pair below instead. */
int ukan_cg_backward(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                     const float *gy, float *gx, const ukan_grads *g, int32_t max_groups, void *ws,
                     size_t ws_bytes, void *stream);

/* Forward -> backward hand-off for training.  ukan_cg_forward_saved is ukan_cg_forward that also
   keeps what steps 1-2 produced (first group and cell offset of every input, the CG's input rows,
   hidden pre-activations and activations, the coefficient table with and without the scale) in
   `saved`, caller-owned device memory of at least ukan_saved_bytes(desc, max_groups) bytes,
   256-byte aligned, and writes the widest group span to *span (HOST memory; 0 on failure).
   ukan_cg_backward_saved takes that buffer and span and runs only the steps after the table:
   no range scan, no CG forward, no synchronisation.  x, p's contents and max_groups must be the
   ones of the forward call, and `saved` must not have been written since; the library cannot
   check this.  Results are bit-identical to ukan_cg_backward.  ws as for the unsaved calls
   (ukan_workspace_bytes with the matching pass).  Errors as above; a span outside 2..max_groups
   gives KAN_ERR_RANGE, a short or misaligned `saved` KAN_ERR_WORKSPACE. */
size_t ukan_saved_bytes(const ukan_layer_desc *desc, int32_t max_groups);
int ukan_cg_forward_saved(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                          float *y, int32_t max_groups, void *saved, size_t saved_bytes, int32_t *span,
                          void *ws, size_t ws_bytes, void *stream);
/* ukan_cg_forward_saved without the read-back: the caller states how many groups per input to provide for
   (n_groups, 2 .. max_groups: e.g. the span an earlier call reported plus a margin) and the call only
   enqueues kernels, so it can be captured in a HIP graph.  It writes 1 to *overflow (DEVICE memory, one
   int32) when some input of this batch spans more groups than n_groups, else 0; with 1, y and `saved` are
   not valid (samples beyond the provided groups contributed nothing) and the call should be repeated with a
   larger n_groups.  Hand n_groups to ukan_cg_backward_saved as its span. */
int ukan_cg_forward_saved_async(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                                float *y, int32_t max_groups, int32_t n_groups, void *saved, size_t saved_bytes,
                                int32_t *overflow, void *ws, size_t ws_bytes, void *stream);
int ukan_cg_backward_saved(const ukan_layer_desc *desc, int64_t B, const float *x, const ukan_params *p,
                           const float *gy, float *gx, const ukan_grads *g, int32_t max_groups,
                           const void *saved, size_t saved_bytes, int32_t span, void *ws, size_t ws_bytes,
                           void *stream);

/* UKAN -> KAN export (appendix "UKAN mapping to KAN in Inference"): the coefficients of the bounded-grid layer that
   equals this UKAN layer on the cells cell_lo .. cell_hi, i.e. on [cell_lo*h, (cell_hi+1)*h):
     coef[i][m][j] = scale[i][j] * CG(i, g)[q*n_out + j],   g*K + q = cell_lo - K + m,   m = 0 .. G + k - 1,
   G = cell_hi - cell_lo + 1.  Use it with kan_layer_desc{n_in, n_out, G, k, cell_lo*h, (cell_hi+1)*h, base_act},
   w_s = 1 and the same w_b.  coef is [n_in][G + k][n_out], device memory, 16-byte aligned.  Does not synchronise. */
size_t ukan_materialize_workspace_bytes(const ukan_layer_desc *desc, int64_t cell_lo, int64_t cell_hi);
int ukan_materialize(const ukan_layer_desc *desc, const ukan_params *p, int64_t cell_lo, int64_t cell_hi,
                     float *coef, void *ws, size_t ws_bytes, void *stream);

/* Parity aid: cell, group and within-group offset of x[p], p < n (any output may be NULL). */
int ukan_group_index(const ukan_layer_desc *desc, int64_t n, const float *x, int32_t *cell,
                     int32_t *group, int32_t *offset, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KAN_H */
