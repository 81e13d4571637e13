// Launch functions of the UKAN-specific kernels (cell/group bookkeeping, CG MLP).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kan {

enum { EPI_PLAIN = 0, EPI_CG_OUT = 1, EPI_SILU_GRAD = 2 };

// C(m,n) = sum_k A(m,k) B(k,n); element (r,c) of an operand is at base[r*rs + c*cs].
struct GemmArgs {
    const float *A; int64_t a_rs, a_cs;
    const float *B; int64_t b_rs, b_cs;
    float *C; int64_t ldc;
    int64_t M, N, K;
    int64_t k_slice;        // K range per blockIdx.z
    int64_t c_slice;        // distance between the C copies of consecutive K slices
    // epilogue operands
    const float *bias;      // EPI_CG_OUT: b2[N]
    const float *scale;     // EPI_CG_OUT: scale[n_in][n_out]
    float *C2;              // EPI_CG_OUT: optional raw (unscaled) copy
    const float *aux;       // EPI_SILU_GRAD: pre-activations, same shape as C
    int64_t rows_per_input; // EPI_CG_OUT: generator rows per input
    int n_out;
};

inline int colsum_slices(int64_t rows) { int64_t s = (rows + 255) / 256; return (int)(s < 1 ? 1 : (s > 256 ? 256 : s)); }

hipError_t launch_group_index(const float *x, int32_t *cell, int32_t *grp, int32_t *off, int64_t n, float inv_h,
                              int K, hipStream_t st);
hipError_t launch_range(const float *x, int64_t B, int n_in, float inv_h, int K, int32_t *cmin, int32_t *cmax,
                        int32_t *g_first, int32_t *n_groups, int32_t *cell_base, int32_t *summary, hipStream_t st);
hipError_t launch_span_check(const int32_t *summary, int provided, int32_t *overflow, hipStream_t st);
hipError_t launch_cg_hidden(const float *E, const float *W1, const float *b1, const int32_t *g_first, float *z,
                            float *pre, float *hid, int n_in, int n_g, int d_pe, int d_feat, int d_hid,
                            hipStream_t st);
hipError_t launch_fill_int(int32_t *p, int32_t v, int n, hipStream_t st);
hipError_t launch_table_rows(const float *table, float *coef, int n_in, int table_rows, int coef_rows, int shift,
                             int n_out, hipStream_t st);
hipError_t launch_gemm(const GemmArgs &a, int epi, int slices, const char *family, hipStream_t st);
hipError_t launch_colsum(const float *A, float *part, float *out, int64_t rows, int cols, hipStream_t st);
hipError_t launch_slice_sum(const float *part, float *out, int64_t n, int slices, hipStream_t st);
hipError_t launch_embed_grad(const float *W1, const float *gpre, float *gE, int n_in, int n_g, int d_feat,
                             int d_hid, hipStream_t st);

}  // namespace kan
