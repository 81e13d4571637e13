/*
 * kan_bench.h - C ABI of the benchmark companion library (libkan_bench.so).
 *
 * Measurement aids for the layer library of kan.h, kept in a library of their own so that the
 * layer library stays free of state, of allocation and of third-party dependencies: per-kernel
 * event timing, and the dense-GEMM formulation of the layer as a comparison baseline (this library
 * links rocBLAS; the layer library does not).  Nothing here is on the product path.
 * Pointer, layout, stream and status conventions are those of kan.h.
 */
#ifndef KAN_BENCH_H
#define KAN_BENCH_H

#include "kan.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing.  kan_profile_before / kan_profile_after have the signature of kan_launch_hook:
   install them with kan_set_launch_observer(kan_profile_before, kan_profile_after) and every kernel
   the layer library launches is bracketed by a pair of HIP events on its launch stream while
   recording is on (at most 8192 launches are recorded, later ones run untimed; the events are this
   library's state and are released by the next kan_profile_enable(1)).  kan_profile_enable(1)
   clears earlier records and starts recording, kan_profile_enable(0) stops it.  kan_profile_read
   waits for the recorded events, fills up to `capacity` entries (one per kernel family, `name` is
   a static string) and returns the number of families seen, or a negative kan_status.
   Not thread-safe; meant for one benchmarking thread. */
typedef struct kan_kernel_time {
    const char *name;
    double total_ms;
    int64_t launches;
} kan_kernel_time;
void kan_profile_before(const char *family, void *stream);
void kan_profile_after(const char *family, void *stream);
int kan_profile_enable(int on);
int kan_profile_read(kan_kernel_time *out, int capacity);

/* Comparison baseline: the forward pass written as one dense GEMM y = Phi * C over all G + k basis
   functions per input (the O(G) formulation of table "Complexity", row "Torch KAN"), with Phi
   materialised in the workspace and the contraction done by rocBLAS.  Degrees 1..3.  Creates a
   rocBLAS handle on first use (which allocates) and keeps it for the life of the process. */
size_t kan_dense_baseline_workspace_bytes(const kan_layer_desc *desc, int64_t B);
int kan_dense_baseline_forward(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                               const float *w_s, const float *w_b, float *y, void *ws, size_t ws_bytes,
                               void *stream);
/* The dense backward pass of the same baseline: gPhi = gy * C^T and gC = Phi^T * gy by rocBLAS,
   dL/dx as the row-wise product of gPhi with dPhi/dx.  Same outputs and conventions as kan_backward. */
size_t kan_dense_baseline_backward_workspace_bytes(const kan_layer_desc *desc, int64_t B);
int kan_dense_baseline_backward(const kan_layer_desc *desc, int64_t B, const float *x, const float *coef,
                                const float *w_s, const float *w_b, const float *gy, float *gx, float *gcoef,
                                float *gw_s, float *gw_b, void *ws, size_t ws_bytes, void *stream);

/* Instruction-rate ceilings of a compute unit (fp32 multiply-add, LDS reads / writes / atomic adds, the
   4x4x1 fp32 matrix-core instruction), the yardsticks the layer kernels' counters are read against.
   kan_bench_ceiling runs microbenchmark number `index` (0 .. kan_bench_ceiling_count() - 1) with one
   workgroup of threads_per_cu (256, 512 or 1024) threads on each of 256 CUs for `iters` iterations on the
   default stream, synchronises, and returns its name, the unit it counts ("FMA" or "B" for LDS bytes),
   units per CU per second and the kernel time.  Allocates and frees a small device buffer. */
int kan_bench_ceiling_count(void);
int kan_bench_ceiling(int index, int threads_per_cu, int iters, const char **name, const char **unit,
                      double *per_cu_per_second, double *ms);

#ifdef __cplusplus
}
#endif
#endif /* KAN_BENCH_H */
