/*
 * CPU oracle for the B-spline KAN layer (forward and backward).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  It shares no code with the HIP path, and
 * nothing in the product may call it: only the tests, the smoke check and
 * the benchmark's cpu_baseline leg do.
 *
 * All arithmetic is fp64.  The only fp32 step is the interval index, which
 * the paper defines as floor((x - t_0)/h) (Algorithm section, text after
 * Eq. "matrixform") without fixing a precision; it is taken here as the
 * fp32 expression floorf((x - a) * inv_h) with separate IEEE subtract and
 * multiply, because the integer result has to be reproducible bit for bit.
 *
 * Two evaluators are provided on purpose:
 *   okan_forward_dense  - the definition: every one of the G+k basis
 *                         functions by the Cox-de Boor recursion on the
 *                         extended knot vector (Eqs. "kanspline",
 *                         "coxdeboor", "activation", "kanphi").
 *   okan_forward        - the local form: only the k+1 non-zero basis
 *                         values of the cell that holds x (Eq. "matrixform").
 * The local one reaches exactly the dense result (it only skips zero terms);
 * the tests pin each against the other, against the printed cubic basis
 * matrix and against a library B-spline routine.
 *
 * Grid convention (pinned by the workloads: "G = 200, k = 3 -> 203
 * coefficients"): G cells on [a, a + G*h), k extra knots on each side,
 * G + 2k + 1 knots tau_p = a + (p - k) h, G + k coefficients per edge.
 * h is DEFINED as 1/inv_h with inv_h the fp32 number the caller passes, so
 * that the index rule and the polynomial pieces talk about the same grid.
 *
 * Layouts (row-major):  x[B][n_in]  y,gy[B][n_out]  gx[B][n_in]
 *   coef,gcoef[n_in][G+k][n_out]   w_s,w_b,gw_s,gw_b[n_in][n_out]
 *
 * base_act: 0 = no base term, 1 = SiLU  b(x) = x / (1 + exp(-x)).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define OKAN_MAX_K 8

int okan_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Thread count of the loops below (timing aid of the benchmark's cpu_baseline leg; no effect on any result:
   every output element is computed by one thread in a fixed order). */
void okan_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- base function ---------------------------------------------------- */

double okan_silu(double x) { return x / (1.0 + exp(-x)); }

double okan_silu_grad(double x)
{
    double s = 1.0 / (1.0 + exp(-x));
    return s * (1.0 + x * (1.0 - s));
}

/* ---- interval index (Algorithm section, i = floor((x - t_0)/h)) -------- */

/* fp32 rule.  volatile stops the compiler from fusing the two roundings. */
int32_t okan_interval_index_f32(float x, float a, float inv_h)
{
    volatile float d = x - a;
    volatile float t = d * inv_h;
    float f = floorf(t);
    /* keep the cast defined for huge |t|; anything this far out is outside
       every extended grid anyway */
    if (!(f > -1073741824.0f)) return -1073741824;
    if (!(f < 1073741824.0f)) return 1073741824;
    return (int32_t)f;
}

void okan_interval_index_batch(int64_t n, const float *x, float a, float inv_h,
                               int32_t *idx)
{
    for (int64_t p = 0; p < n; ++p) idx[p] = okan_interval_index_f32(x[p], a, inv_h);
}

/* index used by the evaluators: fp32 rule on the rounded input, or the same
   formula in fp64 (used by the finite-difference tests, where x moves by
   less than an fp32 ulp) */
static int32_t cell_of(double x, double a, float inv_h, int idx_fp32)
{
    if (idx_fp32) return okan_interval_index_f32((float)x, (float)a, inv_h);
    double f = floor((x - a) * (double)inv_h);
    if (!(f > -1073741824.0)) return -1073741824;
    if (!(f < 1073741824.0)) return 1073741824;
    return (int32_t)f;
}

/* ---- dense basis: Cox-de Boor on the whole extended knot vector -------- */

/* out[m] = B_{m,k}(x), m = 0..G+k-1.  If dout != NULL also d/dx B_{m,k}(x),
   from the textbook derivative  k/(tau_{m+k}-tau_m) B_{m,k-1}
   - k/(tau_{m+k+1}-tau_{m+1}) B_{m+1,k-1}. */
void okan_dense_basis(int G, int k, double a, float inv_h, double x,
                      double *out, double *dout)
{
    const double h = 1.0 / (double)inv_h;
    const int nk = G + 2 * k + 1;                 /* number of knots */
    double *tau = (double *)malloc(sizeof(double) * (size_t)nk);
    double *Bd = (double *)malloc(sizeof(double) * (size_t)nk);
    double *Bprev = (double *)malloc(sizeof(double) * (size_t)nk);
    for (int p = 0; p < nk; ++p) tau[p] = a + (double)(p - k) * h;

    /* degree 0: indicator of the half-open cell [tau_m, tau_{m+1}) */
    for (int m = 0; m < nk - 1; ++m) Bd[m] = (tau[m] <= x && x < tau[m + 1]) ? 1.0 : 0.0;

    for (int d = 1; d <= k; ++d) {
        memcpy(Bprev, Bd, sizeof(double) * (size_t)(nk - d));
        for (int m = 0; m < nk - 1 - d; ++m) {
            double left = (x - tau[m]) / (tau[m + d] - tau[m]);
            double right = (tau[m + d + 1] - x) / (tau[m + d + 1] - tau[m + 1]);
            Bd[m] = left * Bprev[m] + right * Bprev[m + 1];
        }
        if (d == k && dout) {
            for (int m = 0; m < G + k; ++m)
                dout[m] = (double)k / (tau[m + k] - tau[m]) * Bprev[m]
                        - (double)k / (tau[m + k + 1] - tau[m + 1]) * Bprev[m + 1];
        }
    }
    if (k == 0 && dout) for (int m = 0; m < G; ++m) dout[m] = 0.0;
    for (int m = 0; m < G + k; ++m) out[m] = Bd[m];
    free(tau); free(Bd); free(Bprev);
}

/* ---- local basis: the k+1 values that are non-zero on one cell --------- */

/* N[s] = B_{c-k+s,k} at local coordinate u in the cell c, s = 0..k, by the
   Cox-de Boor recursion specialised to uniform knots:
     N^0_0 = 1
     N^d_s = (u + d - s)/d * N^{d-1}_{s-1} + (s + 1 - u)/d * N^{d-1}_s .
   N[0] multiplies the OLDEST coefficient of the window and equals
   (1-u)^k / k!  (first column of the printed cubic basis matrix).
   Nlow (optional, k entries) receives the degree k-1 values, from which
   d N^k_s / dx = (N^{k-1}_{s-1} - N^{k-1}_s) / h. */
void okan_local_basis(int k, double u, double *N, double *Nlow)
{
    double cur[OKAN_MAX_K + 2], prev[OKAN_MAX_K + 2];
    cur[0] = 1.0;
    if (k == 0) { N[0] = 1.0; return; }
    for (int d = 1; d <= k; ++d) {
        for (int s = 0; s < d; ++s) prev[s] = cur[s];
        if (d == k && Nlow) for (int s = 0; s < k; ++s) Nlow[s] = prev[s];
        for (int s = 0; s <= d; ++s) {
            double lo = (s >= 1) ? prev[s - 1] : 0.0;
            double hi = (s <= d - 1) ? prev[s] : 0.0;
            cur[s] = (u + (double)(d - s)) / (double)d * lo
                   + ((double)(s + 1) - u) / (double)d * hi;
        }
    }
    for (int s = 0; s <= k; ++s) N[s] = cur[s];
}

/* ---- forward: the definition (dense) ----------------------------------- */

/* y[b][j] = sum_i ( w_s[i][j] * sum_m coef[i][m][j] B_{m,k}(x[b][i])
 *                 + w_b[i][j] * b(x[b][i]) )                               */
int okan_forward_dense(int n_in, int n_out, int G, int k, double a, float inv_h,
                       int base_act, int64_t B, const double *x,
                       const double *coef, const double *w_s, const double *w_b,
                       double *y)
{
    if (k < 0 || k > OKAN_MAX_K || G <= 0 || n_in <= 0 || n_out <= 0) return -1;
    const int M = G + k;
#pragma omp parallel
    {
        double *bas = (double *)malloc(sizeof(double) * (size_t)M);
#pragma omp for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            double *yb = y + b * n_out;
            for (int j = 0; j < n_out; ++j) yb[j] = 0.0;
            for (int i = 0; i < n_in; ++i) {
                double xv = x[b * n_in + i];
                okan_dense_basis(G, k, a, inv_h, xv, bas, NULL);
                double base = (base_act == 1) ? okan_silu(xv) : 0.0;
                for (int j = 0; j < n_out; ++j) {
                    double sp = 0.0;
                    for (int m = 0; m < M; ++m)
                        sp += coef[((size_t)i * M + m) * n_out + j] * bas[m];
                    double v = w_s[(size_t)i * n_out + j] * sp;
                    if (base_act == 1) v += w_b[(size_t)i * n_out + j] * base;
                    yb[j] += v;
                }
            }
        }
        free(bas);
    }
    return 0;
}

/* ---- forward: local form ------------------------------------------------ */

/* One (sample, input) pair: cell index, the K window weights and their
   x-derivatives.  Returns 0 if x lies outside the extended grid (then every
   basis function is zero there). */
static int pair_setup(double xv, int G, int k, double a, float inv_h, int idx_fp32,
                      int32_t *idx_out, double *N, double *dN)
{
    int32_t idx = cell_of(xv, a, inv_h, idx_fp32);
    *idx_out = idx;
    if (idx < -k || idx >= G + k) return 0;
    double u = (xv - a) * (double)inv_h - (double)idx;
    double low[OKAN_MAX_K + 1];
    okan_local_basis(k, u, N, low);
    if (dN) {
        for (int s = 0; s <= k; ++s) {
            double lo = (s >= 1) ? low[s - 1] : 0.0;
            double hi = (s <= k - 1) ? low[s] : 0.0;
            dN[s] = (k == 0) ? 0.0 : (lo - hi) * (double)inv_h;
        }
    }
    return 1;
}

int okan_forward(int n_in, int n_out, int G, int k, double a, float inv_h,
                 int base_act, int idx_fp32, int64_t B, const double *x,
                 const double *coef, const double *w_s, const double *w_b,
                 double *y)
{
    if (k < 0 || k > OKAN_MAX_K || G <= 0 || n_in <= 0 || n_out <= 0) return -1;
    const int M = G + k;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        double *yb = y + b * n_out;
        for (int j = 0; j < n_out; ++j) yb[j] = 0.0;
        for (int i = 0; i < n_in; ++i) {
            double xv = x[b * n_in + i];
            double N[OKAN_MAX_K + 1];
            int32_t idx;
            int inside = pair_setup(xv, G, k, a, inv_h, idx_fp32, &idx, N, NULL);
            double base = (base_act == 1) ? okan_silu(xv) : 0.0;
            for (int j = 0; j < n_out; ++j) {
                double sp = 0.0;
                if (inside) {
                    for (int s = 0; s <= k; ++s) {
                        int m = idx + s;           /* coefficient index */
                        if (m < 0 || m >= M) continue;   /* padding cell */
                        sp += coef[((size_t)i * M + m) * n_out + j] * N[s];
                    }
                }
                double v = w_s[(size_t)i * n_out + j] * sp;
                if (base_act == 1) v += w_b[(size_t)i * n_out + j] * base;
                yb[j] += v;
            }
        }
    }
    return 0;
}

/* ---- backward ----------------------------------------------------------- */

/* Gradients of L given gy = dL/dy (derived from Eqs. "activation", "kanphi",
 * "kanspline"; the paper states no backward formulas):
 *  gx[b][i]      = sum_j gy[b][j] ( w_s[i][j] sum_s coef[i][idx+s][j] N'_s
 *                                   + w_b[i][j] b'(x[b][i]) )
 *  gcoef[i][m][j]= w_s[i][j] sum_b gy[b][j] N_{m-idx(b,i)}(u(b,i))
 *  gw_s[i][j]    = sum_b gy[b][j] spline_ij(x[b][i])
 *  gw_b[i][j]    = sum_b gy[b][j] b(x[b][i])
 * Any output pointer may be NULL.  Outputs are overwritten.               */
int okan_backward(int n_in, int n_out, int G, int k, double a, float inv_h,
                  int base_act, int idx_fp32, int64_t B, const double *x,
                  const double *coef, const double *w_s, const double *w_b,
                  const double *gy, double *gx, double *gcoef, double *gw_s,
                  double *gw_b)
{
    if (k < 0 || k > OKAN_MAX_K || G <= 0 || n_in <= 0 || n_out <= 0) return -1;
    const int M = G + k;

    if (gx) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            for (int i = 0; i < n_in; ++i) {
                double xv = x[b * n_in + i];
                double N[OKAN_MAX_K + 1], dN[OKAN_MAX_K + 1];
                int32_t idx;
                int inside = pair_setup(xv, G, k, a, inv_h, idx_fp32, &idx, N, dN);
                double dbase = (base_act == 1) ? okan_silu_grad(xv) : 0.0;
                double acc = 0.0;
                for (int j = 0; j < n_out; ++j) {
                    double dsp = 0.0;
                    if (inside) {
                        for (int s = 0; s <= k; ++s) {
                            int m = idx + s;
                            if (m < 0 || m >= M) continue;
                            dsp += coef[((size_t)i * M + m) * n_out + j] * dN[s];
                        }
                    }
                    double v = w_s[(size_t)i * n_out + j] * dsp;
                    if (base_act == 1) v += w_b[(size_t)i * n_out + j] * dbase;
                    acc += gy[b * n_out + j] * v;
                }
                gx[b * n_in + i] = acc;
            }
        }
    }

    if (gcoef || gw_s || gw_b) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < n_in; ++i) {
            if (gcoef) memset(gcoef + (size_t)i * M * n_out, 0, sizeof(double) * (size_t)M * n_out);
            if (gw_s) memset(gw_s + (size_t)i * n_out, 0, sizeof(double) * (size_t)n_out);
            if (gw_b) memset(gw_b + (size_t)i * n_out, 0, sizeof(double) * (size_t)n_out);
            for (int64_t b = 0; b < B; ++b) {
                double xv = x[b * n_in + i];
                double N[OKAN_MAX_K + 1];
                int32_t idx;
                int inside = pair_setup(xv, G, k, a, inv_h, idx_fp32, &idx, N, NULL);
                double base = (base_act == 1) ? okan_silu(xv) : 0.0;
                for (int j = 0; j < n_out; ++j) {
                    double g = gy[b * n_out + j];
                    if (inside) {
                        double sp = 0.0;
                        for (int s = 0; s <= k; ++s) {
                            int m = idx + s;
                            if (m < 0 || m >= M) continue;
                            size_t at = ((size_t)i * M + m) * n_out + j;
                            sp += coef[at] * N[s];
                            if (gcoef) gcoef[at] += w_s[(size_t)i * n_out + j] * g * N[s];
                        }
                        if (gw_s) gw_s[(size_t)i * n_out + j] += g * sp;
                    }
                    if (gw_b && base_act == 1) gw_b[(size_t)i * n_out + j] += g * base;
                }
            }
        }
    }
    return 0;
}
