/*
 * CPU oracle for the UKAN layer: B-spline layer on the unbounded uniform
 * grid t_j = j*h whose coefficients come from a coefficient-generator (CG)
 * MLP (Algorithm section, second half; appendix "UKAN mapping to KAN").
 *
 * TEST INFRASTRUCTURE ONLY: plain fp64 reference for the tests, the smoke
 * check and the benchmark's cpu_baseline leg.  No code is shared with the
 * HIP path and nothing in the product may call this file.
 *
 * What is computed, in the paper's notation (K = k+1):
 *   cell   i(x) = floor(x / h)                     (fp32 rule, see below)
 *   group  g    = floor(i / K)   (floor division, also for negative i)
 *   offset r    = i mod K        (in 0..K-1)
 *   C_g         = CG(feature, g) in R^K per edge
 *   window      = entries r .. r+K-1 of [C_{g-1} ; C_g]
 *   spline(x)   = sum_s window[s] * N_s(u),  u = x/h - i(x)
 *   y[b][j]     = sum_i ( spline_ij(x[b][i]) + w_b[i][j] silu(x[b][i]) )
 *
 * Readings where the paper is silent (all "parity unpinned" by the paper,
 * both sides only have to agree):
 *   - CG(i,g) = W2^T silu(W1^T [E[i] ; PE(g)] + b1) + b2, a two-layer MLP
 *     with SiLU after the first layer; the output has K*n_out entries
 *     ordered [q][j]; the coefficient of edge (i,j) is
 *     scale[i][j] * CG(i,g)[q*n_out + j]   ("scaled by another learnable
 *     parameter", regression experiment).
 *   - PE(g)[2t] = sin(g / 10000^(2t/d_pe)), PE(g)[2t+1] = cos(same), g
 *     signed; evaluated in fp64 and rounded to fp32 (it is an fp32 input of
 *     the CG on the device).
 *   - cell index: floorf(x * inv_h) in fp32, inv_h = 1/h passed as fp32;
 *     h is defined as 1/inv_h.
 *
 * Layouts (row-major): x[B][n_in], y,gy[B][n_out], E[n_in][d_feat],
 *   W1[d_feat+d_pe][d_hid] (embedding rows first), b1[d_hid],
 *   W2[d_hid][K*n_out], b2[K*n_out], scale,w_b[n_in][n_out].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* from kan_oracle.c */
double okan_silu(double x);
double okan_silu_grad(double x);
int32_t okan_interval_index_f32(float x, float a, float inv_h);
void okan_local_basis(int k, double u, double *N, double *Nlow);

#define OUKAN_MAX_K 8
#define OUKAN_MAX_SPAN (1 << 22)     /* cells per input the table may cover */

/* ---- integer bookkeeping (text around the group-index equation) -------- */

/* floor division and non-negative remainder; C's / and % truncate */
void oukan_group_of_cell(int32_t cell, int K, int32_t *g, int32_t *r)
{
    int32_t q = cell / K, m = cell % K;
    if (m < 0) { m += K; q -= 1; }
    *g = q; *r = m;
}

void oukan_group_index_batch(int64_t n, const float *x, float inv_h, int K,
                             int32_t *cell, int32_t *g, int32_t *r)
{
    for (int64_t p = 0; p < n; ++p) {
        int32_t c = okan_interval_index_f32(x[p], 0.0f, inv_h);
        cell[p] = c;
        oukan_group_of_cell(c, K, &g[p], &r[p]);
    }
}

static int32_t cell_of(double x, float inv_h, int idx_fp32)
{
    if (idx_fp32) return okan_interval_index_f32((float)x, 0.0f, inv_h);
    double f = floor(x * (double)inv_h);
    if (!(f > -1073741824.0)) return -1073741824;
    if (!(f < 1073741824.0)) return 1073741824;
    return (int32_t)f;
}

/* ---- sinusoidal encoding of the group index ---------------------------- */

void oukan_pe(int32_t g, int d_pe, double *out)
{
    for (int c = 0; c < d_pe; ++c) {
        int t = c / 2;
        double freq = pow(10000.0, -2.0 * (double)t / (double)d_pe);
        double ang = (double)g * freq;
        double v = (c % 2 == 0) ? sin(ang) : cos(ang);
        out[c] = (double)(float)v;
    }
}

/* ---- coefficient generator --------------------------------------------- */

typedef struct {
    int n_in, n_out, k, d_pe, d_feat, d_hid;
    const double *E, *W1, *b1, *W2, *b2;
} cg_net;

/* out[K*n_out]; optionally keeps z (d_feat+d_pe), pre-activation and hidden */
static void cg_eval(const cg_net *n, int i, int32_t g, double *out,
                    double *z_keep, double *pre_keep, double *hid_keep)
{
    const int dz = n->d_feat + n->d_pe, K = n->k + 1, no = K * n->n_out;
    double *z = (double *)malloc(sizeof(double) * (size_t)dz);
    double *hid = (double *)malloc(sizeof(double) * (size_t)n->d_hid);
    for (int f = 0; f < n->d_feat; ++f) z[f] = n->E[(size_t)i * n->d_feat + f];
    oukan_pe(g, n->d_pe, z + n->d_feat);
    for (int c = 0; c < n->d_hid; ++c) {
        double s = n->b1[c];
        for (int p = 0; p < dz; ++p) s += z[p] * n->W1[(size_t)p * n->d_hid + c];
        if (pre_keep) pre_keep[c] = s;
        hid[c] = okan_silu(s);
    }
    for (int o = 0; o < no; ++o) {
        double s = n->b2[o];
        for (int c = 0; c < n->d_hid; ++c) s += hid[c] * n->W2[(size_t)c * no + o];
        out[o] = s;
    }
    if (z_keep) memcpy(z_keep, z, sizeof(double) * (size_t)dz);
    if (hid_keep) memcpy(hid_keep, hid, sizeof(double) * (size_t)n->d_hid);
    free(z); free(hid);
}

/* CG output for one (feature, group): exported for the tests */
void oukan_cg(int n_in, int n_out, int k, int d_pe, int d_feat, int d_hid,
              const double *E, const double *W1, const double *b1,
              const double *W2, const double *b2, int i, int32_t g, double *out)
{
    cg_net n = { n_in, n_out, k, d_pe, d_feat, d_hid, E, W1, b1, W2, b2 };
    cg_eval(&n, i, g, out, NULL, NULL, NULL);
}

/* ---- forward, evaluated per sample with no memoisation ------------------ */
/* The literal reading: for every (sample, input) call the CG for groups g-1
   and g, concatenate, slide the window.  Only for tiny inputs. */
int oukan_forward_direct(int n_in, int n_out, int k, float inv_h, int d_pe,
                         int d_feat, int d_hid, int base_act, int idx_fp32,
                         int64_t B, const double *x, const double *E,
                         const double *W1, const double *b1, const double *W2,
                         const double *b2, const double *scale,
                         const double *w_b, double *y)
{
    if (k < 0 || k > OUKAN_MAX_K) return -1;
    const int K = k + 1, no = K * n_out;
    cg_net n = { n_in, n_out, k, d_pe, d_feat, d_hid, E, W1, b1, W2, b2 };
    double *pair = (double *)malloc(sizeof(double) * 2 * (size_t)no);
    for (int64_t b = 0; b < B; ++b) {
        for (int j = 0; j < n_out; ++j) y[b * n_out + j] = 0.0;
        for (int i = 0; i < n_in; ++i) {
            double xv = x[b * n_in + i];
            int32_t cell = cell_of(xv, inv_h, idx_fp32), g, r;
            oukan_group_of_cell(cell, K, &g, &r);
            double u = xv * (double)inv_h - (double)cell;
            double N[OUKAN_MAX_K + 1];
            okan_local_basis(k, u, N, NULL);
            cg_eval(&n, i, g - 1, pair, NULL, NULL, NULL);        /* C_{g-1} */
            cg_eval(&n, i, g, pair + no, NULL, NULL, NULL);       /* C_g     */
            double base = (base_act == 1) ? okan_silu(xv) : 0.0;
            for (int j = 0; j < n_out; ++j) {
                double sp = 0.0;
                for (int s = 0; s < K; ++s) {
                    int pos = r + s;                  /* entry of [C_{g-1};C_g] */
                    double c = pair[(size_t)pos * n_out + j];
                    sp += c * N[s];
                }
                double v = scale[(size_t)i * n_out + j] * sp;
                if (base_act == 1) v += w_b[(size_t)i * n_out + j] * base;
                y[b * n_out + j] += v;
            }
        }
    }
    free(pair);
    return 0;
}

/* ---- memoised tables ------------------------------------------------------ */
/* The CG is a pure function of (feature, group), so its outputs are kept in
   one table per input covering the groups the batch touches.  Global
   coefficient index m = g*K + q; the cell `c` uses m = c-K .. c-1, which is
   entries r..r+K-1 of [C_{g-1};C_g] because (g-1)K + r + s = c - K + s. */
typedef struct {
    int32_t g_lo;      /* first group held */
    int32_t n_g;       /* number of groups held */
    double *out;       /* [n_g][K*n_out]  raw CG outputs                  */
    double *z, *pre, *hid;   /* [n_g][..] kept for the backward pass       */
} cg_table;

static int build_tables(const cg_net *n, float inv_h, int idx_fp32, int64_t B,
                        const double *x, cg_table *tab, int keep)
{
    const int K = n->k + 1, no = K * n->n_out, dz = n->d_feat + n->d_pe;
    for (int i = 0; i < n->n_in; ++i) {
        int32_t cmin = 0, cmax = 0;
        for (int64_t b = 0; b < B; ++b) {
            int32_t c = cell_of(x[b * n->n_in + i], inv_h, idx_fp32);
            if (b == 0 || c < cmin) cmin = c;
            if (b == 0 || c > cmax) cmax = c;
        }
        if ((int64_t)cmax - (int64_t)cmin > OUKAN_MAX_SPAN) return -2;
        int32_t gmin, gmax, r;
        oukan_group_of_cell(cmin, K, &gmin, &r);
        oukan_group_of_cell(cmax, K, &gmax, &r);
        tab[i].g_lo = gmin - 1;
        tab[i].n_g = gmax - gmin + 2;
        tab[i].out = (double *)malloc(sizeof(double) * (size_t)tab[i].n_g * no);
        tab[i].z = tab[i].pre = tab[i].hid = NULL;
        if (keep) {
            tab[i].z = (double *)malloc(sizeof(double) * (size_t)tab[i].n_g * dz);
            tab[i].pre = (double *)malloc(sizeof(double) * (size_t)tab[i].n_g * n->d_hid);
            tab[i].hid = (double *)malloc(sizeof(double) * (size_t)tab[i].n_g * n->d_hid);
        }
    }
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < n->n_in; ++i) {
        for (int32_t t = 0; t < tab[i].n_g; ++t)
            cg_eval(n, i, tab[i].g_lo + t, tab[i].out + (size_t)t * no,
                    keep ? tab[i].z + (size_t)t * dz : NULL,
                    keep ? tab[i].pre + (size_t)t * n->d_hid : NULL,
                    keep ? tab[i].hid + (size_t)t * n->d_hid : NULL);
    }
    return 0;
}

static void free_tables(cg_table *tab, int n_in)
{
    for (int i = 0; i < n_in; ++i) { free(tab[i].out); free(tab[i].z); free(tab[i].pre); free(tab[i].hid); }
    free(tab);
}

/* address of raw CG output for global coefficient index m of input i */
static inline size_t tab_at(const cg_table *t, int K, int n_out, int64_t m, int j)
{
    int64_t rel = m - (int64_t)t->g_lo * K;        /* >= 0 by construction */
    return (size_t)rel * n_out + j;                /* [g][q][j] is contiguous in m */
}

int oukan_forward(int n_in, int n_out, int k, float inv_h, int d_pe, int d_feat,
                  int d_hid, int base_act, int idx_fp32, int64_t B,
                  const double *x, const double *E, const double *W1,
                  const double *b1, const double *W2, const double *b2,
                  const double *scale, const double *w_b, double *y)
{
    if (k < 0 || k > OUKAN_MAX_K) return -1;
    const int K = k + 1;
    cg_net n = { n_in, n_out, k, d_pe, d_feat, d_hid, E, W1, b1, W2, b2 };
    cg_table *tab = (cg_table *)calloc((size_t)n_in, sizeof(cg_table));
    int rc = build_tables(&n, inv_h, idx_fp32, B, x, tab, 0);
    if (rc) { free(tab); return rc; }
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int j = 0; j < n_out; ++j) y[b * n_out + j] = 0.0;
        for (int i = 0; i < n_in; ++i) {
            double xv = x[b * n_in + i];
            int32_t cell = cell_of(xv, inv_h, idx_fp32);
            double u = xv * (double)inv_h - (double)cell;
            double N[OUKAN_MAX_K + 1];
            okan_local_basis(k, u, N, NULL);
            double base = (base_act == 1) ? okan_silu(xv) : 0.0;
            for (int j = 0; j < n_out; ++j) {
                double sp = 0.0;
                for (int s = 0; s < K; ++s)
                    sp += tab[i].out[tab_at(&tab[i], K, n_out, (int64_t)cell - K + s, j)] * N[s];
                double v = scale[(size_t)i * n_out + j] * sp;
                if (base_act == 1) v += w_b[(size_t)i * n_out + j] * base;
                y[b * n_out + j] += v;
            }
        }
    }
    free_tables(tab, n_in);
    return 0;
}

/* Materialise a finite KAN from the UKAN on cells c_lo..c_hi of every input
   (appendix "UKAN mapping to KAN"): coef[i][m][j], m = 0..(c_hi-c_lo+1)+k-1,
   is the global coefficient c_lo - K + m, scale applied.  The matching KAN
   has G = c_hi - c_lo + 1, grid start a = c_lo*h, w_s = 1. */
int oukan_materialize(int n_in, int n_out, int k, int d_pe, int d_feat, int d_hid,
                      const double *E, const double *W1, const double *b1,
                      const double *W2, const double *b2, const double *scale,
                      int32_t c_lo, int32_t c_hi, double *coef)
{
    const int K = k + 1, no = K * n_out;
    const int M = (c_hi - c_lo + 1) + k;
    cg_net n = { n_in, n_out, k, d_pe, d_feat, d_hid, E, W1, b1, W2, b2 };
    double *out = (double *)malloc(sizeof(double) * (size_t)no);
    for (int i = 0; i < n_in; ++i) {
        for (int m = 0; m < M; ++m) {
            int32_t glob = c_lo - K + m, g, q;
            oukan_group_of_cell(glob, K, &g, &q);
            cg_eval(&n, i, g, out, NULL, NULL, NULL);
            for (int j = 0; j < n_out; ++j)
                coef[((size_t)i * M + m) * n_out + j] =
                    scale[(size_t)i * n_out + j] * out[(size_t)q * n_out + j];
        }
    }
    free(out);
    return 0;
}

/* ---- backward ------------------------------------------------------------ */
/* Chain rule through  y -> window coefficients -> scale, CG output -> W2,b2,
 * hidden -> SiLU -> W1,b1 -> E.  The group index is piecewise constant in x,
 * so dL/dx flows through u only.  Any output pointer may be NULL; outputs are
 * overwritten.                                                               */
int oukan_backward(int n_in, int n_out, int k, float inv_h, int d_pe, int d_feat,
                   int d_hid, int base_act, int idx_fp32, int64_t B,
                   const double *x, const double *E, const double *W1,
                   const double *b1, const double *W2, const double *b2,
                   const double *scale, const double *w_b, const double *gy,
                   double *gx, double *gE, double *gW1, double *gb1,
                   double *gW2, double *gb2, double *gscale, double *gw_b)
{
    if (k < 0 || k > OUKAN_MAX_K) return -1;
    const int K = k + 1, no = K * n_out, dz = d_feat + d_pe;
    cg_net n = { n_in, n_out, k, d_pe, d_feat, d_hid, E, W1, b1, W2, b2 };
    cg_table *tab = (cg_table *)calloc((size_t)n_in, sizeof(cg_table));
    int rc = build_tables(&n, inv_h, idx_fp32, B, x, tab, 1);
    if (rc) { free(tab); return rc; }

    if (gx) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            for (int i = 0; i < n_in; ++i) {
                double xv = x[b * n_in + i];
                int32_t cell = cell_of(xv, inv_h, idx_fp32);
                double u = xv * (double)inv_h - (double)cell;
                double N[OUKAN_MAX_K + 1], low[OUKAN_MAX_K + 1], dN[OUKAN_MAX_K + 1];
                okan_local_basis(k, u, N, low);
                for (int s = 0; s < K; ++s) {
                    double lo = (s >= 1) ? low[s - 1] : 0.0;
                    double hi = (s <= k - 1) ? low[s] : 0.0;
                    dN[s] = (k == 0) ? 0.0 : (lo - hi) * (double)inv_h;
                }
                double dbase = (base_act == 1) ? okan_silu_grad(xv) : 0.0;
                double acc = 0.0;
                for (int j = 0; j < n_out; ++j) {
                    double dsp = 0.0;
                    for (int s = 0; s < K; ++s)
                        dsp += tab[i].out[tab_at(&tab[i], K, n_out, (int64_t)cell - K + s, j)] * dN[s];
                    double v = scale[(size_t)i * n_out + j] * dsp;
                    if (base_act == 1) v += w_b[(size_t)i * n_out + j] * dbase;
                    acc += gy[b * n_out + j] * v;
                }
                gx[b * n_in + i] = acc;
            }
        }
    }

    /* gradient w.r.t. the raw CG outputs, per input: gout[i][g][q][j] */
    double **gout = (double **)calloc((size_t)n_in, sizeof(double *));
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < n_in; ++i) {
        gout[i] = (double *)calloc((size_t)tab[i].n_g * no, sizeof(double));
        if (gscale) memset(gscale + (size_t)i * n_out, 0, sizeof(double) * (size_t)n_out);
        if (gw_b) memset(gw_b + (size_t)i * n_out, 0, sizeof(double) * (size_t)n_out);
        for (int64_t b = 0; b < B; ++b) {
            double xv = x[b * n_in + i];
            int32_t cell = cell_of(xv, inv_h, idx_fp32);
            double u = xv * (double)inv_h - (double)cell;
            double N[OUKAN_MAX_K + 1];
            okan_local_basis(k, u, N, NULL);
            double base = (base_act == 1) ? okan_silu(xv) : 0.0;
            for (int j = 0; j < n_out; ++j) {
                double g = gy[b * n_out + j];
                for (int s = 0; s < K; ++s) {
                    size_t at = tab_at(&tab[i], K, n_out, (int64_t)cell - K + s, j);
                    /* coefficient = scale * out  */
                    gout[i][at] += g * N[s] * scale[(size_t)i * n_out + j];
                    if (gscale) gscale[(size_t)i * n_out + j] += g * N[s] * tab[i].out[at];
                }
                if (gw_b && base_act == 1) gw_b[(size_t)i * n_out + j] += g * base;
            }
        }
    }

    /* CG backward, serial over (input, group) so that the shared-parameter
       sums need no synchronisation */
    if (gW2) memset(gW2, 0, sizeof(double) * (size_t)d_hid * no);
    if (gb2) memset(gb2, 0, sizeof(double) * (size_t)no);
    if (gW1) memset(gW1, 0, sizeof(double) * (size_t)dz * d_hid);
    if (gb1) memset(gb1, 0, sizeof(double) * (size_t)d_hid);
    if (gE) memset(gE, 0, sizeof(double) * (size_t)n_in * d_feat);
    if (gW2 || gb2 || gW1 || gb1 || gE) {
        double *ghid = (double *)malloc(sizeof(double) * (size_t)d_hid);
        for (int i = 0; i < n_in; ++i) {
            for (int32_t t = 0; t < tab[i].n_g; ++t) {
                const double *go = gout[i] + (size_t)t * no;
                const double *hid = tab[i].hid + (size_t)t * d_hid;
                const double *pre = tab[i].pre + (size_t)t * d_hid;
                const double *z = tab[i].z + (size_t)t * dz;
                for (int c = 0; c < d_hid; ++c) {
                    double s = 0.0;
                    for (int o = 0; o < no; ++o) {
                        s += W2[(size_t)c * no + o] * go[o];
                        if (gW2) gW2[(size_t)c * no + o] += hid[c] * go[o];
                    }
                    ghid[c] = s * okan_silu_grad(pre[c]);      /* d/d pre-activation */
                }
                if (gb2) for (int o = 0; o < no; ++o) gb2[o] += go[o];
                for (int c = 0; c < d_hid; ++c) {
                    if (gb1) gb1[c] += ghid[c];
                    for (int p = 0; p < dz; ++p) {
                        if (gW1) gW1[(size_t)p * d_hid + c] += z[p] * ghid[c];
                        if (gE && p < d_feat) gE[(size_t)i * d_feat + p] += W1[(size_t)p * d_hid + c] * ghid[c];
                    }
                }
            }
        }
        free(ghid);
    }
    for (int i = 0; i < n_in; ++i) free(gout[i]);
    free(gout);
    free_tables(tab, n_in);
    return 0;
}
