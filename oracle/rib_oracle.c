/*
 * CPU oracle for RIB window attention.  TEST INFRASTRUCTURE ONLY: this file is
 * the slow, plain definition that the GPU library is checked against.  It is
 * never part of the product path, shares no code with the HIP kernels, and may
 * only be called from the tests, the smoke check and the benchmark's
 * cpu_baseline leg.
 *
 * What it computes (paper Sec. 2.2 "window-based self-attention", Sec. 3.1
 * Eq. 5 "concat + scale" and Eq. 6 "score identity"):
 *
 *   for every image b, every MxM window (wy,wx) and every head hd, with the
 *   N = M*M tokens of the window numbered row-major n = iy*M + ix and living at
 *   grid position  g(n) = ((wy*M + iy + s) mod H, (wx*M + ix + s) mod W):
 *
 *     S[i][j] = scale_c * <q[g(i)], k[g(j)]>_head  +  scale_p * <f_q[hd,i], f_k[hd,j]>
 *     P[i][:] = softmax(S[i][:])            (Sec. 2.2: P = SoftMax(S))
 *     O[g(i)] = sum_j P[i][j] * v[g(j)]     (Sec. 2.2: O = P V)
 *     LSE[i]  = log sum_j exp(S[i][j])
 *
 *   The bias is the ADDITIVE form of Eq. 6 (content term + bias term); the
 *   concatenated form of Eq. 5 is deliberately not used here, so that a test can
 *   build it separately and pin the identity.
 *
 * Backward (the paper trains through the operator but does not print the
 * gradient; this is the chain rule applied to the three lines above, for a
 * given upstream gradient dO):
 *
 *     dV[g(j)] = sum_i P[i][j] dO[g(i)]
 *     dP[i][j] = <dO[g(i)], v[g(j)]>_head
 *     delta_i  = sum_j P[i][j] dP[i][j]
 *     dS[i][j] = P[i][j] (dP[i][j] - delta_i)
 *     dQ[g(i)] = scale_c sum_j dS[i][j] k[g(j)]
 *     dK[g(j)] = scale_c sum_i dS[i][j] q[g(i)]
 *     dF_q[hd,i] = scale_p sum_{b,window} sum_j dS[i][j] f_k[hd,j]
 *     dF_k[hd,j] = scale_p sum_{b,window} sum_i dS[i][j] f_q[hd,i]
 *   (f_q, f_k depend only on the window geometry, Sec. 3.1 last paragraph, so
 *   every window of every image shares them and their gradients are sums.)
 *
 * Precision: inputs are float (a bf16 workload passes bf16 values widened to
 * float, which is exact); every product, sum, exp and log is done in double.
 * One row of S is held at a time; there is no tiling, fusion or reordering.
 *
 * Layout: q,k,v,dO,O,dQ,dK,dV are channel-last grids [B][H][W][C], C = heads*d,
 * channel c = hd*d + t.  f_q,f_k,dF_q,dF_k are [heads][N][r].  LSE is
 * [B*nW][heads][N] with window index w = (b*(H/M) + wy)*(W/M) + wx.
 * A "unit" is one (window, head) pair, numbered u = w*heads + hd.
 *
 * Pins (tests/test_oracle_pins.py): brute force over global coordinates,
 * hand-computed two-token case, Eq. 6 identity, softmax invariants, M=1 special
 * case, library scaled-dot-product attention, finite differences, autograd of
 * the materialised form, window-permutation and shift invariants.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int B, H, W, heads, d, r, M, s;
    double scale_c, scale_p;
} geom_t;

static int64_t token_offset(const geom_t *g, int b, int wy, int wx, int n, int hd)
{
    int iy = n / g->M, ix = n % g->M;
    int y = (wy * g->M + iy + g->s) % g->H;
    int x = (wx * g->M + ix + g->s) % g->W;
    int64_t C = (int64_t)g->heads * g->d;
    return (((int64_t)b * g->H + y) * g->W + x) * C + (int64_t)hd * g->d;
}

static void unit_coords(const geom_t *g, int64_t u, int *b, int *wy, int *wx, int *hd)
{
    int nwx = g->W / g->M, nwy = g->H / g->M;
    *hd = (int)(u % g->heads);
    int64_t w = u / g->heads;
    *wx = (int)(w % nwx);
    *wy = (int)((w / nwx) % nwy);
    *b = (int)(w / ((int64_t)nwx * nwy));
}

/* Fill one row of logits S[i][0..N) and return its maximum. */
static double score_row(const geom_t *g, const float *q, const float *k,
                        const float *fq, const float *fk,
                        int b, int wy, int wx, int hd, int i, double *S)
{
    int N = g->M * g->M;
    const float *qi = q + token_offset(g, b, wy, wx, i, hd);
    const float *fqi = fq + ((int64_t)hd * N + i) * g->r;
    double mx = -INFINITY;
    for (int j = 0; j < N; ++j) {
        const float *kj = k + token_offset(g, b, wy, wx, j, hd);
        const float *fkj = fk + ((int64_t)hd * N + j) * g->r;
        double content = 0.0, bias = 0.0;
        for (int t = 0; t < g->d; ++t) content += (double)qi[t] * (double)kj[t];
        for (int t = 0; t < g->r; ++t) bias += (double)fqi[t] * (double)fkj[t];
        S[j] = g->scale_c * content + g->scale_p * bias;
        if (S[j] > mx) mx = S[j];
    }
    return mx;
}

/* Turn a row of logits into probabilities in place; returns log-sum-exp. */
static double softmax_row(int N, double mx, double *S)
{
    double sum = 0.0;
    for (int j = 0; j < N; ++j) { S[j] = exp(S[j] - mx); sum += S[j]; }
    for (int j = 0; j < N; ++j) S[j] /= sum;
    return mx + log(sum);
}

/* Forward for one unit: O_u is [N][d], lse_u is [N]. */
static void fwd_unit(const geom_t *g, const float *q, const float *k, const float *v,
                     const float *fq, const float *fk, int64_t u,
                     double *O_u, double *lse_u, double *row)
{
    int b, wy, wx, hd, N = g->M * g->M;
    unit_coords(g, u, &b, &wy, &wx, &hd);
    for (int i = 0; i < N; ++i) {
        double mx = score_row(g, q, k, fq, fk, b, wy, wx, hd, i, row);
        lse_u[i] = softmax_row(N, mx, row);
        double *Oi = O_u + (int64_t)i * g->d;
        for (int t = 0; t < g->d; ++t) Oi[t] = 0.0;
        for (int j = 0; j < N; ++j) {
            const float *vj = v + token_offset(g, b, wy, wx, j, hd);
            for (int t = 0; t < g->d; ++t) Oi[t] += row[j] * (double)vj[t];
        }
    }
}

/* Backward for one unit.  dq_u,dk_u,dv_u are [N][d]; dfq_u,dfk_u are [N][r];
 * all five are overwritten. */
static void bwd_unit(const geom_t *g, const float *q, const float *k, const float *v,
                     const float *fq, const float *fk, const float *dO, int64_t u,
                     double *dq_u, double *dk_u, double *dv_u,
                     double *dfq_u, double *dfk_u, double *P, double *dS)
{
    int b, wy, wx, hd, N = g->M * g->M, d = g->d, r = g->r;
    unit_coords(g, u, &b, &wy, &wx, &hd);
    memset(dq_u, 0, sizeof(double) * N * d);
    memset(dk_u, 0, sizeof(double) * N * d);
    memset(dv_u, 0, sizeof(double) * N * d);
    memset(dfq_u, 0, sizeof(double) * N * r);
    memset(dfk_u, 0, sizeof(double) * N * r);
    for (int i = 0; i < N; ++i) {
        double mx = score_row(g, q, k, fq, fk, b, wy, wx, hd, i, P);
        (void)softmax_row(N, mx, P);
        const float *dOi = dO + token_offset(g, b, wy, wx, i, hd);
        const float *qi = q + token_offset(g, b, wy, wx, i, hd);
        const float *fqi = fq + ((int64_t)hd * N + i) * r;
        double delta = 0.0;
        for (int j = 0; j < N; ++j) {
            const float *vj = v + token_offset(g, b, wy, wx, j, hd);
            double dP = 0.0;
            for (int t = 0; t < d; ++t) dP += (double)dOi[t] * (double)vj[t];
            dS[j] = dP;
            delta += P[j] * dP;
        }
        for (int j = 0; j < N; ++j) dS[j] = P[j] * (dS[j] - delta);
        for (int j = 0; j < N; ++j) {
            const float *kj = k + token_offset(g, b, wy, wx, j, hd);
            const float *fkj = fk + ((int64_t)hd * N + j) * r;
            for (int t = 0; t < d; ++t) {
                dv_u[(int64_t)j * d + t] += P[j] * (double)dOi[t];
                dq_u[(int64_t)i * d + t] += g->scale_c * dS[j] * (double)kj[t];
                dk_u[(int64_t)j * d + t] += g->scale_c * dS[j] * (double)qi[t];
            }
            for (int t = 0; t < r; ++t) {
                dfq_u[(int64_t)i * r + t] += g->scale_p * dS[j] * (double)fkj[t];
                dfk_u[(int64_t)j * r + t] += g->scale_p * dS[j] * (double)fqi[t];
            }
        }
    }
}

static int valid(const geom_t *g)
{
    return g->B > 0 && g->H > 0 && g->W > 0 && g->heads > 0 && g->d > 0 && g->r >= 0 &&
           g->M > 0 && g->H % g->M == 0 && g->W % g->M == 0 && g->s >= 0;
}

static geom_t make_geom(int B, int H, int W, int heads, int d, int r, int M, int s,
                        double scale_c, double scale_p)
{
    geom_t g = { B, H, W, heads, d, r, M, s, scale_c, scale_p };
    return g;
}

int rib_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Forward for the listed units only.  O_units is [n_units][N][d], lse_units is
 * [n_units][N].  Returns 0, or -1 on a bad shape / unit id. */
int rib_oracle_fwd_units(int B, int H, int W, int heads, int d, int r, int M, int s,
                         double scale_c, double scale_p,
                         const float *q, const float *k, const float *v,
                         const float *fq, const float *fk,
                         int64_t n_units, const int64_t *units,
                         double *O_units, double *lse_units)
{
    geom_t g = make_geom(B, H, W, heads, d, r, M, s, scale_c, scale_p);
    if (!valid(&g)) return -1;
    int N = M * M;
    int64_t total = (int64_t)B * (H / M) * (W / M) * heads;
    for (int64_t a = 0; a < n_units; ++a)
        if (units[a] < 0 || units[a] >= total) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * N);
        if (!row) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t a = 0; a < n_units; ++a)
                fwd_unit(&g, q, k, v, fq, fk, units[a],
                         O_units + a * N * (int64_t)d, lse_units + a * N, row);
        }
        free(row);
    }
    return fail ? -2 : 0;
}

/* Full forward.  O is the [B][H][W][C] grid, lse is [B*nW][heads][N]. */
int rib_oracle_fwd(int B, int H, int W, int heads, int d, int r, int M, int s,
                   double scale_c, double scale_p,
                   const float *q, const float *k, const float *v,
                   const float *fq, const float *fk, double *O, double *lse)
{
    geom_t g = make_geom(B, H, W, heads, d, r, M, s, scale_c, scale_p);
    if (!valid(&g)) return -1;
    int N = M * M;
    int64_t total = (int64_t)B * (H / M) * (W / M) * heads;
    int fail = 0;
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * N);
        double *O_u = (double *)malloc(sizeof(double) * N * d);
        if (!row || !O_u) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t u = 0; u < total; ++u) {
                int b, wy, wx, hd;
                unit_coords(&g, u, &b, &wy, &wx, &hd);
                fwd_unit(&g, q, k, v, fq, fk, u, O_u, lse + u * N, row);
                for (int i = 0; i < N; ++i)
                    memcpy(O + token_offset(&g, b, wy, wx, i, hd), O_u + (int64_t)i * d,
                           sizeof(double) * d);
            }
        }
        free(row);
        free(O_u);
    }
    return fail ? -2 : 0;
}

/* Backward for the listed units only: per-unit, un-scattered results.
 * dq_units,dk_units,dv_units are [n_units][N][d]; dfq_units,dfk_units are
 * [n_units][N][r] (this unit's contribution to dF_q, dF_k). */
int rib_oracle_bwd_units(int B, int H, int W, int heads, int d, int r, int M, int s,
                         double scale_c, double scale_p,
                         const float *q, const float *k, const float *v,
                         const float *fq, const float *fk, const float *dO,
                         int64_t n_units, const int64_t *units,
                         double *dq_units, double *dk_units, double *dv_units,
                         double *dfq_units, double *dfk_units)
{
    geom_t g = make_geom(B, H, W, heads, d, r, M, s, scale_c, scale_p);
    if (!valid(&g)) return -1;
    int N = M * M;
    int64_t total = (int64_t)B * (H / M) * (W / M) * heads;
    for (int64_t a = 0; a < n_units; ++a)
        if (units[a] < 0 || units[a] >= total) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *P = (double *)malloc(sizeof(double) * N);
        double *dS = (double *)malloc(sizeof(double) * N);
        if (!P || !dS) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t a = 0; a < n_units; ++a)
                bwd_unit(&g, q, k, v, fq, fk, dO, units[a],
                         dq_units + a * N * (int64_t)d, dk_units + a * N * (int64_t)d,
                         dv_units + a * N * (int64_t)d,
                         dfq_units + a * N * (int64_t)r, dfk_units + a * N * (int64_t)r, P, dS);
        }
        free(P);
        free(dS);
    }
    return fail ? -2 : 0;
}

/* Full backward.  dQ,dK,dV are [B][H][W][C] grids; dF_q,dF_k are [heads][N][r],
 * summed over every image and window.  All are overwritten. */
int rib_oracle_bwd(int B, int H, int W, int heads, int d, int r, int M, int s,
                   double scale_c, double scale_p,
                   const float *q, const float *k, const float *v,
                   const float *fq, const float *fk, const float *dO,
                   double *dQ, double *dK, double *dV, double *dFq, double *dFk)
{
    geom_t g = make_geom(B, H, W, heads, d, r, M, s, scale_c, scale_p);
    if (!valid(&g)) return -1;
    int N = M * M;
    int64_t total = (int64_t)B * (H / M) * (W / M) * heads;
    int64_t fsz = (int64_t)heads * N * r;
    memset(dFq, 0, sizeof(double) * fsz);
    memset(dFk, 0, sizeof(double) * fsz);
    int fail = 0;
#pragma omp parallel
    {
        double *P = (double *)malloc(sizeof(double) * N);
        double *dS = (double *)malloc(sizeof(double) * N);
        double *dq_u = (double *)malloc(sizeof(double) * N * d);
        double *dk_u = (double *)malloc(sizeof(double) * N * d);
        double *dv_u = (double *)malloc(sizeof(double) * N * d);
        double *dfq_u = (double *)malloc(sizeof(double) * N * (r > 0 ? r : 1));
        double *dfk_u = (double *)malloc(sizeof(double) * N * (r > 0 ? r : 1));
        if (!P || !dS || !dq_u || !dk_u || !dv_u || !dfq_u || !dfk_u) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t u = 0; u < total; ++u) {
                int b, wy, wx, hd;
                unit_coords(&g, u, &b, &wy, &wx, &hd);
                bwd_unit(&g, q, k, v, fq, fk, dO, u, dq_u, dk_u, dv_u, dfq_u, dfk_u, P, dS);
                for (int i = 0; i < N; ++i) {
                    int64_t off = token_offset(&g, b, wy, wx, i, hd);
                    memcpy(dQ + off, dq_u + (int64_t)i * d, sizeof(double) * d);
                    memcpy(dK + off, dk_u + (int64_t)i * d, sizeof(double) * d);
                    memcpy(dV + off, dv_u + (int64_t)i * d, sizeof(double) * d);
                }
#pragma omp critical(rib_oracle_df)
                {
                    double *aq = dFq + (int64_t)hd * N * r, *ak = dFk + (int64_t)hd * N * r;
                    for (int64_t e = 0; e < (int64_t)N * r; ++e) { aq[e] += dfq_u[e]; ak[e] += dfk_u[e]; }
                }
            }
        }
        free(P); free(dS); free(dq_u); free(dk_u); free(dv_u); free(dfq_u); free(dfk_u);
    }
    return fail ? -2 : 0;
}
