/* Driver for a sanitizer build of the CPU oracle (test infrastructure).
 *
 * Calls every entry point of rib_oracle.c on small shapes whose buffers are sized
 * exactly (shifted windows, H != W, one token per window, r = 0), so that an
 * out-of-bounds index, a read of uninitialised memory used as an index, or signed
 * overflow in the index arithmetic trips AddressSanitizer / UBSan.  Built and run
 * by tests/test_oracle_sanitized.py:
 *   gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp \
 *       oracle/rib_oracle.c oracle/sanitize_check.c -lm
 * Prints "ok" and exits 0 when every call returned 0 and produced finite values. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int rib_oracle_fwd(int, int, int, int, int, int, int, int, double, double, const float *, const float *, const float *,
                   const float *, const float *, double *, double *);
int rib_oracle_bwd(int, int, int, int, int, int, int, int, double, double, const float *, const float *, const float *,
                   const float *, const float *, const float *, double *, double *, double *, double *, double *);
int rib_oracle_fwd_units(int, int, int, int, int, int, int, int, double, double, const float *, const float *,
                         const float *, const float *, const float *, int64_t, const int64_t *, double *, double *);
int rib_oracle_bwd_units(int, int, int, int, int, int, int, int, double, double, const float *, const float *,
                         const float *, const float *, const float *, const float *, int64_t, const int64_t *,
                         double *, double *, double *, double *, double *);

static uint32_t state = 12345u;
static float draw(void)
{
    state = state * 1664525u + 1013904223u;
    return (float)((state >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static float *fbuf(size_t n)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = draw();
    return p;
}
static double *dbuf(size_t n) { return (double *)malloc(sizeof(double) * (n ? n : 1)); }
static int finite_all(const double *p, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(p[i])) return 0;
    return 1;
}

static int run(int B, int H, int W, int heads, int d, int r, int M, int s)
{
    const int N = M * M, C = heads * d;
    const size_t grid = (size_t)B * H * W * C, feat = (size_t)heads * N * r;
    const int64_t nwin = (int64_t)B * (H / M) * (W / M), units = nwin * heads;
    float *q = fbuf(grid), *k = fbuf(grid), *v = fbuf(grid), *go = fbuf(grid), *fq = fbuf(feat), *fk = fbuf(feat);
    double *O = dbuf(grid), *lse = dbuf((size_t)units * N);
    double *dQ = dbuf(grid), *dK = dbuf(grid), *dV = dbuf(grid), *dFq = dbuf(feat), *dFk = dbuf(feat);
    int ok = rib_oracle_fwd(B, H, W, heads, d, r, M, s, 0.3, 0.2, q, k, v, fq, fk, O, lse) == 0;
    ok = ok && finite_all(O, grid) && finite_all(lse, (size_t)units * N);
    ok = ok && rib_oracle_bwd(B, H, W, heads, d, r, M, s, 0.3, 0.2, q, k, v, fq, fk, go, dQ, dK, dV, dFq, dFk) == 0;
    ok = ok && finite_all(dQ, grid) && finite_all(dK, grid) && finite_all(dV, grid) && finite_all(dFq, feat);
    /* the first and the last unit through the per-unit entry points */
    int64_t pick[2] = { 0, units - 1 };
    double *Ou = dbuf((size_t)2 * N * d), *lu = dbuf((size_t)2 * N);
    double *a = dbuf((size_t)2 * N * d), *b = dbuf((size_t)2 * N * d), *c = dbuf((size_t)2 * N * d);
    double *e = dbuf((size_t)2 * N * r), *f = dbuf((size_t)2 * N * r);
    ok = ok && rib_oracle_fwd_units(B, H, W, heads, d, r, M, s, 0.3, 0.2, q, k, v, fq, fk, 2, pick, Ou, lu) == 0;
    ok = ok && rib_oracle_bwd_units(B, H, W, heads, d, r, M, s, 0.3, 0.2, q, k, v, fq, fk, go, 2, pick, a, b, c, e, f) == 0;
    ok = ok && finite_all(Ou, (size_t)2 * N * d) && finite_all(a, (size_t)2 * N * d);
    free(q); free(k); free(v); free(go); free(fq); free(fk); free(O); free(lse);
    free(dQ); free(dK); free(dV); free(dFq); free(dFk); free(Ou); free(lu); free(a); free(b); free(c); free(e); free(f);
    return ok;
}

int main(void)
{
    int ok = run(2, 4, 6, 2, 3, 2, 2, 1)      /* H != W, shifted */
          && run(1, 3, 5, 2, 3, 2, 1, 0)      /* one token per window */
          && run(1, 8, 8, 3, 5, 0, 4, 3)      /* r = 0 */
          && run(2, 9, 6, 1, 7, 3, 3, 2)      /* odd everything */
          && run(1, 16, 16, 2, 30, 16, 16, 8);/* the paper's head shape, one 16 x 16 window */
    /* invalid shapes must be refused without touching memory */
    ok = ok && rib_oracle_fwd(1, 5, 4, 1, 2, 1, 2, 0, 1.0, 1.0, NULL, NULL, NULL, NULL, NULL, NULL, NULL) != 0;
    puts(ok ? "ok" : "FAILED");
    return ok ? 0 : 1;
}
