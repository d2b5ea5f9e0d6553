/*
 * Driver for a sanitizer build of the CPU oracle (host code only): calls every exported function of
 * oracle/lot_oracle.c on small, ragged shapes with exactly sized heap buffers, so that
 * -fsanitize=address,undefined reports any access past an array or any undefined arithmetic.
 * The values are checked only for being finite; what they must equal is the business of the pins.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

void lot_oracle_cost(const double* X, const double* Z, int n, int r, int d, double* C);
void lot_oracle_sinkhorn(const double* C, int n, int r, const double* a, const double* b, double eps, int T,
                         double* f, double* g);
void lot_oracle_coupling(const double* C, const double* f, const double* g, int n, int r, double eps, double* gamma);
void lot_oracle_apply_factored(const double* gamma1, const double* gamma2, const double* beta, const double* V,
                               int n, int r, int d_v, double* O);
void lot_oracle_dense_plan(const double* gamma1, const double* gamma2, const double* beta, int n, int r, double* P);
void lot_oracle_outer_plan(const double* gamma1, const double* gamma2, const double* beta, int n, int r, double* P);
void lot_oracle_apply_dense(const double* P, const double* V, int n, int d_v, double* O);
int lot_oracle_attention(int B, int H, int n, int d_k, int d_v, int r, const double* Q, const double* K,
                         const double* V, const double* Z, const double* beta, double eps, int T, double* O,
                         double* gamma1, double* gamma2, int threads);

static unsigned long long state = 0x9E3779B97F4A7C15ull;
static double uniform(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}
static double* filled(size_t count, double scale)
{
    double* p = (double*)malloc(sizeof(double) * (count ? count : 1));
    for (size_t i = 0; i < count; ++i) p[i] = uniform() * scale;
    return p;
}
static int all_finite(const double* p, size_t count)
{
    for (size_t i = 0; i < count; ++i)
        if (!isfinite(p[i])) return 0;
    return 1;
}

static int one_case(int B, int H, int n, int d_k, int d_v, int r, double eps, int T, int threads)
{
    const size_t G = (size_t)B * H;
    double* Q = filled(G * n * d_k, 1.0);
    double* K = filled(G * n * d_k, 1.0);
    double* V = filled(G * n * d_v, 1.0);
    double* Z = filled((size_t)H * r * d_k, 1.0);
    double* beta = (double*)malloc(sizeof(double) * H * r);
    for (int h = 0; h < H; ++h) {
        double tot = 0.0;
        for (int t = 0; t < r; ++t) tot += (beta[h * r + t] = 0.1 + uniform() + 0.5);
        for (int t = 0; t < r; ++t) beta[h * r + t] /= tot;
    }
    double* O = (double*)malloc(sizeof(double) * G * n * d_v);
    double* g1 = (double*)malloc(sizeof(double) * G * n * r);
    double* g2 = (double*)malloc(sizeof(double) * G * n * r);
    int ok = lot_oracle_attention(B, H, n, d_k, d_v, r, Q, K, V, Z, beta, eps, T, O, g1, g2, threads) >= 1;
    ok = ok && all_finite(O, G * n * d_v) && all_finite(g1, G * n * r) && all_finite(g2, G * n * r);
    ok = ok && lot_oracle_attention(B, H, n, d_k, d_v, r, Q, K, V, Z, beta, eps, T, O, NULL, NULL, 1) == 1;

    /* the pieces, on the first problem */
    double* C = (double*)malloc(sizeof(double) * n * r);
    double* a = (double*)malloc(sizeof(double) * n);
    double* f = (double*)malloc(sizeof(double) * n);
    double* g = (double*)malloc(sizeof(double) * r);
    double* gam = (double*)malloc(sizeof(double) * n * r);
    for (int i = 0; i < n; ++i) a[i] = 1.0 / n;
    lot_oracle_cost(Q, Z, n, r, d_k, C);
    lot_oracle_sinkhorn(C, n, r, a, beta, eps, T, f, g);
    lot_oracle_coupling(C, f, g, n, r, eps, gam);
    ok = ok && all_finite(gam, (size_t)n * r);
    double* P = (double*)malloc(sizeof(double) * n * n);
    double* P2 = (double*)malloc(sizeof(double) * n * n);
    double* Od = (double*)malloc(sizeof(double) * n * d_v);
    lot_oracle_dense_plan(g1, g2, beta, n, r, P);
    lot_oracle_outer_plan(g1, g2, beta, n, r, P2);
    lot_oracle_apply_dense(P, V, n, d_v, Od);
    lot_oracle_apply_factored(g1, g2, beta, V, n, r, d_v, O);
    ok = ok && all_finite(P, (size_t)n * n) && all_finite(P2, (size_t)n * n) && all_finite(Od, (size_t)n * d_v);
    free(Q); free(K); free(V); free(Z); free(beta); free(O); free(g1); free(g2);
    free(C); free(a); free(f); free(g); free(gam); free(P); free(P2); free(Od);
    return ok;
}

int main(void)
{
    int ok = 1;
    ok = ok && one_case(1, 1, 1, 1, 1, 1, 0.1, 1, 1);
    ok = ok && one_case(2, 3, 37, 5, 7, 4, 0.05, 6, 3);
    ok = ok && one_case(1, 2, 64, 32, 16, 33, 0.01, 3, 2);
    ok = ok && one_case(3, 1, 5, 8, 8, 9, 100.0, 2, 4);
    printf(ok ? "oracle sanitize run: ok\n" : "oracle sanitize run: NON-FINITE VALUE\n");
    return ok ? 0 : 1;
}
