/*
 * CPU oracle for the LOT attention forward (test infrastructure, not the product).
 *
 * Plain C, double precision, no blocking, no fusion, no reuse of partial results between
 * steps: every function is the paper's definition or algorithm step written out, so that
 * it can be checked against the paper by eye.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it; it shares no code with the HIP library.
 *
 * Notation (paper, Method section): Q, K in R^{n x d_k}, V in R^{n x d_v} (rows are tokens);
 * pivot locations Z in R^{r x d_k} with masses beta = p^0 in the open simplex; query and key
 * measures carry masses a (uniform 1/n in the paper's balanced case).
 *
 * Readings of the paper used here (each is also listed in the design notes):
 *  - orientation: Gamma1 is n x r (queries x pivots) and Gamma2 is r x n (pivots x keys),
 *    the shapes in which the paper's factored apply uses them ("Rank and complexity");
 *  - the similarity is maximised, so the Gibbs kernel is exp(+C/eps) as in the printed
 *    scaling form Gamma = Diag(u) exp(C/eps) Diag(v);
 *  - the marginals are not folded into the kernel: log a and log b enter the updates;
 *  - start from v = 1 (g = 0); one iteration = token-side update, then pivot-side update,
 *    so after every iteration the pivot marginal of each coupling equals beta exactly,
 *    which is what the gluing step assumes of its two factors;
 *  - the attention matrix is A = n * Gamma1 Diag(beta)^-1 Gamma2: the glued coupling has
 *    marginals 1/n, and only n times it has unit row and column sums as the paper requires
 *    of A ("Glued coupling and doubly-stochastic attention").
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* C[i,t] = <x_i, z_t>  (paper: C^(1)_it = z_t^T q_i, C^(2)_jt = z_t^T k_j). */
void lot_oracle_cost(const double* X, const double* Z, int n, int r, int d, double* C)
{
    for (int i = 0; i < n; ++i)
        for (int t = 0; t < r; ++t) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += X[(size_t)i * d + c] * Z[(size_t)t * d + c];
            C[(size_t)i * r + t] = s;
        }
}

/* log sum_k exp(x_k) over `count` values spaced `stride` apart, with the maximum taken out. */
static double logsumexp(const double* x, int count, size_t stride)
{
    double m = x[0];
    for (int k = 1; k < count; ++k) if (x[k * stride] > m) m = x[k * stride];
    double s = 0.0;
    for (int k = 0; k < count; ++k) s += exp(x[k * stride] - m);
    return m + log(s);
}

/*
 * T Sinkhorn iterations for  max <C,G> + eps H(G)  over G >= 0 with G 1 = a, G^T 1 = b,
 * in the log domain: u = exp(f/eps), v = exp(g/eps) are the paper's scaling vectors of
 * Gamma = Diag(u) exp(C/eps) Diag(v).  The u-update makes the row sums equal a, the
 * v-update makes the column sums equal b:
 *     f_i = eps (log a_i - log sum_t exp((C_it + g_t)/eps))
 *     g_t = eps (log b_t - log sum_i exp((C_it + f_i)/eps))
 * C is n x r row-major; f has n entries, g has r entries; g starts at 0.
 */
void lot_oracle_sinkhorn(const double* C, int n, int r, const double* a, const double* b,
                         double eps, int T, double* f, double* g)
{
    double* col = (double*)malloc(sizeof(double) * (size_t)(n > r ? n : r));
    for (int t = 0; t < r; ++t) g[t] = 0.0;
    for (int i = 0; i < n; ++i) f[i] = 0.0;
    for (int it = 0; it < T; ++it) {
        for (int i = 0; i < n; ++i) {
            for (int t = 0; t < r; ++t) col[t] = (C[(size_t)i * r + t] + g[t]) / eps;
            f[i] = eps * (log(a[i]) - logsumexp(col, r, 1));
        }
        for (int t = 0; t < r; ++t) {
            for (int i = 0; i < n; ++i) col[i] = (C[(size_t)i * r + t] + f[i]) / eps;
            g[t] = eps * (log(b[t]) - logsumexp(col, n, 1));
        }
    }
    free(col);
}

/* Gamma_it = exp((C_it + f_i + g_t)/eps), n x r row-major. */
void lot_oracle_coupling(const double* C, const double* f, const double* g, int n, int r,
                         double eps, double* Gamma)
{
    for (int i = 0; i < n; ++i)
        for (int t = 0; t < r; ++t)
            Gamma[(size_t)i * r + t] = exp((C[(size_t)i * r + t] + f[i] + g[t]) / eps);
}

/*
 * The two couplings of one (batch, head) problem with uniform token masses 1/n:
 * gamma1 (n x r) from C1 = Q Z^T and gamma2 (r x n), the transpose of the coupling
 * obtained from C2 = K Z^T.
 */
void lot_oracle_couplings_one(const double* Q, const double* K, const double* Z,
                              const double* beta, int n, int d_k, int r, double eps, int T,
                              double* gamma1, double* gamma2)
{
    double* C = (double*)malloc(sizeof(double) * (size_t)n * r);
    double* G = (double*)malloc(sizeof(double) * (size_t)n * r);
    double* f = (double*)malloc(sizeof(double) * (size_t)n);
    double* g = (double*)malloc(sizeof(double) * (size_t)r);
    double* a = (double*)malloc(sizeof(double) * (size_t)n);
    for (int i = 0; i < n; ++i) a[i] = 1.0 / (double)n;

    lot_oracle_cost(Q, Z, n, r, d_k, C);
    lot_oracle_sinkhorn(C, n, r, a, beta, eps, T, f, g);
    lot_oracle_coupling(C, f, g, n, r, eps, gamma1);

    lot_oracle_cost(K, Z, n, r, d_k, C);
    lot_oracle_sinkhorn(C, n, r, a, beta, eps, T, f, g);
    lot_oracle_coupling(C, f, g, n, r, eps, G);
    for (int j = 0; j < n; ++j)
        for (int t = 0; t < r; ++t) gamma2[(size_t)t * n + j] = G[(size_t)j * r + t];

    free(C); free(G); free(f); free(g); free(a);
}

/*
 * Factored apply (paper, "Rank and complexity"):  Y = Gamma2 V (r x d_v),
 * Y' = Diag(beta)^-1 Y,  O = n * Gamma1 Y'  (n x d_v).
 */
void lot_oracle_apply_factored(const double* gamma1, const double* gamma2, const double* beta,
                               const double* V, int n, int r, int d_v, double* O)
{
    double* Y = (double*)calloc((size_t)r * d_v, sizeof(double));
    for (int t = 0; t < r; ++t)
        for (int j = 0; j < n; ++j)
            for (int c = 0; c < d_v; ++c)
                Y[(size_t)t * d_v + c] += gamma2[(size_t)t * n + j] * V[(size_t)j * d_v + c];
    for (int t = 0; t < r; ++t)
        for (int c = 0; c < d_v; ++c) Y[(size_t)t * d_v + c] /= beta[t];
    for (int i = 0; i < n; ++i)
        for (int c = 0; c < d_v; ++c) {
            double s = 0.0;
            for (int t = 0; t < r; ++t) s += gamma1[(size_t)i * r + t] * Y[(size_t)t * d_v + c];
            O[(size_t)i * d_v + c] = (double)n * s;
        }
    free(Y);
}

/* Dense glued coupling P = Gamma1 Diag(beta)^-1 Gamma2 (n x n); small n only. */
void lot_oracle_dense_plan(const double* gamma1, const double* gamma2, const double* beta,
                           int n, int r, double* P)
{
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int t = 0; t < r; ++t)
                s += gamma1[(size_t)i * r + t] / beta[t] * gamma2[(size_t)t * n + j];
            P[(size_t)i * n + j] = s;
        }
}

/*
 * The same matrix as a sum of r outer products of the pivots' soft clusters
 * (paper, appendix "LOTFormer and soft clustering"):
 * P = sum_t (1/beta_t) Gamma1[:,t] (x) Gamma2[t,:].
 */
void lot_oracle_outer_plan(const double* gamma1, const double* gamma2, const double* beta,
                           int n, int r, double* P)
{
    memset(P, 0, sizeof(double) * (size_t)n * n);
    for (int t = 0; t < r; ++t)
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                P[(size_t)i * n + j] += (1.0 / beta[t]) * gamma1[(size_t)i * r + t]
                                        * gamma2[(size_t)t * n + j];
}

/* O = n * P V with the dense n x n plan (brute force; small n only). */
void lot_oracle_apply_dense(const double* P, const double* V, int n, int d_v, double* O)
{
    for (int i = 0; i < n; ++i)
        for (int c = 0; c < d_v; ++c) {
            double s = 0.0;
            for (int j = 0; j < n; ++j) s += P[(size_t)i * n + j] * V[(size_t)j * d_v + c];
            O[(size_t)i * d_v + c] = (double)n * s;
        }
}

/*
 * Whole batch.  Q, K: [B,H,n,d_k]; V, O: [B,H,n,d_v]; Z: [H,r,d_k]; beta: [H,r] (one pivot
 * measure per head, shared by the batch).  gamma1 [B,H,n,r] and gamma2 [B,H,r,n] are
 * optional outputs (NULL to skip).  The (b,h) problems are independent; `threads` > 1
 * spreads them over OpenMP threads, which changes no arithmetic.
 * Returns the number of threads used.
 */
int lot_oracle_attention(int B, int H, int n, int d_k, int d_v, int r,
                         const double* Q, const double* K, const double* V,
                         const double* Z, const double* beta, double eps, int T,
                         double* O, double* gamma1, double* gamma2, int threads)
{
    int used = 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#else
    (void)threads;
#endif
    for (int p = 0; p < B * H; ++p) {
        int h = p % H;
        size_t nr = (size_t)n * r;
        double* g1 = gamma1 ? gamma1 + (size_t)p * nr : (double*)malloc(sizeof(double) * nr);
        double* g2 = gamma2 ? gamma2 + (size_t)p * nr : (double*)malloc(sizeof(double) * nr);
        lot_oracle_couplings_one(Q + (size_t)p * n * d_k, K + (size_t)p * n * d_k,
                                 Z + (size_t)h * r * d_k, beta + (size_t)h * r,
                                 n, d_k, r, eps, T, g1, g2);
        lot_oracle_apply_factored(g1, g2, beta + (size_t)h * r, V + (size_t)p * n * d_v,
                                  n, r, d_v, O + (size_t)p * n * d_v);
        if (!gamma1) free(g1);
        if (!gamma2) free(g2);
    }
    return used;
}
