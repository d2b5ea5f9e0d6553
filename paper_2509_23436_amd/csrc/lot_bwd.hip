// Backward pass of LOT attention, plain path: gradients of <O, dO> with respect to Q, K, V, Z, beta
// through the glued composition and through every iteration of both Sinkhorn solves (paper,
// "Learning": everything is trained by backpropagating through the two problems and the glue).
// One plain fp32 kernel per step, intermediates materialised in the workspace, every reduction in
// a fixed order (bit-reproducible).  Any shape.
//
// Forward quantities are recomputed, not saved by the caller: the similarities C, the pivot
// potentials after every iteration g^0 .. g^T (T+1 vectors of r numbers per solve: the only
// per-iteration state the reverse sweep needs) and the final couplings.
//
// Notation for one solve (a = 1/n, b = beta):  P^k = a * softmax_rows((C + g^{k-1})/eps) is the plan
// after the token-side update of iteration k, c^k its column sums, g^k = g^{k-1} + eps log(b / c^k),
// and the returned coupling is Gamma = P^T * (b / c^T) column-wise.  Reverse sweep, given dGamma:
//   last step:  s_t = sum_i dGamma_it Gamma_it;  dc_t = -s_t / c^T_t;  db_t += s_t / b_t;
//               dP_it = dGamma_it b_t / c^T_t + dc_t
//   step k<T:   (given dg^k)  dc_t = -eps dg^k_t / c^k_t;  db_t += eps dg^k_t / b_t;  dP_it = dc_t
//   both:       e_i = (1/a) sum_t dP_it P_it;  dY_it = P_it (dP_it - e_i);  dC += dY/eps;
//               dg^{k-1}_t = [k<T] dg^k_t + (1/eps) sum_i dY_it
// with c^k_t = b_t exp((g^{k-1}_t - g^k_t)/eps) read off the stored potentials.
// Glue (O = n Gamma1 Y', Y' = Diag(b)^-1 Gamma2 V):  dY' = n Gamma1^T dO;  dGamma1 = n dO Y'^T;
//   dYraw = dY'/b;  db_t -= <dY'_t, Y'_t>/b_t;  dV = Gamma2^T dYraw;  dGamma2 = dYraw V^T.
// Finally dQ = dC1 Z, dK = dC2 Z, dZ = sum over the batch of dC1^T Q + dC2^T K.
#include "lot_internal.h"
#include "lot_plain_kernels.h"

namespace lot {
namespace {

constexpr int kChunk = kRefChunk;   // tokens per partial sum

// Gamma[pair][i][t] = exp((C_it + f_i + g_t)/eps), both sides token-major.
__global__ void bwd_couplings(const float* __restrict__ C, const float* __restrict__ f,
                              const float* __restrict__ gpot, float* __restrict__ gam,
                              size_t total, int n, int r, float eps)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const size_t row = idx / r;
    const int t = (int)(idx % r);
    gam[idx] = expf((C[idx] + f[row] + gpot[(row / n) * r + t]) / eps);
}

// part[p][chunk][t][c] = sum over the chunk's tokens i of A[p][i][t] * X[p][i][c]
// (A is fp32 [P][n][r]; X is [P][stride][dx] in the I/O type, n rows used).  One block per (p, chunk, t).
template <typename T>
__global__ void bwd_tx_partial(const float* __restrict__ A, const T* __restrict__ X, float* __restrict__ part,
                               int n, int stride, int r, int dx, int chunks)
{
    const int t = blockIdx.x % r;
    const int chunk = (blockIdx.x / r) % chunks;
    const size_t p = blockIdx.x / ((size_t)r * chunks);
    const int i0 = chunk * kChunk, i1 = min(n, i0 + kChunk);
    for (int c = threadIdx.x; c < dx; c += blockDim.x) {
        float acc = 0.f;
        for (int i = i0; i < i1; ++i) acc = fmaf(A[(p * n + i) * r + t], ld(X, (p * stride + i) * dx + c), acc);
        part[((p * chunks + chunk) * r + t) * dx + c] = acc;
    }
}
// out[p][t][c] = scale * sum over chunks (index order)
__global__ void bwd_tx_final(const float* __restrict__ part, float* __restrict__ out, size_t total,
                             int r, int dx, int chunks, float scale)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (p, t, c)
    if (idx >= total) return;
    const size_t p = idx / ((size_t)r * dx);
    const size_t tc = idx % ((size_t)r * dx);
    float acc = 0.f;
    for (int k = 0; k < chunks; ++k) acc += part[(p * chunks + k) * r * dx + tc];
    out[idx] = scale * acc;
}

// Y'[g][t][:] = Yraw / beta_t ; dYraw = dY' / beta_t ; db_glue[g][t] = -<dY'_t, Y'_t> / beta_t
__global__ void bwd_glue_pivots(float* __restrict__ Yp, float* __restrict__ dYp, const float* __restrict__ beta,
                                float* __restrict__ db_glue, int GR, int H, int r, int dv, int stage)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;   // (g, t)
    if (idx >= GR) return;
    const int g = idx / r, t = idx % r;
    const float b = beta[(g % H) * r + t];
    if (stage == 0) {
        for (int c = 0; c < dv; ++c) Yp[(size_t)idx * dv + c] /= b;
    } else {
        float dot = 0.f;
        for (int c = 0; c < dv; ++c) dot = fmaf(dYp[(size_t)idx * dv + c], Yp[(size_t)idx * dv + c], dot);
        db_glue[idx] = -dot / b;
        for (int c = 0; c < dv; ++c) dYp[(size_t)idx * dv + c] /= b;
    }
}

// out[p][i][t] = scale * sum_c X[p][i][c] * M[p][t][c]        (dGamma1 = n dO Y'^T, dGamma2 = V dYraw^T)
template <typename T>
__global__ void bwd_outer(const T* __restrict__ X, const float* __restrict__ M, float* __restrict__ out,
                          size_t total, int n, int stride, int r, int dx, float scale)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (p, i, t)
    if (idx >= total) return;
    const size_t pi = idx / r;
    const int t = (int)(idx % r);
    const size_t p = pi / n;
    float acc = 0.f;
    const size_t row = p * stride + pi % n;          // X is [P][stride][dx]
    for (int c = 0; c < dx; ++c) acc = fmaf(ld(X, row * dx + c), M[(p * r + t) * dx + c], acc);
    out[idx] = scale * acc;
}

// out[p][i][c] = sum_t A[p][i][t] * M[m(p)][t][c], M per problem (per_head = 0) or per head.
template <typename T>
__global__ void bwd_apply(const float* __restrict__ A, const float* __restrict__ M, T* __restrict__ out,
                          size_t total, int n, int stride, int r, int dx, int per_head, int H)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (p, i, c)
    if (idx >= total) return;
    const size_t pi = idx / dx;
    const int c = (int)(idx % dx);
    const size_t p = pi / n;
    const size_t m = per_head ? (p % H) : p;
    float acc = 0.f;
    for (int t = 0; t < r; ++t) acc = fmaf(A[pi * r + t], M[(m * r + t) * dx + c], acc);
    st(out, (p * stride + pi % n) * dx + c, acc);          // out is [P][stride][dx]
}

// colpart[pair][chunk][t] = sum over the chunk's tokens of A_it * B_it (B may be null: plain sum).
__global__ void bwd_col_partial(const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ part,
                                int n, int r, int chunks)
{
    const size_t pair = blockIdx.x / chunks;
    const int chunk = blockIdx.x % chunks;
    const int i0 = chunk * kChunk, i1 = min(n, i0 + kChunk);
    for (int t = threadIdx.x; t < r; t += blockDim.x) {
        float acc = 0.f;
        if (B) for (int i = i0; i < i1; ++i) acc = fmaf(A[(pair * n + i) * r + t], B[(pair * n + i) * r + t], acc);
        else for (int i = i0; i < i1; ++i) acc += A[(pair * n + i) * r + t];
        part[(pair * chunks + chunk) * r + t] = acc;
    }
}

// Pivot-side bookkeeping of one reverse step, one thread per (pair, t).
//   last != 0: colsum holds s_t = sum_i dGamma Gamma  -> dc, rho, db
//   last == 0: dg holds dg^k                         -> dc, db
// c^k_t = beta_t exp((g^{k-1}_t - g^k_t)/eps).
__global__ void bwd_pivot_pre(const float* __restrict__ part, const float* __restrict__ g_prev,
                              const float* __restrict__ g_cur, const float* __restrict__ beta,
                              const float* __restrict__ dg, float* __restrict__ dc, float* __restrict__ rho,
                              float* __restrict__ db, int pairs, int G, int H, int r, int chunks, float eps, int last)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= pairs * r) return;
    const int pair = idx / r, t = idx % r;
    const float b = beta[((pair % G) % H) * r + t];
    const float c = b * expf((g_prev[idx] - g_cur[idx]) / eps);
    if (last) {
        float s = 0.f;
        for (int k = 0; k < chunks; ++k) s += part[((size_t)pair * chunks + k) * r + t];
        dc[idx] = -s / c;
        rho[idx] = b / c;
        db[idx] = s / b;          // first contribution of this solve
    } else {
        dc[idx] = -eps * dg[idx] / c;
        db[idx] += eps * dg[idx] / b;
    }
}

// Token side of one reverse step, one thread per (pair, i):
//   P_it = a softmax_t((C_it + gprev_t)/eps);  dP_it = [last] dGamma_it rho_t + dc_t;
//   e_i = (1/a) sum_t dP_it P_it;  dY_it = P_it (dP_it - e_i);  dC_it (+)= dY_it/eps;  Ybuf = dY.
__global__ void bwd_rows(const float* __restrict__ C, const float* __restrict__ g_prev,
                         const float* __restrict__ dGam, const float* __restrict__ rho,
                         const float* __restrict__ dc, float* __restrict__ dC, float* __restrict__ Ybuf,
                         size_t rows, int n, int r, float eps, int last)
{
    const size_t row = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const size_t pair = row / n;
    const float* c = C + row * r;
    const float* gp = g_prev + pair * r;
    const float* dcp = dc + pair * r;
    const float* rh = rho + pair * r;
    float m = -INFINITY;
    for (int t = 0; t < r; ++t) m = fmaxf(m, (c[t] + gp[t]) / eps);
    float s = 0.f;
    for (int t = 0; t < r; ++t) s += expf((c[t] + gp[t]) / eps - m);
    const float inv_s = 1.f / s;
    // e_i = (1/a) sum_t dP_it P_it with P_it = a * exp(.)/s  ->  sum_t dP_it exp(.)/s
    float e = 0.f;
    for (int t = 0; t < r; ++t) {
        const float w = expf((c[t] + gp[t]) / eps - m) * inv_s;
        const float dP = (last ? dGam[row * r + t] * rh[t] : 0.f) + dcp[t];
        e = fmaf(dP, w, e);
    }
    const float a = 1.f / (float)n;
    for (int t = 0; t < r; ++t) {
        const float w = expf((c[t] + gp[t]) / eps - m) * inv_s;
        const float dP = (last ? dGam[row * r + t] * rh[t] : 0.f) + dcp[t];
        const float dY = a * w * (dP - e);
        Ybuf[row * r + t] = dY;
        if (last) dC[row * r + t] = dY / eps;
        else dC[row * r + t] += dY / eps;
    }
}

// dg^{k-1}_t = [last ? 0 : dg^k_t] + (1/eps) sum over chunks of colpart
__global__ void bwd_pivot_post(const float* __restrict__ part, float* __restrict__ dg, int pairs, int r,
                               int chunks, float eps, int last)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= pairs * r) return;
    const int pair = idx / r, t = idx % r;
    float s = 0.f;
    for (int k = 0; k < chunks; ++k) s += part[((size_t)pair * chunks + k) * r + t];
    dg[idx] = (last ? 0.f : dg[idx]) + s / eps;
}

// dZ[h][t][c] = sum over b (index order) of the two sides; dbeta[h][t] likewise with the glue term.
__global__ void bwd_head_sums(const float* __restrict__ dZ_pair, const float* __restrict__ db_pair,
                              const float* __restrict__ db_glue, float* __restrict__ dZ, float* __restrict__ dbeta,
                              int B, int H, int r, int d)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;   // (h, t, c) with c == d meaning beta
    const int per = r * (d + 1);
    if (idx >= H * per) return;
    const int h = idx / per, t = (idx % per) / (d + 1), c = idx % (d + 1);
    const int G = B * H;
    float acc = 0.f;
    for (int b = 0; b < B; ++b) {
        const int g = b * H + h;
        if (c < d) {
            acc += dZ_pair[(((size_t)0 * G + g) * r + t) * d + c];
            acc += dZ_pair[(((size_t)1 * G + g) * r + t) * d + c];
        } else {
            acc += db_glue[g * r + t];
            acc += db_pair[((size_t)0 * G + g) * r + t];
            acc += db_pair[((size_t)1 * G + g) * r + t];
        }
    }
    if (c < d) dZ[((size_t)h * r + t) * d + c] = acc;
    else dbeta[h * r + t] = acc;
}

// Z as the forward pass used it (rounded to bf16 for bf16 I/O), [H][r][d] fp32.
__global__ void bwd_round_z(const float* __restrict__ Z, float* __restrict__ Zr, int count, int round_z)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= count) return;
    Zr[idx] = round_z ? bf16_to_f32(f32_to_bf16_rne(Z[idx])) : Z[idx];
}

template <typename T>
int run_backward_t(const BwdArgs& a)
{
    const lot_shape& s = a.s;
    const int G = s.B * s.H, n = s.n, r = s.r, pairs = 2 * G, T_ = a.iters;
    const int chunks = (n + kChunk - 1) / kChunk;
    const int stride = a.n_stride > 0 ? a.n_stride : n;      // tokens between problems in the caller's tensors
    const BwdWorkspace& L = a.lay;
    float* C = (float*)(a.ws + L.C);
    float* f = (float*)(a.ws + L.f);
    float* ghist = (float*)(a.ws + L.ghist);       // [T+1][pairs][r]
    float* pm = (float*)(a.ws + L.part_m);
    float* ps = (float*)(a.ws + L.part_s);
    float* gam = (float*)(a.ws + L.gam);           // [pairs][n][r]
    float* dgam = (float*)(a.ws + L.dgam);
    float* dC = (float*)(a.ws + L.dC);
    float* ybuf = (float*)(a.ws + L.ybuf);
    float* tx_part = (float*)(a.ws + L.tx_part);   // [pairs][chunks][r][dmax]
    float* Yp = (float*)(a.ws + L.Yp);
    float* dYp = (float*)(a.ws + L.dYp);
    float* db_glue = (float*)(a.ws + L.db_glue);
    float* colpart = (float*)(a.ws + L.colpart);
    float* dc = (float*)(a.ws + L.dc);
    float* rho = (float*)(a.ws + L.rho);
    float* dg = (float*)(a.ws + L.dg);
    float* db_pair = (float*)(a.ws + L.db_pair);
    float* dZ_pair = (float*)(a.ws + L.dZ_pair);   // [pairs][r][d_k]
    float* Zr = (float*)(a.ws + L.Zr);
    hipStream_t st_ = a.stream;
    ref_mark<<<1, 1, 0, st_>>>((unsigned long long*)a.ws, next_nonce());   // no device-side waits on this path
    const size_t slab = (size_t)pairs * r;
    const size_t nelem = (size_t)pairs * n * r;
    const size_t rows = (size_t)pairs * n;
    const size_t half = (size_t)G * n * r;
    const unsigned pr_blocks = blocks_for(slab, 256);

    // ---- forward, keeping the pivot potentials of every iteration
    ref_cost<T><<<blocks_for(nelem, 256), 256, 0, st_>>>((const T*)a.Q, (const T*)a.K, a.Z, C, G, s.H, n, stride, s.d_k, r,
                                                         s.io_dtype == LOT_BF16);
    ref_zero<<<pr_blocks, 256, 0, st_>>>(ghist, slab);
    for (int k = 1; k <= T_; ++k) {
        ref_f_update<<<blocks_for(rows, 256), 256, 0, st_>>>(C, ghist + (size_t)(k - 1) * slab, f, rows, n, r, a.eps);
        ref_g_partial<<<(unsigned)pairs * chunks, 64, 0, st_>>>(C, f, pm, ps, n, r, chunks, a.eps);
        ref_g_final<<<pr_blocks, 256, 0, st_>>>(pm, ps, a.beta, ghist + (size_t)k * slab, pairs, G, s.H, r, chunks, a.eps);
    }
    bwd_couplings<<<blocks_for(nelem, 256), 256, 0, st_>>>(C, f, ghist + (size_t)T_ * slab, gam, nelem, n, r, a.eps);
    const float* gam1 = gam;            // [G][n][r]
    const float* gam2 = gam + half;     // [G][n][r]  (token-major: the transpose of the r x n plan)

    // ---- glue
    // Y' = Diag(beta)^-1 Gamma2 V
    bwd_tx_partial<T><<<(unsigned)((size_t)G * chunks * r), 64, 0, st_>>>(gam2, (const T*)a.V, tx_part, n, stride, r, s.d_v, chunks);
    bwd_tx_final<<<blocks_for((size_t)G * r * s.d_v, 256), 256, 0, st_>>>(tx_part, Yp, (size_t)G * r * s.d_v, r, s.d_v, chunks, 1.f);
    bwd_glue_pivots<<<blocks_for((size_t)G * r, 128), 128, 0, st_>>>(Yp, dYp, a.beta, db_glue, G * r, s.H, r, s.d_v, 0);
    // dY' = n Gamma1^T dO
    bwd_tx_partial<T><<<(unsigned)((size_t)G * chunks * r), 64, 0, st_>>>(gam1, (const T*)a.dO, tx_part, n, stride, r, s.d_v, chunks);
    bwd_tx_final<<<blocks_for((size_t)G * r * s.d_v, 256), 256, 0, st_>>>(tx_part, dYp, (size_t)G * r * s.d_v, r, s.d_v, chunks, (float)n);
    // dGamma1 = n dO Y'^T (before dY' is rescaled; it does not use dY')
    bwd_outer<T><<<blocks_for(half, 256), 256, 0, st_>>>((const T*)a.dO, Yp, dgam, half, n, stride, r, s.d_v, (float)n);
    // db_glue, dYraw = dY'/beta
    bwd_glue_pivots<<<blocks_for((size_t)G * r, 128), 128, 0, st_>>>(Yp, dYp, a.beta, db_glue, G * r, s.H, r, s.d_v, 1);
    // dV = Gamma2^T dYraw ; dGamma2 = V dYraw^T
    bwd_apply<T><<<blocks_for((size_t)G * n * s.d_v, 256), 256, 0, st_>>>(gam2, dYp, (T*)a.dV, (size_t)G * n * s.d_v, n, stride, r, s.d_v, 0, s.H);
    bwd_outer<T><<<blocks_for(half, 256), 256, 0, st_>>>((const T*)a.V, dYp, dgam + half, half, n, stride, r, s.d_v, 1.f);

    // ---- both Sinkhorn solves, reverse sweep (the two solves side by side: pair = side * G + g)
    bwd_col_partial<<<(unsigned)pairs * chunks, 64, 0, st_>>>(dgam, gam, colpart, n, r, chunks);
    for (int k = T_; k >= 1; --k) {
        const int last = k == T_;
        const float* g_prev = ghist + (size_t)(k - 1) * slab;
        const float* g_cur = ghist + (size_t)k * slab;
        bwd_pivot_pre<<<pr_blocks, 256, 0, st_>>>(colpart, g_prev, g_cur, a.beta, dg, dc, rho, db_pair, pairs, G, s.H, r, chunks, a.eps, last);
        bwd_rows<<<blocks_for(rows, 256), 256, 0, st_>>>(C, g_prev, dgam, rho, dc, dC, ybuf, rows, n, r, a.eps, last);
        bwd_col_partial<<<(unsigned)pairs * chunks, 64, 0, st_>>>(ybuf, nullptr, colpart, n, r, chunks);
        bwd_pivot_post<<<pr_blocks, 256, 0, st_>>>(colpart, dg, pairs, r, chunks, a.eps, last);
    }

    // ---- similarities: dQ = dC1 Z, dK = dC2 Z, dZ = sum_b (dC1^T Q + dC2^T K)
    bwd_round_z<<<blocks_for((size_t)s.H * r * s.d_k, 256), 256, 0, st_>>>(a.Z, Zr, s.H * r * s.d_k, s.io_dtype == LOT_BF16);
    bwd_apply<T><<<blocks_for((size_t)G * n * s.d_k, 256), 256, 0, st_>>>(dC, Zr, (T*)a.dQ, (size_t)G * n * s.d_k, n, stride, r, s.d_k, 1, s.H);
    bwd_apply<T><<<blocks_for((size_t)G * n * s.d_k, 256), 256, 0, st_>>>(dC + half, Zr, (T*)a.dK, (size_t)G * n * s.d_k, n, stride, r, s.d_k, 1, s.H);
    bwd_tx_partial<T><<<(unsigned)((size_t)G * chunks * r), 64, 0, st_>>>(dC, (const T*)a.Q, tx_part, n, stride, r, s.d_k, chunks);
    bwd_tx_final<<<blocks_for((size_t)G * r * s.d_k, 256), 256, 0, st_>>>(tx_part, dZ_pair, (size_t)G * r * s.d_k, r, s.d_k, chunks, 1.f);
    bwd_tx_partial<T><<<(unsigned)((size_t)G * chunks * r), 64, 0, st_>>>(dC + half, (const T*)a.K, tx_part, n, stride, r, s.d_k, chunks);
    bwd_tx_final<<<blocks_for((size_t)G * r * s.d_k, 256), 256, 0, st_>>>(tx_part, dZ_pair + (size_t)G * r * s.d_k, (size_t)G * r * s.d_k, r, s.d_k, chunks, 1.f);
    bwd_head_sums<<<blocks_for((size_t)s.H * r * (s.d_k + 1), 256), 256, 0, st_>>>(dZ_pair, db_pair, db_glue, a.dZ, a.dbeta, s.B, s.H, r, s.d_k);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

}  // namespace

BwdWorkspace carve_bwd(const lot_shape& s, int iters)
{
    BwdWorkspace w{};
    size_t off = 256;      // the status words come first, as in the other workspaces
    auto take = [&](size_t bytes) { size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
    const size_t G = (size_t)s.B * s.H, n = s.n, r = s.r, pairs = 2 * G;
    const size_t chunks = (n + kRefChunk - 1) / kRefChunk;
    const size_t dmax = s.d_k > s.d_v ? s.d_k : s.d_v;
    w.C = take(pairs * n * r * 4);
    w.f = take(pairs * n * 4);
    w.ghist = take((size_t)(iters + 1) * pairs * r * 4);
    w.part_m = take(pairs * chunks * r * 4);
    w.part_s = take(pairs * chunks * r * 4);
    w.gam = take(pairs * n * r * 4);
    w.dgam = take(pairs * n * r * 4);
    w.dC = take(pairs * n * r * 4);
    w.ybuf = take(pairs * n * r * 4);
    w.tx_part = take(G * chunks * r * dmax * 4);
    w.Yp = take(G * r * s.d_v * 4);
    w.dYp = take(G * r * s.d_v * 4);
    w.db_glue = take(G * r * 4);
    w.colpart = take(pairs * chunks * r * 4);
    w.dc = take(pairs * r * 4);
    w.rho = take(pairs * r * 4);
    w.dg = take(pairs * r * 4);
    w.db_pair = take(pairs * r * 4);
    w.dZ_pair = take(pairs * r * s.d_k * 4);
    w.Zr = take((size_t)s.H * r * s.d_k * 4);
    w.total = off;
    return w;
}

int run_backward(const BwdArgs& a)
{
    return a.s.io_dtype == LOT_BF16 ? run_backward_t<uint16_t>(a) : run_backward_t<float>(a);
}

}  // namespace lot
