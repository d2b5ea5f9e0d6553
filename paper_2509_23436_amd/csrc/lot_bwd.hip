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
// Notation for one solve (token masses a_i: 1/n, or the caller's for cross attention; b = beta):
// W^k = softmax_rows((C + g^{k-1})/eps) is the row-normalised kernel of iteration k,
// c^k_t = sum_i a_i W^k_it the column sums of the plan after the token-side update,
// g^k = g^{k-1} + eps log(b / c^k), and the unit-mass coupling is Ghat_it = W^T_it b_t / c^T_t
// (= Gamma_it / a_i; defined for tokens of mass zero as well).  Reverse sweep, given dGhat:
//   last step:  s_t = sum_i dGhat_it Ghat_it;  dc_t = -s_t / c^T_t;  db_t += s_t / b_t;
//               dW_it = dGhat_it b_t / c^T_t + a_i dc_t
//   step k<T:   (given dg^k)  dc_t = -eps dg^k_t / c^k_t;  db_t += eps dg^k_t / b_t;  dW_it = a_i dc_t
//   both:       e_i = sum_t dW_it W_it;  dY_it = W_it (dW_it - e_i);  dC += dY/eps;
//               dg^{k-1}_t = [k<T] dg^k_t + (1/eps) sum_i dY_it
// with c^k_t = b_t exp((g^{k-1}_t - g^k_t)/eps) read off the stored potentials.
// Glue (O = Ghat1 Y', Y'_t = (1/b_t) sum_j a2_j Ghat2_jt V_j):  dY' = Ghat1^T dO;  dGhat1 = dO Y'^T;
//   dYraw = dY'/b;  db_t -= <dY'_t, Y'_t>/b_t;  dV_j = a2_j sum_t Ghat2_jt dYraw_t;
//   dGhat2_jt = a2_j <V_j, dYraw_t>.
// Finally dQ = dC1 Z, dK = dC2 Z, dZ = sum over the batch of dC1^T Q + dC2^T K.
// The two sides may have different numbers of tokens (cross attention): every step runs per side.
#include "lot_internal.h"
#include "lot_plain_kernels.h"

namespace lot {
namespace {

constexpr int kChunk = kRefChunk;   // tokens per partial column sum
constexpr int kTxChunk = 256;       // tokens per partial r x d contraction (its partial results are r x d each)

// Weight of token i of problem p: its mass, or `uniform` where the masses are implicit.
__device__ inline float row_weight(const float* mass, float uniform, size_t row)
{
    return mass ? mass[row] : uniform;
}

// Ghat[p][i][t] = exp((C_it + g_t)/eps - lse_i), lse from the last token-side update.
__global__ void bwd_unit_couplings(const float* __restrict__ C, const float* __restrict__ lse,
                                   const float* __restrict__ gpot, float* __restrict__ ghat,
                                   size_t total, int n, int r, float eps)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const size_t row = idx / r;
    const int t = (int)(idx % r);
    ghat[idx] = expf((C[idx] + gpot[(row / n) * r + t]) / eps - lse[row]);
}

// part[p][chunk][t][c] = sum over the chunk's tokens i of w_i A[p][i][t] * X[p][i][c]
// (A is fp32 [P][n][r]; X is [P][stride][dx] in the I/O type, n rows used; w = row_weight).
// One block of 256 threads per (p, chunk, tile of kTxPivots pivots): thread = (pivot of the tile,
// column class); a thread walks the chunk's tokens for its pivot and every kTxCols-th column, so that
// a wavefront reads whole stretches of a row of A and of a row of X.
constexpr int kTxPivots = 16, kTxCols = 16;
template <typename T>
__global__ void bwd_tx_partial(const float* __restrict__ A, const T* __restrict__ X, float* __restrict__ part,
                               const float* __restrict__ mass, float uniform,
                               int n, int stride, int r, int dx, int chunks)
{
    const int ttiles = (r + kTxPivots - 1) / kTxPivots;
    const int tt = blockIdx.x % ttiles;
    const int chunk = (blockIdx.x / ttiles) % chunks;
    const size_t p = blockIdx.x / ((size_t)ttiles * chunks);
    const int t = tt * kTxPivots + threadIdx.x / kTxCols, cc = threadIdx.x % kTxCols;
    if (t >= r) return;
    const int i0 = chunk * kTxChunk, i1 = min(n, i0 + kTxChunk);
    for (int c0 = 0; c0 < dx; c0 += 4 * kTxCols) {          // four columns of a thread at a time
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int i = i0; i < i1; ++i) {
            const float a = row_weight(mass, uniform, p * n + i) * A[(p * n + i) * r + t];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = c0 + q * kTxCols + cc;
                if (c < dx) acc[q] = fmaf(a, ld(X, (p * stride + i) * dx + c), acc[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + q * kTxCols + cc;
            if (c < dx) part[((p * chunks + chunk) * r + t) * dx + c] = acc[q];
        }
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

// Mt[p][c][t] = M[p][t][c]: the r x dx matrices that meet token rows are transposed once, so that the
// threads of a wavefront (consecutive pivots t) read consecutive addresses.
__global__ void bwd_transpose(const float* __restrict__ M, float* __restrict__ Mt, size_t total, int r, int dx)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (p, c, t)
    if (idx >= total) return;
    const size_t p = idx / ((size_t)r * dx);
    const int c = (int)(idx / r % dx), t = (int)(idx % r);
    Mt[idx] = M[(p * r + t) * dx + c];
}

// out[p][i][t] = w_i * sum_c X[p][i][c] * Mt[m(p)][c][t]: the similarities C = X Z^T (Mt = Z^T per head,
// w = 1), dGhat1 = dO Y'^T and dGhat2 = a2 V dYraw^T (Mt per problem).
template <typename T>
__global__ void bwd_outer(const T* __restrict__ X, const float* __restrict__ Mt, float* __restrict__ out,
                          const float* __restrict__ mass, float uniform,
                          size_t total, int n, int stride, int r, int dx, int per_head, int H)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (p, i, t)
    if (idx >= total) return;
    const size_t pi = idx / r;
    const int t = (int)(idx % r);
    const size_t p = pi / n;
    const size_t m = per_head ? (p % H) : p;
    float acc = 0.f;
    const size_t row = p * stride + pi % n;          // X is [P][stride][dx]
    for (int c = 0; c < dx; ++c) acc = fmaf(ld(X, row * dx + c), Mt[(m * dx + c) * r + t], acc);
    out[idx] = row_weight(mass, uniform, pi) * acc;
}

// out[p][i][c] = w_i sum_t A[p][i][t] * M[m(p)][t][c], M per problem (per_head = 0) or per head.
template <typename T>
__global__ void bwd_apply(const float* __restrict__ A, const float* __restrict__ M, T* __restrict__ out,
                          const float* __restrict__ mass, float uniform,
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
    st(out, (p * stride + pi % n) * dx + c, row_weight(mass, uniform, pi) * acc);          // out is [P][stride][dx]
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

// Pivot-side bookkeeping of one reverse step, one workgroup of 256 threads per pair.
//   last != 0: colsum holds s_t = sum_i dGhat Ghat  -> dc, rho, db
//   last == 0: dg holds dg^k                         -> dc, db
// c^k_t = beta_t exp((g^{k-1}_t - g^k_t)/eps).
// The potentials are defined up to a common constant, so every dg^k sums to zero over the pivots; the
// step dg^k -> dg^{k-1} leaves the direction c^k unchanged (it is the one eigenvector of that map with
// eigenvalue 1, and it changes no similarity gradient), so whatever rounding puts into the sum would
// stay for all remaining iterations and end up, T times over, in the gradient of the masses.  The sum is
// therefore taken out of dg^k along c^k (sum_t c^k_t = 1) before it is used.
__global__ void __launch_bounds__(256) bwd_pivot_pre(const float* __restrict__ part, const float* __restrict__ g_prev,
                              const float* __restrict__ g_cur, const float* __restrict__ beta,
                              float* __restrict__ dg, float* __restrict__ dc, float* __restrict__ rho,
                              float* __restrict__ db, int G, int H, int r, int chunks, float eps, int last)
{
    __shared__ float s_sum[256];
    const int pair = blockIdx.x;
    const float* bh = beta + ((pair % G) % H) * r;
    float total = 0.f;
    if (!last) {
        float mine = 0.f;
        for (int t = threadIdx.x; t < r; t += 256) mine += dg[(size_t)pair * r + t];
        s_sum[threadIdx.x] = mine;
        __syncthreads();
        for (int half = 128; half > 0; half >>= 1) {
            if ((int)threadIdx.x < half) s_sum[threadIdx.x] += s_sum[threadIdx.x + half];
            __syncthreads();
        }
        total = s_sum[0];
    }
    for (int t = threadIdx.x; t < r; t += 256) {
        const size_t idx = (size_t)pair * r + t;
        const float b = bh[t];
        const float c = b * expf((g_prev[idx] - g_cur[idx]) / eps);
        if (last) {
            float s = 0.f;
            for (int k = 0; k < chunks; ++k) s += part[((size_t)pair * chunks + k) * r + t];
            dc[idx] = -s / c;
            rho[idx] = b / c;
            db[idx] = s / b;          // first contribution of this solve
        } else {
            const float d = dg[idx] - c * total;
            dg[idx] = d;
            dc[idx] = -eps * d / c;
            db[idx] += eps * d / b;
        }
    }
}

// Token side of one reverse step, a group of lanes per (problem, i):
//   W_it = softmax_t((C_it + gprev_t)/eps);  dW_it = [last] dGhat_it rho_t + a_i dc_t;
//   e_i = sum_t dW_it W_it;  dY_it = W_it (dW_it - e_i);  dC_it (+)= dY_it/eps;  Ybuf = dY.
__global__ void bwd_rows(const float* __restrict__ C, const float* __restrict__ g_prev,
                         const float* __restrict__ dGhat, const float* __restrict__ rho,
                         const float* __restrict__ dc, float* __restrict__ dC, float* __restrict__ Ybuf,
                         const float* __restrict__ mass, size_t rows, int n, int r, float eps, int last, int width)
{
    // `width` lanes per row (see row_group_width)
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = tid / width < rows;
    const size_t row = min(tid / width, rows - 1);
    const int sub = (int)(tid % width);
    const size_t pair = row / n;
    const float* c = C + row * r;
    const float* gp = g_prev + pair * r;
    const float* dcp = dc + pair * r;
    const float* rh = rho + pair * r;
    const float a = row_weight(mass, 1.f / (float)n, row);
    float m = -INFINITY;
    for (int t = sub; t < r; t += width) m = fmaxf(m, (c[t] + gp[t]) / eps);
    m = group_max(m, width);
    float s = 0.f;
    for (int t = sub; t < r; t += width) s += expf((c[t] + gp[t]) / eps - m);
    const float inv_s = 1.f / group_sum(s, width);
    float e = 0.f;
    for (int t = sub; t < r; t += width) {
        const float w = expf((c[t] + gp[t]) / eps - m) * inv_s;
        const float dW = (last ? dGhat[row * r + t] * rh[t] : 0.f) + a * dcp[t];
        e = fmaf(dW, w, e);
    }
    e = group_sum(e, width);
    if (!live) return;
    for (int t = sub; t < r; t += width) {
        const float w = expf((c[t] + gp[t]) / eps - m) * inv_s;
        const float dW = (last ? dGhat[row * r + t] * rh[t] : 0.f) + a * dcp[t];
        const float dY = w * (dW - e);
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
    const int G = s.B * s.H, r = s.r, pairs = 2 * G, T_ = a.iters;
    // side 0 = queries (and dO, dQ), side 1 = keys and values
    const int ns[2] = {a.n_q > 0 ? a.n_q : s.n, a.n_k > 0 ? a.n_k : s.n};
    const int strides[2] = {a.n_stride > 0 ? a.n_stride : ns[0], a.n_stride > 0 ? a.n_stride : ns[1]};
    const float* masses[2] = {a.mass_q, a.mass_k};
    const float unis[2] = {1.f / (float)ns[0], 1.f / (float)ns[1]};
    const int chunkss[2] = {(ns[0] + kChunk - 1) / kChunk, (ns[1] + kChunk - 1) / kChunk};
    const int txchunks[2] = {(ns[0] + kTxChunk - 1) / kTxChunk, (ns[1] + kTxChunk - 1) / kTxChunk};
    const void* Xs[2] = {a.Q, a.K};
    void* dXs[2] = {a.dQ, a.dK};
    const BwdWorkspace& L = a.lay;
    const size_t side1 = (size_t)G * ns[0] * r;          // where side 1 starts in the [rows][r] arrays
    float* Cb = (float*)(a.ws + L.C);
    float* lseb = (float*)(a.ws + L.f);
    float* ghatb = (float*)(a.ws + L.gam);
    float* dghatb = (float*)(a.ws + L.dgam);
    float* dCb = (float*)(a.ws + L.dC);
    float* ybufb = (float*)(a.ws + L.ybuf);
    float* Cs[2] = {Cb, Cb + side1};
    float* lses[2] = {lseb, lseb + (size_t)G * ns[0]};
    float* ghats[2] = {ghatb, ghatb + side1};
    float* dghats[2] = {dghatb, dghatb + side1};
    float* dCs[2] = {dCb, dCb + side1};
    float* ybufs[2] = {ybufb, ybufb + side1};
    float* ghist = (float*)(a.ws + L.ghist);       // [T+1][2][G][r]
    float* pm = (float*)(a.ws + L.part_m);
    float* ps = (float*)(a.ws + L.part_s);
    float* tx_part = (float*)(a.ws + L.tx_part);   // [G][chunks][r][dmax]
    float* Yp = (float*)(a.ws + L.Yp);
    float* dYp = (float*)(a.ws + L.dYp);
    float* db_glue = (float*)(a.ws + L.db_glue);
    float* colpart = (float*)(a.ws + L.colpart);
    float* dc = (float*)(a.ws + L.dc);             // [2][G][r], like rho, dg, db_pair
    float* rho = (float*)(a.ws + L.rho);
    float* dg = (float*)(a.ws + L.dg);
    float* db_pair = (float*)(a.ws + L.db_pair);
    float* dZ_pair = (float*)(a.ws + L.dZ_pair);   // [2][G][r][d_k]
    float* Zr = (float*)(a.ws + L.Zr);
    float* Zt = (float*)(a.ws + L.Zt);             // [H][d_k][r]: Z as the forward pass used it, transposed
    float* Yt = (float*)(a.ws + L.Yt);             // [G][d_v][r]: Y' or dYraw, transposed
    hipStream_t st_ = a.stream;
    ref_mark<<<1, 1, 0, st_>>>((unsigned long long*)a.ws, next_nonce());   // no device-side waits on this path
    const size_t slab = (size_t)G * r;                                     // one side's pivot vector
    const unsigned pr_blocks = blocks_for(slab, 256);
    auto pot = [&](int k, int side) { return ghist + ((size_t)k * 2 + side) * slab; };
    const int width = row_group_width(r);
    const int ttiles = (r + kTxPivots - 1) / kTxPivots;

    // ---- forward, keeping the pivot potentials of every iteration and the last row normalisers
    bwd_round_z<<<blocks_for((size_t)s.H * r * s.d_k, 256), 256, 0, st_>>>(a.Z, Zr, s.H * r * s.d_k, s.io_dtype == LOT_BF16);
    bwd_transpose<<<blocks_for((size_t)s.H * r * s.d_k, 256), 256, 0, st_>>>(Zr, Zt, (size_t)s.H * r * s.d_k, r, s.d_k);
    for (int sd = 0; sd < 2; ++sd) {
        const int n = ns[sd], chunks = chunkss[sd];
        const size_t total = (size_t)G * n * r, rows = (size_t)G * n;
        bwd_outer<T><<<blocks_for(total, 256), 256, 0, st_>>>((const T*)Xs[sd], Zt, Cs[sd], nullptr, 1.f, total, n, strides[sd], r,
                                                              s.d_k, 1, s.H);
        ref_zero<<<pr_blocks, 256, 0, st_>>>(pot(0, sd), slab);
        for (int k = 1; k <= T_; ++k) {
            xr_row_lse<<<blocks_for(rows * width, 256), 256, 0, st_>>>(Cs[sd], pot(k - 1, sd), lses[sd], rows, n, r, a.eps, width);
            xr_col_partial<<<(unsigned)G * chunks, 64, 0, st_>>>(Cs[sd], lses[sd], masses[sd], pm, ps, n, r, chunks, a.eps);
            xr_col_final<<<pr_blocks, 256, 0, st_>>>(pm, ps, a.beta, pot(k, sd), G, s.H, r, chunks, a.eps);
        }
        bwd_unit_couplings<<<blocks_for(total, 256), 256, 0, st_>>>(Cs[sd], lses[sd], pot(T_, sd), ghats[sd], total, n, r, a.eps);
    }

    // ---- glue
    const size_t yelems = (size_t)G * r * s.d_v;
    // Y'_t = (1/beta_t) sum_j a2_j Ghat2_jt V_j
    bwd_tx_partial<T><<<(unsigned)((size_t)G * txchunks[1] * ttiles), kTxPivots * kTxCols, 0, st_>>>(ghats[1], (const T*)a.V, tx_part, masses[1], unis[1],
                                                                               ns[1], strides[1], r, s.d_v, txchunks[1]);
    bwd_tx_final<<<blocks_for(yelems, 256), 256, 0, st_>>>(tx_part, Yp, yelems, r, s.d_v, txchunks[1], 1.f);
    bwd_glue_pivots<<<blocks_for((size_t)G * r, 128), 128, 0, st_>>>(Yp, dYp, a.beta, db_glue, G * r, s.H, r, s.d_v, 0);
    // dY' = Ghat1^T dO
    bwd_tx_partial<T><<<(unsigned)((size_t)G * txchunks[0] * ttiles), kTxPivots * kTxCols, 0, st_>>>(ghats[0], (const T*)a.dO, tx_part, nullptr, 1.f,
                                                                               ns[0], strides[0], r, s.d_v, txchunks[0]);
    bwd_tx_final<<<blocks_for(yelems, 256), 256, 0, st_>>>(tx_part, dYp, yelems, r, s.d_v, txchunks[0], 1.f);
    // dGhat1 = dO Y'^T (does not use dY')
    bwd_transpose<<<blocks_for(yelems, 256), 256, 0, st_>>>(Yp, Yt, yelems, r, s.d_v);
    bwd_outer<T><<<blocks_for((size_t)G * ns[0] * r, 256), 256, 0, st_>>>((const T*)a.dO, Yt, dghats[0], nullptr, 1.f,
                                                                          (size_t)G * ns[0] * r, ns[0], strides[0], r, s.d_v, 0, s.H);
    // db_glue, dYraw = dY'/beta
    bwd_glue_pivots<<<blocks_for((size_t)G * r, 128), 128, 0, st_>>>(Yp, dYp, a.beta, db_glue, G * r, s.H, r, s.d_v, 1);
    // dV_j = a2_j sum_t Ghat2_jt dYraw_t ; dGhat2_jt = a2_j <V_j, dYraw_t>
    bwd_apply<T><<<blocks_for((size_t)G * ns[1] * s.d_v, 256), 256, 0, st_>>>(ghats[1], dYp, (T*)a.dV, masses[1], unis[1],
                                                                              (size_t)G * ns[1] * s.d_v, ns[1], strides[1], r, s.d_v, 0, s.H);
    bwd_transpose<<<blocks_for(yelems, 256), 256, 0, st_>>>(dYp, Yt, yelems, r, s.d_v);
    bwd_outer<T><<<blocks_for((size_t)G * ns[1] * r, 256), 256, 0, st_>>>((const T*)a.V, Yt, dghats[1], masses[1], unis[1],
                                                                          (size_t)G * ns[1] * r, ns[1], strides[1], r, s.d_v, 0, s.H);

    // ---- both Sinkhorn solves, reverse sweep
    for (int sd = 0; sd < 2; ++sd) {
        const int n = ns[sd], chunks = chunkss[sd];
        const size_t rows = (size_t)G * n;
        float* dc_s = dc + sd * slab; float* rho_s = rho + sd * slab; float* dg_s = dg + sd * slab;
        float* db_s = db_pair + sd * slab;
        bwd_col_partial<<<(unsigned)G * chunks, 64, 0, st_>>>(dghats[sd], ghats[sd], colpart, n, r, chunks);
        for (int k = T_; k >= 1; --k) {
            const int last = k == T_;
            bwd_pivot_pre<<<(unsigned)G, 256, 0, st_>>>(colpart, pot(k - 1, sd), pot(k, sd), a.beta, dg_s, dc_s, rho_s, db_s, G, s.H, r,
                                                        chunks, a.eps, last);
            bwd_rows<<<blocks_for(rows * width, 256), 256, 0, st_>>>(Cs[sd], pot(k - 1, sd), dghats[sd], rho_s, dc_s, dCs[sd],
                                                                     ybufs[sd], masses[sd], rows, n, r, a.eps, last, width);
            bwd_col_partial<<<(unsigned)G * chunks, 64, 0, st_>>>(ybufs[sd], nullptr, colpart, n, r, chunks);
            bwd_pivot_post<<<pr_blocks, 256, 0, st_>>>(colpart, dg_s, G, r, chunks, a.eps, last);
        }
        // similarities: dX = dC Z, dZ share = dC^T X
        bwd_apply<T><<<blocks_for(rows * s.d_k, 256), 256, 0, st_>>>(dCs[sd], Zr, (T*)dXs[sd], nullptr, 1.f, rows * s.d_k, n, strides[sd],
                                                                     r, s.d_k, 1, s.H);
        bwd_tx_partial<T><<<(unsigned)((size_t)G * txchunks[sd] * ttiles), kTxPivots * kTxCols, 0, st_>>>(dCs[sd], (const T*)Xs[sd], tx_part, nullptr, 1.f, n,
                                                                                    strides[sd], r, s.d_k, txchunks[sd]);
        bwd_tx_final<<<blocks_for((size_t)G * r * s.d_k, 256), 256, 0, st_>>>(tx_part, dZ_pair + (size_t)sd * G * r * s.d_k,
                                                                              (size_t)G * r * s.d_k, r, s.d_k, txchunks[sd], 1.f);
    }
    bwd_head_sums<<<blocks_for((size_t)s.H * r * (s.d_k + 1), 256), 256, 0, st_>>>(dZ_pair, db_pair, db_glue, a.dZ, a.dbeta, s.B, s.H, r, s.d_k);
    (void)pairs;
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

}  // namespace

BwdWorkspace carve_bwd_sides(int B, int H, int n_q, int n_k, int r, int d_k, int d_v, int iters)
{
    BwdWorkspace w{};
    size_t off = 256;      // the status words come first, as in the other workspaces
    auto take = [&](size_t bytes) { size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
    const size_t G = (size_t)B * H, rows = G * ((size_t)n_q + n_k), pairs = 2 * G;
    const size_t nmax = n_q > n_k ? n_q : n_k;
    const size_t chunks = (nmax + kRefChunk - 1) / kRefChunk;
    const size_t txchunks = (nmax + kTxChunk - 1) / kTxChunk;
    const size_t dmax = d_k > d_v ? d_k : d_v;
    w.C = take(rows * r * 4);
    w.f = take(rows * 4);
    w.ghist = take((size_t)(iters + 1) * pairs * r * 4);
    w.part_m = take(G * chunks * r * 4);
    w.part_s = take(G * chunks * r * 4);
    w.gam = take(rows * r * 4);
    w.dgam = take(rows * r * 4);
    w.dC = take(rows * r * 4);
    w.ybuf = take(rows * r * 4);
    w.tx_part = take(G * txchunks * r * dmax * 4);
    w.Yp = take(G * r * d_v * 4);
    w.dYp = take(G * r * d_v * 4);
    w.db_glue = take(G * r * 4);
    w.colpart = take(G * chunks * r * 4);
    w.dc = take(pairs * r * 4);
    w.rho = take(pairs * r * 4);
    w.dg = take(pairs * r * 4);
    w.db_pair = take(pairs * r * 4);
    w.dZ_pair = take(pairs * r * d_k * 4);
    w.Zr = take((size_t)H * r * d_k * 4);
    w.Zt = take((size_t)H * r * d_k * 4);
    w.Yt = take(G * r * d_v * 4);
    w.total = off;
    return w;
}

BwdWorkspace carve_bwd(const lot_shape& s, int iters)
{
    return carve_bwd_sides(s.B, s.H, s.n, s.n, s.r, s.d_k, s.d_v, iters);
}

int run_backward(const BwdArgs& a)
{
    return a.s.io_dtype == LOT_BF16 ? run_backward_t<uint16_t>(a) : run_backward_t<float>(a);
}

}  // namespace lot
