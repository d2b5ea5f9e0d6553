// Backward pass of LOT attention for pivot sizes beyond one register tile: 64 < r <= 256, d_k = d_v in
// {32, 64}; per-side token counts and token masses as in cross attention.  Same gradients as the other
// backward paths; nothing of size n x r is written.  The pivots are taken in groups of 64, as in the
// forward pass for these sizes.
//
// Notation as in the tiled backward path: per solve, W^k_it = softmax_t((C_it + g^{k-1}_t)/eps) is the
// row-normalised kernel of iteration k, cs^k_t = sum_i W^k_it, c^k = a cs^k (a = 1/n), dc^k the adjoint of
// c^k, dg^k that of the pivot potentials, dc^k = -eps dg^k / c^k.  With
//       dP^k_it = dc^k_t (k < T),   dP^T_it = n rho'_t dGamma_it + dc^T_t   (rho'_t = beta_t / cs^T_t),
//       e^k_i   = sum_t W^k_it dP^k_it,
// the reverse recursion is  dg^{k-1}_t = -(a/eps) sum_i W^k_it e^k_i  and the gradient of the similarities is
// dC_it = (a/eps) sum_k W^k_it (dP^k_it - e^k_i).  With r x r Gram matrices of 256 x 256 out of reach of a
// workgroup's registers, the recursion is run matrix-free: one pass over the tokens per iteration (a row
// reduction e^k_i, then a column reduction), T passes in sequence.  Per token and iteration two numbers
// are kept, the base-2 row log-normaliser L^k_i (written by the forward passes) and e^k_i, so that every
// later kernel rebuilds W^k_it = exp2((C_it + g^{k-1}_t) c1 - L^k_i) with one exponential and without a
// reduction over the groups.  With token masses (m_i = n a_i, 1 if uniform): cs^k_t = sum_i m_i W^k_it,
// dP^k_it = m_i dc^k_t, and on the key side dGamma, the contraction with V and the rows of dV carry m_j.
// (Paper, "Learning": everything is trained by backpropagating through both Sinkhorn problems and the
// glued composition; its runtime study sweeps r up to 256.  The derivation is this file's.)
//
// Launches (launch boundaries are the only synchronisation between workgroups; both solves share every
// launch, pair = side * G + g, side 0 = queries):
//   clear | T x pass (column sums, L^k) | contract (U = sum W2 V, Wd = sum W1 dO, a workgroup per group) |
//   mid (Y', dYraw, rho') | expand (dV) | glue (s, n q_i) | T x recursion pass (k = T..1: dc^k from the
//   partial sums of the pass before, e^k_i, column sums of W^k e^k) | assemble-x (dQ, dK) |
//   assemble-z (dZ partials, a workgroup per group) | final (dZ, dbeta).
// Every reduction has a fixed order except the forward column sums, which are exchanged as integers:
// results are reproducible.
#include <mutex>
#include "lot_internal.h"
#include "lot_tile.h"
#include "lot_tile_ops.h"
#include "lot_plain_kernels.h"
#include "lot_grouped_ops.h"

namespace lot {
namespace {

struct GbParams {
    LgParams f;                   // inputs, potentials and column sums as the forward passes use them
    const void* dO;
    void* dQ; void* dK; void* dV;
    float* dZ; float* dbeta;
    float* erow;                  // [T][pairs][n]  e^k_i at k - 1 (the glue leaves n q_i at T - 1)
    float* u_part;                // [pairs][chunks][256][D]  side 1: sum W2 V, side 0: sum W1 dO
    float* yp;                    // [G][256][D]  Y'
    float* dyraw;                 // [G][256][D]  dY' / beta
    float* ydv;                   // [G][256][D]  rho'_t dYraw_t (keys)
    float* rhop;                  // [pairs][256]  beta_t / cs^T_t
    float* s_part;                // [pairs][chunks][256]  s_t = sum_i dGamma_it Gamma_it
    float* dg_part;               // [T][pairs][chunks][256]  sum_i W^k_it e^k_i at k - 1
    float* dcs;                   // [T][pairs][256]  dc^k at k - 1
    float* gmax;                  // [T][pairs]  max_t g^{k-1}_t at k - 1
    float* db_pair;               // [pairs][256]
    float* db_glue;               // [G][256]
    float* dz_part;               // [pairs][chunks][256][D]
    float* x_part;                // [pairs][n][D]: partial dQ / dK rows between launches of the assemble-x kernel (if several)
    int B;
};

// Mass of a token times the number of tokens of its side (1 for uniform masses).
__device__ __forceinline__ float gb_token_weight(const GbParams& p, int side, int g, int tok)
{
    const float* m = p.f.mass_side[side];
    return m ? (float)p.f.n_side[side] * m[(size_t)g * p.f.n_side[side] + tok] : 1.f;
}

__device__ __forceinline__ float gb_colsum(const GbParams& p, int k, int pair, int t)
{
    const unsigned long long word = p.f.colacc[((size_t)k * 2 * p.f.G + pair) * kRmax + t];
    return fmaxf((float)(long long)word * p.f.fx_unscale, 0.5f * p.f.fx_unscale);
}

// Pivot fragments of one group to an LDS stash (one wavefront).
template <typename IO, int D>
__device__ __forceinline__ void stash_group_pivots(char* zstash, const float* Z, int h, int r, int grp, int lane)
{
    const int i = lane & 31, kg = lane >> 5;
    Frag<IO, D> z0[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const int t = kGroup * grp + 32 * mb + i;
        load_pivots<D>(z0[mb], Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
    }
    stash_pivots<D, 2>(zstash, z0, lane);
}

// 64 rows of a [256][D] matrix (times scale) as the "pivot" operand of the similarity MFMA, via LDS
// staging: hi part, and for bf16 I/O the part the bf16 rounding leaves out.  Contains barriers.
template <typename IO, int D>
__device__ __forceinline__ void stash_matrix_rows(char* hi, char* lo, float* s_y, const float* rows, float scale,
                                                  int tid, int wave, int lane)
{
    constexpr bool kSplit = io_is_f32<IO>::value;
    const int i = lane & 31, kg = lane >> 5;
    __syncthreads();
    for (int e = tid; e < kGroup * D; e += kThreads) s_y[e] = rows[e] * scale;
    __syncthreads();
    if (wave == 0) {
        Frag<IO, D> y0[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) load_pivots_lds<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
        stash_pivots<D, 2>(hi, y0, lane);
        if (!kSplit) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) load_pivots_lds_lo<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
            stash_pivots<D, 2>(lo, y0, lane);
        }
    }
}

// The incoming gradient of the coupling for one group: dGamma_it = <value row i, matrix row t>.
template <typename IO, int D>
__device__ __forceinline__ void coupling_gradient(f32x16 (&dgam)[2], const char* yhi, const char* ylo,
                                                  const Frag<IO, D>& vc, int lane)
{
    constexpr bool kSplit = io_is_f32<IO>::value;
    int skew = 0;
    asm volatile("" : "+v"(skew));
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) dgam[mb][j] = 0.f;
    Frag<IO, D> yfrag[2];
    fetch_pivots<D, 2>(yfrag, yhi, lane, skew);
    similarity<D, 2>(dgam, yfrag, vc);
    if (!kSplit) {
        fetch_pivots<D, 2>(yfrag, ylo, lane, skew);
        similarity<D, 2>(dgam, yfrag, vc);
    }
}

// ---------------------------------------------------------------------------------------------
// contract: per (pair, chunk, group) U_t = sum_i W^T_it value_i  (values: V for the keys, dO for the queries)
// ---------------------------------------------------------------------------------------------
template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) gb_contract(GbParams p)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    __shared__ float s_g[kGroup];
    __shared__ __attribute__((aligned(16))) float s_buf[64 * D];
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[kWaves * 2 * 64 * kTrStride];
    __shared__ __attribute__((aligned(16))) char s_zstash[StashBytes<IO, D, 2>::value];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.f.G, T = p.f.T;
    int wg, grp;
    if (!group_block(wg, grp, pairs * p.f.chunks, p.f.groups)) return;
    const int pair = wg / p.f.chunks, chunk = wg % p.f.chunks;
    const int side = pair / p.f.G, g = pair % p.f.G, h = g % p.f.H;
    const int n = p.f.n_side[side];        // tokens of this side (p.f.n, the longer side, strides the per-token arrays)
    const float c1 = kLog2e / p.f.eps;
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.f.Q : p.f.K);
    const IO* vals = reinterpret_cast<const IO*>(side == 0 ? p.dO : p.f.V);
    const float* lse = p.f.rowlse + ((size_t)(T - 1) * pairs + pair) * p.f.n;
    uint16_t* tr_hi = s_tr + (wave * 2 + 0) * 64 * kTrStride;
    uint16_t* tr_lo = s_tr + (wave * 2 + 1) * 64 * kTrStride;
    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.f.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.f.tiles_per_wg);

    if (tid < kGroup) s_g[tid] = p.f.ghist[((size_t)(T - 1) * pairs + pair) * kRmax + kGroup * grp + tid];
    if (wave == 0) stash_group_pivots<IO, D>(s_zstash, p.f.Z, h, p.f.r, grp, lane);
    __syncthreads();

    f32x16 U[2][NB];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 16; ++j) U[mb][nb][j] = 0.f;
    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        const int tok = min(tile * kTileTokens + i, n - 1);
        const float L = tile * kTileTokens + i < n ? lse[tok] : INFINITY;
        Frag<IO, D> xc;
        load_tokens<D>(xc, X + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        bf16x8 vh[2][NB], vl[2][NB];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
            const int left = max(1, min(8, n - t0));
            load_values<D>(vh[s], vl[s], vals, (size_t)g * p.f.stride_side[side] + min(t0, n - 1), left, i);
        }
        f32x16 acc[2];
        weights_from_lse<IO, D>(acc, s_zstash, s_g, xc, L, lane, kg, c1);
        if (side == 1 && p.f.mass_side[1]) {      // the keys' masses weight their contraction with V
            const float mt = gb_token_weight(p, 1, g, tok);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[mb][j] *= mt;
        }
        transpose_tile<2, kSplit>(acc, tr_hi, tr_lo, i, kg);
        contract_tokens<D, 2, kSplit>(U, tr_hi, tr_lo, vh, vl, i, kg);
        transpose_done();
    }
    sum_over_waves<D, 2>(U, s_buf, wave, i, kg);
    float* up = p.u_part + (((size_t)pair * p.f.chunks + chunk) * kRmax + (size_t)kGroup * grp) * D;
    for (int e = tid; e < kGroup * D; e += kThreads) up[e] = s_buf[e];
}

// ---------------------------------------------------------------------------------------------
// mid: Y'_t = U_t / cs2_t, dYraw_t = n Wd_t / cs1_t, db_glue_t = -<dYraw_t, Y'_t>, rho'_t = beta_t / cs_t,
// and rho'2_t dYraw_t for the expansion to dV.  One thread per (g, t, column); the D threads of a row
// are adjacent lanes of one wavefront.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ void gb_mid(GbParams p)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;      // the grid covers G * 256 * D exactly
    const int g = idx / (kRmax * D), e = idx % (kRmax * D), t = e / D;
    const int G = p.f.G, T = p.f.T, chunks = p.f.chunks;
    float y = 0.f, dy = 0.f, r1 = 0.f, r2 = 0.f;
    if (t < p.f.r) {
        float u0 = 0.f, u1 = 0.f, w0 = 0.f, w1 = 0.f;
        const float* wp = p.u_part + ((size_t)(0 * G + g) * chunks) * kRmax * D + e;
        const float* up = p.u_part + ((size_t)(1 * G + g) * chunks) * kRmax * D + e;
        int c = 0;
        for (; c + 1 < chunks; c += 2) {
            w0 += wp[(size_t)c * kRmax * D]; w1 += wp[(size_t)(c + 1) * kRmax * D];
            u0 += up[(size_t)c * kRmax * D]; u1 += up[(size_t)(c + 1) * kRmax * D];
        }
        if (c < chunks) { w0 += wp[(size_t)c * kRmax * D]; u0 += up[(size_t)c * kRmax * D]; }
        const float cs1 = gb_colsum(p, T, g, t), cs2 = gb_colsum(p, T, G + g, t);
        y = (u0 + u1) / cs2;
        dy = (float)p.f.n_side[0] * (w0 + w1) / cs1;
        const float b = p.f.beta[(g % p.f.H) * p.f.r + t];
        r1 = b / cs1;
        r2 = b / cs2;
    }
    p.yp[idx] = y;
    p.dyraw[idx] = dy;
    p.ydv[idx] = r2 * dy;
    float dot = dy * y;
#pragma unroll
    for (int o = D / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
    if (e % D == 0) {
        p.db_glue[g * kRmax + t] = -dot;
        p.rhop[(size_t)g * kRmax + t] = r1;
        p.rhop[(size_t)(G + g) * kRmax + t] = r2;
    }
}

// ---------------------------------------------------------------------------------------------
// glue: s_t = rho'_t sum_i W_it dGamma_it (per-workgroup partial sums) and n q_i = n sum_t W_it rho'_t dGamma_it
// (into erow at T - 1), both solves.
// ---------------------------------------------------------------------------------------------
// (kGlueWaves wavefronts per workgroup: the stashes fill most of a compute unit's local memory, so a
// second wavefront per SIMD has to come from the same workgroup; worth it when a workgroup has many tiles)
template <typename IO, int D, int kGlueWaves>
__global__ void __launch_bounds__(64 * kGlueWaves) gb_glue(GbParams p)
{
    constexpr int kStash = StashBytes<IO, D, 2>::value;
    __shared__ float s_g[kRmax], s_rho[kRmax];
    __shared__ float s_cs[kGlueWaves][kRmax];
    __shared__ __attribute__((aligned(16))) float s_y[64 * D];
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];   // pivot stash | matrix stash hi | (bf16 I/O) lo, per group

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.f.G, T = p.f.T, groups = p.f.groups;
    const int pair = blockIdx.x / p.f.chunks, chunk = blockIdx.x % p.f.chunks;
    const int side = pair / p.f.G, g = pair % p.f.G, h = g % p.f.H;
    const int n = p.f.n_side[side];        // tokens of this side (p.f.n, the longer side, strides the per-token arrays)
    const float c1 = kLog2e / p.f.eps;
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.f.Q : p.f.K);
    const IO* vals = reinterpret_cast<const IO*>(side == 0 ? p.dO : p.f.V);
    // the matrix whose rows meet the value rows: n Y' for the queries, dYraw for the keys
    const float* ymat = (side == 0 ? p.yp : p.dyraw) + (size_t)g * kRmax * D;
    const float yscale = side == 0 ? (float)n : 1.f;
    const float* lse = p.f.rowlse + ((size_t)(T - 1) * pairs + pair) * p.f.n;
    float* erow = p.erow + ((size_t)(T - 1) * pairs + pair) * p.f.n;
    char* s_zstash = s_dyn;
    char* s_yhi = s_dyn + (size_t)groups * kStash;
    char* s_ylo = s_yhi + (size_t)groups * kStash;

    for (int t = tid; t < kRmax; t += kThreads) {
        s_g[t] = p.f.ghist[((size_t)(T - 1) * pairs + pair) * kRmax + t];
        s_rho[t] = p.rhop[(size_t)pair * kRmax + t];
    }
    stash_all_pivots<IO, D>(s_zstash, p.f.Z, h, p.f.r, groups, wave, lane);
    for (int q = 0; q < groups; ++q)
        stash_matrix_rows<IO, D>(s_yhi + (size_t)q * kStash, s_ylo + (size_t)q * kStash, s_y,
                                 ymat + (size_t)kGroup * q * D, yscale, tid, wave, lane);
    __syncthreads();

    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.f.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.f.tiles_per_wg);
    float sg[kMaxGroups] = {0.f, 0.f, 0.f, 0.f};       // this lane's pivot of each group
    for (int tile = tile_begin + wave; tile < tile_end; tile += kGlueWaves) {
        const bool valid = tile * kTileTokens + i < n;
        const int tok = min(tile * kTileTokens + i, n - 1);
        const float L = valid ? lse[tok] : INFINITY;
        Frag<IO, D> xc, vc;
        load_tokens<D>(xc, X + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        load_tokens<D>(vc, vals + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        float q0 = 0.f, q1 = 0.f;
        const float mk = side == 1 ? gb_token_weight(p, 1, g, tok) : 1.f;
#pragma unroll
        for (int q = 0; q < kMaxGroups; ++q) {
            if (q < groups) {
                f32x16 acc[2], dgam[2], rho[2];
                weights_from_lse<IO, D>(acc, s_zstash + (size_t)q * kStash, s_g + kGroup * q, xc, L, lane, kg, c1);
                coupling_gradient<IO, D>(dgam, s_yhi + (size_t)q * kStash, s_ylo + (size_t)q * kStash, vc, lane);
                load_pivot_vector<2>(rho, s_rho + kGroup * q, kg);
                float c[32];
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 2) {
                        // (mk: the key's mass times n_k, 1 for queries: dGamma2 carries the keys' masses)
                        const float a0 = acc[mb][j] * dgam[mb][j] * mk, a1 = acc[mb][j + 1] * dgam[mb][j + 1] * mk;
                        c[16 * mb + j] = a0; c[16 * mb + j + 1] = a1;
                        q0 = fmaf(a0, rho[mb][j], q0);
                        q1 = fmaf(a1, rho[mb][j + 1], q1);
                    }
                sg[q] += reduce_scatter_tokens<32>(c, i);
            }
        }
        const float qi = pair_sum(q0 + q1);
        if (valid && kg == 0) erow[tok] = (float)n * qi;
    }
    const int mine = 32 * (i >> 4) + 8 * ((i & 15) >> 2) + 4 * kg + (i & 3);
#pragma unroll
    for (int q = 0; q < kMaxGroups; ++q) s_cs[wave][kGroup * q + mine] = sg[q];
    __syncthreads();
    for (int t = tid; t < kRmax; t += 64 * kGlueWaves) {
        float tot = 0.f;
#pragma unroll
        for (int wv = 0; wv < kGlueWaves; ++wv) tot += s_cs[wv][t];
        p.s_part[((size_t)pair * p.f.chunks + chunk) * kRmax + t] = t < p.f.r ? tot * s_rho[t] : 0.f;
    }
}

// ---------------------------------------------------------------------------------------------
// recursion pass k (k = T .. 1): dc^k from the partial sums of the launch before (every workgroup of a
// pair computes the same numbers; the first writes them out), then per tile e^k_i and, for k > 1, the
// column sums of W^k e^k that give dg^{k-1}.
// ---------------------------------------------------------------------------------------------
template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) gb_rec_pass(GbParams p, int k)
{
    constexpr int kStash = StashBytes<IO, D, 2>::value;
    __shared__ float s_g[kRmax], s_dc[kRmax];
    __shared__ float s_cs[kWaves][kRmax];
    extern __shared__ __attribute__((aligned(16))) char s_zstash[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.f.G, T = p.f.T, groups = p.f.groups, chunks = p.f.chunks;
    const int pair = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
    const int side = pair / p.f.G, g = pair % p.f.G, h = g % p.f.H;
    const int n = p.f.n_side[side];        // tokens of this side (p.f.n, the longer side, strides the per-token arrays)
    const float c1 = kLog2e / p.f.eps, a = 1.f / (float)n;
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.f.Q : p.f.K);
    const float* lse = p.f.rowlse + ((size_t)(k - 1) * pairs + pair) * p.f.n;
    float* erow = p.erow + ((size_t)(k - 1) * pairs + pair) * p.f.n;

    static_assert(kThreads == kRmax, "one thread per pivot in the prologue");
    {
        const int t = tid;
        const bool live = t < p.f.r;
        float dc = 0.f;
        float dg = 0.f;
        if (live && k < T) {
            float acc = 0.f;
            for (int c = 0; c < chunks; ++c) acc += p.dg_part[(((size_t)k * pairs + pair) * chunks + c) * kRmax + t];
            dg = -(a / p.f.eps) * acc;                  // dg^k
        }
        // The potentials are defined up to a common constant, so dg^k sums to zero over the pivots, and the
        // step to dg^{k-1} leaves the direction c^k unchanged (it changes no similarity gradient): what
        // rounding puts into that sum would stay for all remaining iterations and end up, T times over, in
        // the gradient of the masses.  It is taken out along c^k (sum_t c^k_t = 1).  Fixed order of additions.
        float dg_total = 0.f;
        if (k < T) {
            float v = dg;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            if (lane == 0) s_cs[1][wave] = v;
            __syncthreads();
            dg_total = (s_cs[1][0] + s_cs[1][1]) + (s_cs[1][2] + s_cs[1][3]);
            __syncthreads();
        }
        if (live) {
            const float b = p.f.beta[h * p.f.r + t];
            const float ck = gb_colsum(p, k, pair, t) * a;
            float db_add;
            if (k == T) {
                float s = 0.f;
                for (int c = 0; c < chunks; ++c) s += p.s_part[((size_t)pair * chunks + c) * kRmax + t];
                dc = -s / ck;
                db_add = s / b;
            } else {
                dg -= ck * dg_total;
                dc = -p.f.eps * dg / ck;
                db_add = p.f.eps * dg / b;
            }
            // dbeta's share of this pair: only the first workgroup touches it (read in one launch, written in the next)
            if (chunk == 0) p.db_pair[(size_t)pair * kRmax + t] = (k == T ? 0.f : p.db_pair[(size_t)pair * kRmax + t]) + db_add;
        } else if (chunk == 0) {
            p.db_pair[(size_t)pair * kRmax + t] = 0.f;
        }
        s_dc[t] = dc;
        if (chunk == 0) p.dcs[((size_t)(k - 1) * pairs + pair) * kRmax + t] = dc;
        const float gv = p.f.ghist[((size_t)(k - 1) * pairs + pair) * kRmax + t];
        s_g[t] = gv;
        // the largest potential of this iteration: the assembly scales its per-pivot factors by it
        float gm = live ? gv : -INFINITY;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) gm = fmaxf(gm, __shfl_xor(gm, o, 64));
        if (lane == 0) s_cs[0][wave] = gm;
        __syncthreads();
        if (chunk == 0 && tid == 0)
            p.gmax[(size_t)(k - 1) * pairs + pair] = fmaxf(fmaxf(s_cs[0][0], s_cs[0][1]), fmaxf(s_cs[0][2], s_cs[0][3]));
    }
    stash_all_pivots<IO, D>(s_zstash, p.f.Z, h, p.f.r, groups, wave, lane);
    __syncthreads();

    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.f.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.f.tiles_per_wg);
    float csg[kMaxGroups] = {0.f, 0.f, 0.f, 0.f};
    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        const bool valid = tile * kTileTokens + i < n;
        const int tok = min(tile * kTileTokens + i, n - 1);
        const float L = valid ? lse[tok] : INFINITY;
        const float e_in = k == T ? erow[tok] : 0.f;         // n q_i from the glue
        Frag<IO, D> xc;
        load_tokens<D>(xc, X + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        f32x16 wt[kMaxGroups][2];
        float y0 = 0.f, y1 = 0.f;
#pragma unroll
        for (int q = 0; q < kMaxGroups; ++q) {
            if (q < groups) {
                f32x16 dcv[2];
                weights_from_lse<IO, D>(wt[q], s_zstash + (size_t)q * kStash, s_g + kGroup * q, xc, L, lane, kg, c1);
                load_pivot_vector<2>(dcv, s_dc + kGroup * q, kg);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 2) {
                        y0 = fmaf(wt[q][mb][j], dcv[mb][j], y0);
                        y1 = fmaf(wt[q][mb][j + 1], dcv[mb][j + 1], y1);
                    }
            }
        }
        const float e = gb_token_weight(p, side, g, tok) * pair_sum(y0 + y1) + e_in;    // dP^k_it = m_i dc^k_t (+ the glue's part)
        if (valid && kg == 0) erow[tok] = e;
        if (k > 1) {
#pragma unroll
            for (int q = 0; q < kMaxGroups; ++q) {
                if (q < groups) {
                    float c[32];
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                        for (int j = 0; j < 16; ++j) c[16 * mb + j] = wt[q][mb][j] * e;
                    csg[q] += reduce_scatter_tokens<32>(c, i);
                }
            }
        }
    }
    if (k > 1) {
        const int mine = 32 * (i >> 4) + 8 * ((i & 15) >> 2) + 4 * kg + (i & 3);
#pragma unroll
        for (int q = 0; q < kMaxGroups; ++q) s_cs[wave][kGroup * q + mine] = csg[q];
        __syncthreads();
        for (int t = tid; t < kRmax; t += kThreads) {
            float tot = 0.f;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) tot += s_cs[wv][t];
            p.dg_part[(((size_t)(k - 1) * pairs + pair) * chunks + chunk) * kRmax + t] = tot;
        }
    }
}

// The gradient of the similarities for one tile and one group, summed over the iterations:
// dacc_it = (a/eps) sum_k W^k_it (dP^k_it - e^k_i).  One exponential per element, not one per iteration:
// with m_i the row's largest scaled similarity in this group and h_k the largest scaled potential of
// iteration k,  W^k_it = E_it P^k_t R^k_i,  E_it = exp2(C_it c1 - m_i),  P^k_t = exp2(g^{k-1}_t c1 - h_k),
// R^k_i = exp2(m_i + h_k - L^k_i)  (E, P <= 1; R is capped at 2^60: beyond that the row's weights in this
// group are below 2^-60 of the bound anyway), so that
//   dacc_it = (a/eps) E_it [ sum_k R^k_i A^k_t - sum_k (R^k_i e^k_i) P^k_t + R^T_i B_t dGamma_it ],
// A^k = P^k dc^k, B = n rho' P^T.
// tab: [T][2][64] for this group, (P^k, A^k) at k - 1; bvec: B for this group; shifts: h_k at k - 1.
template <typename IO, int D>
__device__ __forceinline__ void similarity_gradient(f32x16 (&dacc)[2], const char* zst, const char* yhi, const char* ylo,
                                                    const float* tab, const float* bvec, const float* shifts,
                                                    const Frag<IO, D>& xc, const Frag<IO, D>& vc,
                                                    const float* lse, const float* erow, size_t per_k, int tok, bool valid,
                                                    float m_tok, float m_key, int T, float c1, float scale_out, int lane, int kg)
{
    int skew = 0;
    asm volatile("" : "+v"(skew));
    f32x16 E[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) E[mb][j] = 0.f;
    {
        Frag<IO, D> zf[2];
        fetch_pivots<D, 2>(zf, zst, lane, skew);
        similarity<D, 2>(E, zf, xc);
    }
    float m0 = -INFINITY, m1 = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; j += 2) {
            m0 = fmaxf(m0, E[mb][j]);
            m1 = fmaxf(m1, E[mb][j + 1]);
        }
    const float m = pair_max(fmaxf(m0, m1)) * c1;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) E[mb][j] = exp2_fast(fmaf(E[mb][j], c1, -m));
    // row factors: R^k_i (0 for a row past the end) and R^k_i e^k_i
    auto row_factors = [&](int k, float& R, float& S) {
        const float L = valid ? lse[(size_t)(k - 1) * per_k + tok] : INFINITY;
        R = exp2_fast(fminf(m + shifts[k - 1] - L, 60.f));
        S = R * erow[(size_t)(k - 1) * per_k + tok];
    };
    // sum_k R^k_i A^k_t - S^k_i P^k_t: a (64 x 2T) by (2T x 32) product on the fp32 matrix cores, two table rows
    // per instruction (this lane supplies row 2 (k - 1) + kg of the table and the matching row factor)
    const int i = lane & 31;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) dacc[mb][j] = 0.f;
    float r_last = 0.f;
    for (int k = 1; k <= T; ++k) {
        float R, S;
        row_factors(k, R, S);
        r_last = R;
        const float b = kg ? R * m_tok : -S;        // dP^k_it = m_i dc^k_t
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const float a = tab[((k - 1) * 2 + kg) * kGroup + 32 * mb + i + skew];
            dacc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, dacc[mb], 0, 0, 0);
        }
    }
    // last iteration: dP^T = n rho' dGamma + dc^T
    {
        f32x16 dgam[2], bv[2];
        coupling_gradient<IO, D>(dgam, yhi, ylo, vc, lane);
        load_pivot_vector<2>(bv, bvec + skew, kg);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j)
                dacc[mb][j] = E[mb][j] * scale_out * fmaf(r_last * m_key * bv[mb][j], dgam[mb][j], dacc[mb][j]);
    }
}

// Per-pivot tables of the assembly for the pivots [t0, t0 + 64): (P^k, A^k) for all k into tab ([T][2][64])
// and B into bvec.
__device__ __forceinline__ void load_tables(float* tab, float* bvec, const GbParams& p, int pair, int t0, float c1, int tid)
{
    const int pairs = 2 * p.f.G, T = p.f.T;
    for (int e = tid; e < T * kGroup; e += kThreads) {
        const int k = e / kGroup + 1, t = e % kGroup;
        const float h = p.gmax[(size_t)(k - 1) * pairs + pair] * c1;
        const float P = exp2_fast(p.f.ghist[((size_t)(k - 1) * pairs + pair) * kRmax + t0 + t] * c1 - h);   // padding: 0
        tab[((k - 1) * 2 + 0) * kGroup + t] = P;
        tab[((k - 1) * 2 + 1) * kGroup + t] = P * p.dcs[((size_t)(k - 1) * pairs + pair) * kRmax + t0 + t];
        if (k == T) bvec[t] = P * (float)p.f.n_side[pair / p.f.G] * p.rhop[(size_t)pair * kRmax + t0 + t];
    }
}

// ---------------------------------------------------------------------------------------------
// assemble-x: dQ / dK rows = dC Z, summed over the groups in order
// ---------------------------------------------------------------------------------------------
// (WAVES wavefronts per workgroup: the tables fill most of a compute unit's local memory, so a second
// wavefront per SIMD has to come from the same workgroup)
// Where the tables of all groups do not fit a workgroup's local memory together, the kernel is launched
// once per run of `nq` consecutive groups (from group q0): every launch but the last leaves its partial
// rows, in fp32, in `partial` [pair][token][D], and every launch but the first starts from them.
template <typename IO, int D, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) gb_assemble_x(GbParams p, int stage_bytes, int q0, int nq, float* partial,
                                                            int first, int last)
{
    constexpr int NB = D / 32;
    constexpr int kStash = StashBytes<IO, D, 2>::value;
    constexpr bool kSplit = io_is_f32<IO>::value;
    constexpr int kFragsPerGroup = 2 * 2 * NB * 64;
    constexpr int kParts = kSplit ? 2 : 1;
    __shared__ float s_bvec[kRmax], s_shift[64];
    // staging area (a [64][D] matrix during set-up, then the tables [groups][T][2][64]) | pivot stash |
    // matrix stash hi | (bf16 I/O) lo | Z as B fragments hi | (fp32 I/O) lo
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.f.G, T = p.f.T, groups = nq;   // (the groups of this launch)
    const int pair = blockIdx.x / p.f.chunks, chunk = blockIdx.x % p.f.chunks;
    const int side = pair / p.f.G, g = pair % p.f.G, h = g % p.f.H;
    const int n = p.f.n_side[side], r = p.f.r;
    const float c1 = kLog2e / p.f.eps;
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.f.Q : p.f.K);
    const IO* vals = reinterpret_cast<const IO*>(side == 0 ? p.dO : p.f.V);
    const float* ymat = (side == 0 ? p.yp : p.dyraw) + (size_t)g * kRmax * D;
    const float yscale = side == 0 ? (float)n : 1.f;
    const size_t per_k = (size_t)pairs * p.f.n;
    const float* lse = p.f.rowlse + (size_t)pair * p.f.n;
    const float* erow = p.erow + (size_t)pair * p.f.n;
    float* s_y = reinterpret_cast<float*>(s_dyn);
    float* s_hist = reinterpret_cast<float*>(s_dyn);
    char* s_zstash = s_dyn + stage_bytes;
    char* s_yhi = s_zstash + (size_t)groups * kStash;
    char* s_ylo = s_yhi + (size_t)groups * kStash;
    bf16x8* s_zf = reinterpret_cast<bf16x8*>(s_yhi + (size_t)groups * kStash * (kSplit ? 1 : 2));

    if (tid < T) s_shift[tid] = p.gmax[(size_t)tid * pairs + pair] * c1;
    for (int q = wave; q < groups; q += WAVES) {
        Frag<IO, D> z0[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const int t = kGroup * (q0 + q) + 32 * mb + i;
            load_pivots<D>(z0[mb], p.f.Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
        }
        stash_pivots<D, 2>(s_zstash + (size_t)q * kStash, z0, lane);
    }
    for (int q = 0; q < groups; ++q) {
        // Z rows as B fragments (the values the forward pass multiplied with: rounded to bf16 for bf16 I/O)
        __syncthreads();
        for (int e = tid; e < kGroup * D; e += kThreads) {
            const int t = kGroup * (q0 + q) + e / D;
            float z = t < r ? p.f.Z[((size_t)h * r + t) * D + e % D] : 0.f;
            if (!kSplit) z = (float)(__bf16)z;
            s_y[e] = z;
        }
        __syncthreads();
        // (bf16 I/O has no use for the lo fragments: they land where this group's lo matrix stash is written next)
        static_assert(kSplit || kFragsPerGroup * sizeof(bf16x8) <= (size_t)kStash, "lo fragments fit the lo stash");
        bf16x8* hi = s_zf + (size_t)(kParts * q) * kFragsPerGroup;
        lay_out_fragments<D, 2>(s_y, hi, kSplit ? hi + kFragsPerGroup : reinterpret_cast<bf16x8*>(s_ylo + (size_t)q * kStash), tid);
        stash_matrix_rows<IO, D>(s_yhi + (size_t)q * kStash, s_ylo + (size_t)q * kStash, s_y,
                                 ymat + (size_t)kGroup * (q0 + q) * D, yscale, tid, wave, lane);
    }
    __syncthreads();
    for (int q = 0; q < groups; ++q)
        load_tables(s_hist + (size_t)q * T * 2 * kGroup, s_bvec + kGroup * q, p, pair, kGroup * (q0 + q), c1, tid);
    __syncthreads();

    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.f.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.f.tiles_per_wg);
    const float scale_out = 1.f / ((float)n * p.f.eps);   // a / eps
    for (int tile = tile_begin + wave; tile < tile_end; tile += WAVES) {
        const bool valid = tile * kTileTokens + i < n;
        const int tok = min(tile * kTileTokens + i, n - 1);
        Frag<IO, D> xc, vc;
        load_tokens<D>(xc, X + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        load_tokens<D>(vc, vals + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        const float m_tok = gb_token_weight(p, side, g, tok);
        f32x16 o[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[nb][j] = 0.f;
        const int prow0 = tile * kTileTokens + 4 * kg;
        float* const pbase = partial + ((size_t)pair * p.f.n + prow0) * D + NB * i;
        if (!first) {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (prow0 + 8 * (j >> 2) + (j & 3) < n)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) o[nb][j] = pbase[(size_t)(8 * (j >> 2) + (j & 3)) * D + nb];
        }
        for (int q = 0; q < groups; ++q) {
            f32x16 dacc[2], part[NB];
            similarity_gradient<IO, D>(dacc, s_zstash + (size_t)q * kStash, s_yhi + (size_t)q * kStash,
                                       s_ylo + (size_t)q * kStash, s_hist + (size_t)q * T * 2 * kGroup, s_bvec + kGroup * q,
                                       s_shift, xc, vc, lse, erow, per_k, tok, valid, m_tok, side == 1 ? m_tok : 1.f, T, c1, scale_out,
                                       lane, kg);
            const bf16x8* hi = s_zf + (size_t)(kParts * q) * kFragsPerGroup;
            contract_pivots<D, 2, kSplit>(part, dacc, hi, kSplit ? hi + kFragsPerGroup : hi, lane);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 16; ++j) o[nb][j] += part[nb][j];
        }
        if (!last) {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (prow0 + 8 * (j >> 2) + (j & 3) < n)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) pbase[(size_t)(8 * (j >> 2) + (j & 3)) * D + nb] = o[nb][j];
            continue;
        }
        IO* out = reinterpret_cast<IO*>(side == 0 ? p.dQ : p.dK);
        const int row0 = tile * kTileTokens + 4 * kg;
        IO* const lane_base = out + ((size_t)g * p.f.stride_side[side] + row0) * D;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (row0 + 8 * (j >> 2) + (j & 3) < n)
                store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, o[0][j], o[NB - 1][j]);
    }
}

// ---------------------------------------------------------------------------------------------
// assemble-z: per (pair, chunk, group) the workgroup's share of dZ = dC^T X
// ---------------------------------------------------------------------------------------------
template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) gb_assemble_z(GbParams p)
{
    constexpr int NB = D / 32;
    constexpr int kStash = StashBytes<IO, D, 2>::value;
    constexpr bool kSplit = io_is_f32<IO>::value;
    constexpr int kParts = kSplit ? 2 : 1;
    __shared__ float s_bvec[kGroup], s_shift[64];
    __shared__ __attribute__((aligned(16))) float s_y[64 * D];
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[kWaves * kParts * 64 * kTrStride];
    __shared__ __attribute__((aligned(16))) char s_zstash[kStash];
    __shared__ __attribute__((aligned(16))) char s_yhi[kStash];
    __shared__ __attribute__((aligned(16))) char s_ylo[kSplit ? 16 : kStash];
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];   // [T][2][64] floats: g^{k-1} c1, dc^k
    float* s_hist = reinterpret_cast<float*>(s_dyn);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.f.G, T = p.f.T;
    int wg, grp;
    if (!group_block(wg, grp, pairs * p.f.chunks, p.f.groups)) return;
    const int pair = wg / p.f.chunks, chunk = wg % p.f.chunks;
    const int side = pair / p.f.G, g = pair % p.f.G, h = g % p.f.H;
    const int n = p.f.n_side[side];        // tokens of this side (p.f.n, the longer side, strides the per-token arrays)
    const float c1 = kLog2e / p.f.eps;
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.f.Q : p.f.K);
    const IO* vals = reinterpret_cast<const IO*>(side == 0 ? p.dO : p.f.V);
    const float* ymat = (side == 0 ? p.yp : p.dyraw) + ((size_t)g * kRmax + (size_t)kGroup * grp) * D;
    const float yscale = side == 0 ? (float)n : 1.f;
    const size_t per_k = (size_t)pairs * p.f.n;
    const float* lse = p.f.rowlse + (size_t)pair * p.f.n;
    const float* erow = p.erow + (size_t)pair * p.f.n;
    uint16_t* tr_hi = s_tr + (wave * kParts + 0) * 64 * kTrStride;
    uint16_t* tr_lo = s_tr + (wave * kParts + kParts - 1) * 64 * kTrStride;

    if (tid < T) s_shift[tid] = p.gmax[(size_t)tid * pairs + pair] * c1;
    load_tables(s_hist, s_bvec, p, pair, kGroup * grp, c1, tid);
    if (wave == 0) stash_group_pivots<IO, D>(s_zstash, p.f.Z, h, p.f.r, grp, lane);
    stash_matrix_rows<IO, D>(s_yhi, s_ylo, s_y, ymat, yscale, tid, wave, lane);
    __syncthreads();   // s_y is reused below for the dZ partial

    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.f.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.f.tiles_per_wg);
    const float scale_out = 1.f / ((float)n * p.f.eps);
    f32x16 dZacc[2][NB];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 16; ++j) dZacc[mb][nb][j] = 0.f;
    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        const bool valid = tile * kTileTokens + i < n;
        const int tok = min(tile * kTileTokens + i, n - 1);
        Frag<IO, D> xc, vc;
        load_tokens<D>(xc, X + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        load_tokens<D>(vc, vals + ((size_t)g * p.f.stride_side[side] + tok) * D, kg);
        f32x16 dacc[2];
        const float m_tok = gb_token_weight(p, side, g, tok);
        similarity_gradient<IO, D>(dacc, s_zstash, s_yhi, s_ylo, s_hist, s_bvec, s_shift, xc, vc, lse, erow, per_k, tok, valid,
                                   m_tok, side == 1 ? m_tok : 1.f, T, c1, scale_out, lane, kg);
        bf16x8 vh[2][NB], vl[2][NB];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
            const int left = max(1, min(8, n - t0));
            load_values<D>(vh[s], vl[s], X, (size_t)g * p.f.stride_side[side] + min(t0, n - 1), left, i);
        }
        transpose_tile<2, kSplit>(dacc, tr_hi, tr_lo, i, kg);
        contract_tokens<D, 2, kSplit>(dZacc, tr_hi, tr_lo, vh, vl, i, kg);
        transpose_done();
    }
    __syncthreads();
    sum_over_waves<D, 2>(dZacc, s_y, wave, i, kg);
    float* zp = p.dz_part + (((size_t)pair * p.f.chunks + chunk) * kRmax + (size_t)kGroup * grp) * D;
    for (int e = tid; e < kGroup * D; e += kThreads) zp[e] = s_y[e];
}

// ---------------------------------------------------------------------------------------------
// final: dZ[h][t][c] and dbeta[h][t], summed over chunks, sides and the batch.  32 outputs per workgroup,
// each summed by 8 to 32 threads (`slices`) that take every slices-th of the (problem of the batch, side, chunk) shares, four loads
// in flight each, and are then added in order: a fixed order, and one or two rounds of loads whatever the
// numbers of problems and of chunks.
// ---------------------------------------------------------------------------------------------
constexpr int kFinalSlices = 32, kFinalOutputs = 32;      // (kFinalSlices: the most a launch may ask for)
// Threads per output: as many as keep the launch within a quarter of a million threads (beyond that, starting the
// wavefronts costs more than their loads save: 33280 outputs with 32 threads each 9.1 us, with 8 each 5.9 us).
inline int final_slices(long long outputs)
{
    int slices = kFinalSlices;
    while (slices > 8 && outputs * slices > 262144) slices /= 2;
    return slices;
}
__global__ void __launch_bounds__(kFinalSlices * kFinalOutputs) gb_final(GbParams p, int D, int step_q, int step_ch)   // (slices / chunks, slices % chunks)
{
    __shared__ float s_part[kFinalSlices][kFinalOutputs];
    const int o = threadIdx.x % kFinalOutputs, slice = threadIdx.x / kFinalOutputs, slices = blockDim.x / kFinalOutputs;
    const int idx = blockIdx.x * kFinalOutputs + o;     // (h, t, c), c == D meaning beta
    const int r = p.f.r, G = p.f.G, chunks = p.f.chunks;
    const int per = r * (D + 1);
    const bool live = idx < p.f.H * per;
    const int h = live ? idx / per : 0, t = live ? (idx % per) / (D + 1) : 0, c = live ? idx % (D + 1) : 0;
    float acc = 0.f;
    if (live && c < D) {
        // the shares of every (problem of the batch, side, chunk), numbered (side B + b) chunks + chunk: every
        // slices-th one, four loads in flight; the walk carries (row, chunk) along instead of dividing each time
        const int rows = 2 * p.B;
        int q = slice / chunks, ch = slice % chunks;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        auto next_share = [&]() {
            float v = 0.f;
            if (q < rows) {
                const int side = q >= p.B ? 1 : 0, g = (q - side * p.B) * p.f.H + h;
                v = p.dz_part[(((size_t)(side * G + g) * chunks) + ch) * kRmax * D + t * D + c];
            }
            q += step_q; ch += step_ch;
            if (ch >= chunks) { ch -= chunks; ++q; }
            return v;
        };
        while (q < rows) {
            const float v0 = next_share(), v1 = next_share(), v2 = next_share(), v3 = next_share();
            a0 += v0; a1 += v1; a2 += v2; a3 += v3;
        }
        acc = (a0 + a1) + (a2 + a3);
    } else if (live) {
        for (int b = slice; b < p.B; b += slices) {
            const int g = b * p.f.H + h;
            acc += p.db_glue[g * kRmax + t];
            acc += p.db_pair[(size_t)g * kRmax + t];
            acc += p.db_pair[(size_t)(G + g) * kRmax + t];
        }
    }
    s_part[slice][o] = acc;
    __syncthreads();
    if (slice == 0 && live) {
        float tot = 0.f;
        for (int sl = 0; sl < slices; ++sl) tot += s_part[sl][o];
        if (c < D) p.dZ[((size_t)h * r + t) * D + c] = tot;
        else p.dbeta[h * r + t] = tot;
    }
}

// Dynamic LDS of the assemble-x kernel, the largest of this path.
inline size_t assemble_x_stage_bytes(int D, int groups, int T)
{
    const size_t stage = (size_t)kGroup * D * sizeof(float), hist = (size_t)T * groups * 2 * kGroup * sizeof(float);
    return stage > hist ? stage : hist;
}
inline size_t assemble_x_lds_bytes(bool f32, int D, int groups, int T)
{
    const size_t stash = (size_t)2 * 64 * (f32 ? (size_t)(D / 2) * 4 : (size_t)(D / 16) * 16);   // StashBytes<IO, D, 2>
    const size_t frags = (size_t)2 * 2 * (D / 32) * 64 * sizeof(bf16x8);
    return assemble_x_stage_bytes(D, groups, T) + groups * stash * (f32 ? 2 : 3) + groups * frags * (f32 ? 2 : 1);
}
constexpr size_t kLdsBudget = 160 * 1024 - 2048;    // per workgroup, less the kernel's static arrays
// Groups of pivots whose tables the assemble-x kernel holds at once: all of them where they fit, otherwise
// as many as fit (at least one: a group with 64 iterations is 32 KB of tables beside 32-48 KB of operands).
inline int assemble_x_groups_per_launch(bool f32, int D, int groups, int T)
{
    int nq = groups;
    while (nq > 1 && assemble_x_lds_bytes(f32, D, nq, T) > kLdsBudget) --nq;
    return nq;
}

template <typename IO, int D>
int launch_bwd_grouped(const BwdArgs& a, GbParams p)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    constexpr int kAssembleWaves = kSplit ? 4 : 8;     // (fp32 I/O: eight would not fit the register file)
    static_assert(StashBytes<IO, D, 2>::value == 2 * 64 * (kSplit ? (D / 2) * 4 : (D / 16) * 16), "stash size as the host computes it");
    hipStream_t st = a.stream;
    const int pairs = 2 * p.f.G, T = a.iters, groups = p.f.groups;
    const size_t words = (size_t)(T + 1) * pairs * kRmax;
    lg_clear<<<(unsigned)((words + 255) / 256), 256, 0, st>>>(p.f.colacc, words, (unsigned long long*)a.ws, next_nonce());
    const size_t stash = (size_t)groups * StashBytes<IO, D, 2>::value;
    const size_t frag_bytes = (size_t)groups * 2 * (2 * 2 * NB * 64) * sizeof(bf16x8);
    const size_t glue_bytes = stash * (kSplit ? 2 : 3);
    const int ax_groups = assemble_x_groups_per_launch(kSplit, D, groups, T);
    const size_t stage = assemble_x_stage_bytes(D, ax_groups, T);
    const size_t ax_bytes = assemble_x_lds_bytes(kSplit, D, ax_groups, T);
    const size_t az_bytes = (size_t)T * 2 * kGroup * sizeof(float);
    if (ax_bytes > kLdsBudget || T > 64) return LOT_ERR_PATH;
    // more than 64 KB of LDS per workgroup has to be asked for explicitly
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(lg_pass<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)stash));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(lg_expand<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(stash + frag_bytes)));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(gb_glue<IO, D, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)glue_bytes));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(gb_glue<IO, D, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)glue_bytes));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(gb_rec_pass<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)stash));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(gb_assemble_x<IO, D, kAssembleWaves>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ax_bytes));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(gb_assemble_z<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)az_bytes));
    const unsigned grid = (unsigned)pairs * p.f.chunks;
    for (int k = 1; k <= T; ++k) {
        p.f.k = k;
        lg_pass<IO, D><<<grid, kThreads, stash, st>>>(p.f);
    }
    gb_contract<IO, D><<<group_grid(grid, groups), kThreads, 0, st>>>(p);
    gb_mid<D><<<(unsigned)(p.f.G * kRmax * D / 256), 256, 0, st>>>(p);
    lg_expand<IO, D><<<(unsigned)p.f.G * p.f.chunks, kThreads, stash + frag_bytes, st>>>(p.f, 1, p.f.K, p.ydv, p.dV, 1);
    if (p.f.tiles_per_wg >= 32) gb_glue<IO, D, 8><<<grid, 512, glue_bytes, st>>>(p);
    else gb_glue<IO, D, 4><<<grid, 256, glue_bytes, st>>>(p);
    for (int k = T; k >= 1; --k) gb_rec_pass<IO, D><<<grid, kThreads, stash, st>>>(p, k);
    {
        // The dQ/dK assembly writes rows, nothing per workgroup, so it need not share the other kernels' split of
        // a side into workgroups -- and should not: its set-up (the tables and operands of all groups) costs as
        // much as several tiles, and its LDS lets one or two workgroups on a compute unit.  It takes at least one
        // tile per wavefront, and up to four where that brings the grid down to what the device holds at once (with
        // twice that, every compute unit pays the set-up twice: n = 4096, r = 128 56 -> 30 us; with many tiles per
        // wavefront the set-up no longer counts and two rounds of shorter workgroups balance better: n = 131072,
        // r = 256 650 us as it was, 699 in one round).
        int occ = 1;
        {
            // (asked once per device and LDS size: the last answer is kept)
            static std::mutex guard;
            static int last_dev = -1, last_occ = 0;
            static size_t last_bytes = 0;
            int dev = 0;
            LOT_HIP_CHECK(hipGetDevice(&dev));
            std::lock_guard<std::mutex> lock(guard);
            if (dev != last_dev || ax_bytes != last_bytes) {
                LOT_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&last_occ, gb_assemble_x<IO, D, kAssembleWaves>,
                                                                           64 * kAssembleWaves, ax_bytes));
                last_dev = dev; last_bytes = ax_bytes;
            }
            occ = last_occ;
        }
        const long long capacity = (long long)(occ > 0 ? occ : 1) * device_cus();
        const int ntiles = (p.f.n + kTileTokens - 1) / kTileTokens;
        int per = p.f.tiles_per_wg > kAssembleWaves ? p.f.tiles_per_wg : kAssembleWaves;
        while ((long long)pairs * ((ntiles + per - 1) / per) > capacity && per < 4 * kAssembleWaves) per += kAssembleWaves;
        GbParams px = p;
        px.f.tiles_per_wg = per;
        px.f.chunks = (ntiles + per - 1) / per;
        const unsigned grid_x = (unsigned)pairs * px.f.chunks;
        for (int q0 = 0; q0 < groups; q0 += ax_groups) {
            const int nq = groups - q0 < ax_groups ? groups - q0 : ax_groups;
            gb_assemble_x<IO, D, kAssembleWaves><<<grid_x, 64 * kAssembleWaves, ax_bytes, st>>>(
                px, (int)stage, q0, nq, p.x_part, q0 == 0 ? 1 : 0, q0 + nq >= groups ? 1 : 0);
        }
    }
    gb_assemble_z<IO, D><<<group_grid(grid, groups), kThreads, az_bytes, st>>>(p);
    {
        const int slices = final_slices(a.s.H * a.s.r * (D + 1));
        gb_final<<<(unsigned)((a.s.H * a.s.r * (D + 1) + kFinalOutputs - 1) / kFinalOutputs), slices * kFinalOutputs, 0, st>>>(p, D, slices / p.f.chunks, slices % p.f.chunks);
    }
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

}  // namespace

bool bwd_grouped_supports(const lot_shape& s, int iters)
{
    if (!grouped_supports(s) || s.r <= 64 || iters < 1) return false;
    const int groups = (s.r + kGroup - 1) / kGroup;
    const bool f32 = s.io_dtype != LOT_BF16;
    return assemble_x_lds_bytes(f32, s.d_k, assemble_x_groups_per_launch(f32, s.d_k, groups, iters), iters) <= kLdsBudget &&
           iters <= 64;
}

BwdGroupedWorkspace carve_bwd_grouped(const lot_shape& s, int iters)
{
    BwdGroupedWorkspace w{};
    size_t off = 256;      // the status words come first, as in the other workspaces
    auto take = [&](size_t bytes) { size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
    const size_t G = (size_t)s.B * s.H, pairs = 2 * G, T = iters, D = s.d_k, n = s.n;
    const size_t ntiles = (n + kTileTokens - 1) / kTileTokens;
    const size_t per = (size_t)lg_tiles_per_wg(s);
    const size_t chunks = (ntiles + per - 1) / per;
    w.chunks = (int)chunks;
    w.colacc = take((T + 1) * pairs * kRmax * 8);
    w.ghist = take((T + 1) * pairs * kRmax * 4);
    w.rowlse = take(T * pairs * n * 4);
    w.erow = take(T * pairs * n * 4);
    w.u_part = take(pairs * chunks * kRmax * D * 4);
    w.yp = take(G * kRmax * D * 4);
    w.dyraw = take(G * kRmax * D * 4);
    w.ydv = take(G * kRmax * D * 4);
    w.rhop = take(pairs * kRmax * 4);
    w.s_part = take(pairs * chunks * kRmax * 4);
    w.dg_part = take(T * pairs * chunks * kRmax * 4);
    w.dcs = take(T * pairs * kRmax * 4);
    w.gmax = take(T * pairs * 4);
    w.db_pair = take(pairs * kRmax * 4);
    w.db_glue = take(G * kRmax * 4);
    w.dz_part = take(pairs * chunks * kRmax * D * 4);
    {
        // partial dQ / dK rows between the launches of the assemble-x kernel, where it takes several
        const int groups = (s.r + kGroup - 1) / kGroup;
        const bool f32 = s.io_dtype != LOT_BF16;
        const bool several = assemble_x_groups_per_launch(f32, s.d_k, groups, iters) < groups;
        w.x_part = take(several ? pairs * n * D * 4 : 0);
    }
    w.total = off;
    return w;
}

int run_backward_grouped(const BwdArgs& a)
{
    const lot_shape& s = a.s;
    if (!bwd_grouped_supports(s, a.iters)) return LOT_ERR_PATH;
    const BwdGroupedWorkspace L = carve_bwd_grouped(s, a.iters);
    GbParams p{};
    p.f.Q = a.Q; p.f.K = a.K; p.f.V = a.V; p.f.Z = a.Z; p.f.beta = a.beta; p.f.out = nullptr;
    p.dO = a.dO; p.dQ = a.dQ; p.dK = a.dK; p.dV = a.dV; p.dZ = a.dZ; p.dbeta = a.dbeta;
    p.f.colacc = (unsigned long long*)(a.ws + L.colacc);
    p.f.ghist = (float*)(a.ws + L.ghist);
    p.f.rowlse = (float*)(a.ws + L.rowlse); p.f.rowlse_all = 1;
    p.f.u_part = nullptr; p.f.ypp = nullptr;
    p.erow = (float*)(a.ws + L.erow);
    p.u_part = (float*)(a.ws + L.u_part);
    p.yp = (float*)(a.ws + L.yp);
    p.dyraw = (float*)(a.ws + L.dyraw);
    p.ydv = (float*)(a.ws + L.ydv);
    p.rhop = (float*)(a.ws + L.rhop);
    p.s_part = (float*)(a.ws + L.s_part);
    p.dg_part = (float*)(a.ws + L.dg_part);
    p.dcs = (float*)(a.ws + L.dcs);
    p.gmax = (float*)(a.ws + L.gmax);
    p.db_pair = (float*)(a.ws + L.db_pair);
    p.db_glue = (float*)(a.ws + L.db_glue);
    p.dz_part = (float*)(a.ws + L.dz_part);
    p.x_part = (float*)(a.ws + L.x_part);
    p.B = s.B;
    p.f.G = s.B * s.H; p.f.H = s.H; p.f.n = s.n; p.f.r = s.r;
    p.f.n_side[0] = a.n_q > 0 ? a.n_q : s.n;      // s.n is the longer side (cross attention)
    p.f.n_side[1] = a.n_k > 0 ? a.n_k : s.n;
    for (int sd = 0; sd < 2; ++sd) p.f.stride_side[sd] = a.n_stride > 0 ? a.n_stride : p.f.n_side[sd];
    p.f.mass_side[0] = a.mass_q; p.f.mass_side[1] = a.mass_k;
    p.f.groups = (s.r + kGroup - 1) / kGroup; p.f.chunks = L.chunks; p.f.tiles_per_wg = lg_tiles_per_wg(s); p.f.T = a.iters;
    p.f.eps = a.eps;
    {
        int frac = 62 - (int)std::ceil(std::log2((double)s.n + 1.0));
        p.f.fx_scale = std::ldexp(1.0f, frac);
        p.f.fx_unscale = std::ldexp(1.0f, -frac);
    }
    if (s.io_dtype == LOT_BF16) return s.d_k == 64 ? launch_bwd_grouped<uint16_t, 64>(a, p) : launch_bwd_grouped<uint16_t, 32>(a, p);
    return s.d_k == 64 ? launch_bwd_grouped<float, 64>(a, p) : launch_bwd_grouped<float, 32>(a, p);
}

}  // namespace lot
