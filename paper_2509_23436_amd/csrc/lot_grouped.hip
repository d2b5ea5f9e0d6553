// LOT attention forward for pivot sizes beyond one register tile: 64 < r <= 256, d_k = d_v in
// {32, 64}.  (The paper's runtime study sweeps r up to 256.)  Smaller r runs here too when the caller asks
// for a path on which no kernel waits for another workgroup.  Same method as the fused kernel --
// similarities by MFMA, log-domain Sinkhorn with implicit token potentials, factored apply -- with the
// pivots taken in groups of 64:
//   * a pass keeps the similarities of all groups of a tile of 32 tokens in registers (up to 128 per
//     lane) between the row reduction and the exponentials: one exponential per element;
//   * the last pass leaves each row's log-normaliser in the workspace (4 bytes per token and solve),
//     from which the contraction with V and the expansion with Y'' rebuild one group's weights at a time;
//   * column sums are reduced to one pivot per lane after every tile (transposing reduction), so a
//     lane carries one accumulator per group instead of 32.
// One launch per step; launch boundaries are the only synchronisation between workgroups:
//   clear | T x pass (both solves: pair = side * G + g, side 0 = queries) | reduce (keys, one workgroup
//   per group: U = sum_j W2 V) | mid (Y'' = n beta/cs1 * U/cs2) | expand (queries -> O).
// Column sums are exchanged as fixed-point integers (atomic adds): order-independent, reproducible.
#include "lot_internal.h"
#include "lot_tile.h"
#include "lot_tile_ops.h"
#include "lot_plain_kernels.h"
#include "lot_grouped_ops.h"

namespace lot {
namespace {

// ---------------------------------------------------------------------------------------------
// reduce: U_t = sum_j W2_jt V_j for the pivots of one group per workgroup (keys; potentials g2^{T-1})
// ---------------------------------------------------------------------------------------------
template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) lg_reduce(LgParams p)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    __shared__ float s_g[kRmax];
    __shared__ __attribute__((aligned(16))) float s_buf[64 * D];
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[kWaves * 2 * 64 * kTrStride];
    extern __shared__ __attribute__((aligned(16))) char s_zstash[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    int wg, grp;
    if (!group_block(wg, grp, p.G * p.chunks, p.groups)) return;
    const int g = wg / p.chunks, chunk = wg % p.chunks;
    const int pair = p.G + g, h = g % p.H;
    const int n = p.n_side[1], stride = p.stride_side[1];
    const float* const mass = p.mass_side[1];     // the keys' masses times n weight the reduction
    const float c1 = kLog2e / p.eps;
    const IO* X = reinterpret_cast<const IO*>(p.K);
    const IO* vals = reinterpret_cast<const IO*>(p.V);
    uint16_t* tr_hi = s_tr + (wave * 2 + 0) * 64 * kTrStride;
    uint16_t* tr_lo = s_tr + (wave * 2 + 1) * 64 * kTrStride;
    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.tiles_per_wg);

    const float* lse = last_lse(p) + (size_t)pair * p.n;
    load_potentials(p, s_g, p.T, pair, h, false, tid);
    stash_all_pivots<IO, D>(s_zstash, p.Z, h, p.r, p.groups, wave, lane);
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
        Frag<IO, D> xc;
        load_tokens<D>(xc, X + ((size_t)g * stride + tok) * D, kg);
        bf16x8 vh[2][NB], vl[2][NB];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
            const int left = max(1, min(8, n - t0));
            load_values<D>(vh[s], vl[s], vals, (size_t)g * stride + min(t0, n - 1), left, i);
        }
        const float L = tile * kTileTokens + i < n ? lse[tok] : INFINITY;
        f32x16 acc[2];
        weights_from_lse<IO, D>(acc, s_zstash + (size_t)grp * StashBytes<IO, D, 2>::value, s_g + kGroup * grp, xc, L, lane, kg, c1);
        if (mass) {
            const float mt = (float)n * mass[(size_t)g * n + tok];
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
    float* up = p.u_part + (((size_t)g * p.chunks + chunk) * kRmax + (size_t)kGroup * grp) * D;
    for (int e = tid; e < kGroup * D; e += kThreads) up[e] = s_buf[e];
}

// ---------------------------------------------------------------------------------------------
// mid: Y''_t = (n beta_t / cs1_t) * U_t / cs2_t, one thread per (g, t, column)
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ void lg_mid(LgParams p)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= p.G * kRmax * D) return;
    const int g = idx / (kRmax * D), e = idx % (kRmax * D), t = e / D;
    const int pairs = 2 * p.G, T = p.T;
    float y = 0.f;
    if (t < p.r) {
        float u0 = 0.f, u1 = 0.f;
        const float* up = p.u_part + ((size_t)g * p.chunks) * kRmax * D + e;
        int c = 0;
        for (; c + 1 < p.chunks; c += 2) { u0 += up[(size_t)c * kRmax * D]; u1 += up[(size_t)(c + 1) * kRmax * D]; }
        if (c < p.chunks) u0 += up[(size_t)c * kRmax * D];
        const float cs1 = fmaxf((float)(long long)p.colacc[((size_t)T * pairs + g) * kRmax + t] * p.fx_unscale, 0.5f * p.fx_unscale);
        const float cs2 = fmaxf((float)(long long)p.colacc[((size_t)T * pairs + p.G + g) * kRmax + t] * p.fx_unscale, 0.5f * p.fx_unscale);
        y = ((float)p.n_side[0] * p.beta[(g % p.H) * p.r + t] / cs1) * ((u0 + u1) / cs2);
    }
    p.ypp[idx] = y;
}

template <typename IO, int D>
int launch_grouped(const Args& a, LgParams p)
{
    constexpr int NB = D / 32;
    hipStream_t st = a.stream;
    const int pairs = 2 * p.G, T = a.iters;
    const size_t words = (size_t)(T + 1) * pairs * kRmax;
    lg_clear<<<(unsigned)((words + 255) / 256), 256, 0, st>>>(p.colacc, words, (unsigned long long*)a.ws, next_nonce());
    const size_t stash = (size_t)p.groups * StashBytes<IO, D, 2>::value;
    const size_t frag_bytes = (size_t)p.groups * 2 * (2 * 2 * NB * 64) * sizeof(bf16x8);
    // more than 64 KB of LDS per workgroup has to be asked for explicitly
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(lg_pass<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)stash));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(lg_reduce<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)stash));
    LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(lg_expand<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(stash + frag_bytes)));
    for (int k = 1; k <= T; ++k) {
        p.k = k;
        lg_pass<IO, D><<<(unsigned)pairs * p.chunks, kThreads, stash, st>>>(p);
    }
    lg_reduce<IO, D><<<group_grid((unsigned)p.G * p.chunks, p.groups), kThreads, stash, st>>>(p);
    lg_mid<D><<<(unsigned)((p.G * kRmax * D + 255) / 256), 256, 0, st>>>(p);
    lg_expand<IO, D><<<(unsigned)p.G * p.chunks, kThreads, stash + frag_bytes, st>>>(p, 0, p.Q, p.ypp, p.out, 0);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

}  // namespace

bool grouped_supports(const lot_shape& s)
{
    return s.d_k == s.d_v && (s.d_k == 32 || s.d_k == 64) && s.r <= kRmax;
}

GroupedWorkspace carve_grouped(const lot_shape& s, int iters)
{
    GroupedWorkspace w{};
    size_t off = 256;      // status words first, as in the other layouts
    auto take = [&](size_t bytes) { size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
    const size_t G = (size_t)s.B * s.H, pairs = 2 * G, T = iters, D = s.d_k;
    const size_t ntiles = ((size_t)s.n + kTileTokens - 1) / kTileTokens;
    const size_t per = (size_t)lg_tiles_per_wg(s);
    w.chunks = (int)((ntiles + per - 1) / per);
    w.colacc = take((T + 1) * pairs * kRmax * 8);
    w.ghist = take((T + 1) * pairs * kRmax * 4);
    w.u_part = take(G * w.chunks * kRmax * D * 4);
    w.ypp = take(G * kRmax * D * 4);
    w.rowlse = take(pairs * (size_t)s.n * 4);
    w.total = off;
    return w;
}

int run_grouped(const Args& a)
{
    const lot_shape& s = a.s;
    if (!grouped_supports(s)) return LOT_ERR_PATH;
    const GroupedWorkspace L = carve_grouped(s, a.iters);
    LgParams p{};
    p.Q = a.Q; p.K = a.K; p.V = a.V; p.Z = a.Z; p.beta = a.beta; p.out = a.out;
    p.colacc = (unsigned long long*)(a.ws + L.colacc);
    p.ghist = (float*)(a.ws + L.ghist);
    p.u_part = (float*)(a.ws + L.u_part);
    p.ypp = (float*)(a.ws + L.ypp);
    p.rowlse = (float*)(a.ws + L.rowlse); p.rowlse_all = 0;
    p.G = s.B * s.H; p.H = s.H; p.n = s.n; p.r = s.r;
    p.n_side[0] = a.n_q > 0 ? a.n_q : s.n;      // s.n is the longer side (cross attention)
    p.n_side[1] = a.n_k > 0 ? a.n_k : s.n;
    for (int sd = 0; sd < 2; ++sd) p.stride_side[sd] = a.n_stride > 0 ? a.n_stride : p.n_side[sd];
    p.mass_side[0] = a.mass_q; p.mass_side[1] = a.mass_k;
    p.groups = (s.r + kGroup - 1) / kGroup; p.chunks = L.chunks; p.tiles_per_wg = lg_tiles_per_wg(s); p.T = a.iters;
    p.eps = a.eps;
    {
        int frac = 62 - (int)std::ceil(std::log2((double)s.n + 1.0));
        p.fx_scale = std::ldexp(1.0f, frac);
        p.fx_unscale = std::ldexp(1.0f, -frac);
    }
    if (s.io_dtype == LOT_BF16) return s.d_k == 64 ? launch_grouped<uint16_t, 64>(a, p) : launch_grouped<uint16_t, 32>(a, p);
    return s.d_k == 64 ? launch_grouped<float, 64>(a, p) : launch_grouped<float, 32>(a, p);
}

}  // namespace lot
