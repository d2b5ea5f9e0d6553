// Device code shared by the forward and the backward pass for pivot sizes beyond one register tile
// (64 < r <= 256): the pivots are taken in groups of 64.  A pass keeps the similarities of all groups of a
// tile of 32 tokens in registers (up to 128 per lane) between the row reduction and the exponentials, and
// leaves each row's log-normaliser L_i in memory, from which the kernels after the last pass rebuild one
// group's weights W_it = softmax_t((C_it + g_t)/eps) = exp2((C_it + g_t) c1 - L_i) at a time.
// (Paper, Method: similarities C = X Z^T, Sinkhorn scaling in the log domain; its runtime study sweeps r up to 256.)
#pragma once
#include "lot_internal.h"
#include "lot_tile.h"
#include "lot_tile_ops.h"

namespace lot {
namespace {

constexpr int kGroup = 64;          // pivots per group (two MFMA blocks)
constexpr int kMaxGroups = 4;
constexpr int kRmax = kGroup * kMaxGroups;
inline int g_target_wgs() { return 2 * device_cus(); }   // two workgroups per compute unit

struct LgParams {
    const void* Q; const void* K; const void* V;
    const float* Z; const float* beta;
    void* out;
    unsigned long long* colacc;   // [T+1][pairs][256]
    float* ghist;                 // [T+1][pairs][256]  g^k, k = 0..T-1 (padding pivots: -1e30)
    float* u_part;                // [G][chunks][256][D]
    float* ypp;                   // [G][256][D]  Y''
    float* rowlse;                // base-2 log-normaliser L_i of every row: [T][pairs][n], pass k at k - 1 (rowlse_all), or
    int rowlse_all;               // [pairs][n] of the last pass only; W_it = exp2((C_it + g_t) c1 - L_i)
    int G, H, n, r, groups, chunks, tiles_per_wg, k, T;   // n: the longer side (layout of the per-token arrays, chunking)
    // per side (0 = queries and the output, 1 = keys and values):
    int n_side[2];                // tokens per problem
    int stride_side[2];           // tokens between consecutive problems in the caller's tensors (>= n_side)
    const float* mass_side[2];    // [G][n_side] token masses, or null: uniform 1/n_side
    float eps, fx_scale, fx_unscale;
    // The one-launch form only (zero otherwise): the top byte of an exchanged word counts the workgroups that
    // have added their share (count_one = 1 << 56 rides on every addition, count_mask covers the byte).
    unsigned long long count_one, count_mask;
    unsigned long long* status;   // [0] = nonce of a launch in which a wait gave up, [1] = nonce of the last launch
    unsigned long long nonce;
    unsigned* sync;               // [G][2]: key workgroups that have stored their share of U; ... their slice of Y''
                                  // (cleared per launch)
    uint32_t spin_limit;
};

// the sum an exchanged word carries (a sum below the fixed-point resolution reads as half a unit: the
// potentials stay bounded)
__device__ __forceinline__ float colsum_of(const LgParams& p, unsigned long long word)
{
    return fmaxf((float)(long long)(word & ~p.count_mask) * p.fx_unscale, 0.5f * p.fx_unscale);
}

inline int lg_tiles_per_wg(const lot_shape& s)
{
    const long long ntiles = ((long long)s.n + kTileTokens - 1) / kTileTokens;
    const long long target = g_target_wgs();
    long long per = (ntiles * 2LL * s.B * s.H + target - 1) / target;
    per = (per + kWaves - 1) / kWaves * kWaves;
    if (per < kWaves) per = kWaves;
    if (per > 32 * kWaves) per = 32 * kWaves;
    return (int)per;
}

// Workgroup (wg, grp) of a launch that gives every one of nwg token ranges to `groups` workgroups, one per
// pivot group.  Block ids go round the 8 XCDs, each with its own L2: the workgroups that read the same token
// rows get ids 8 apart, consecutive on one XCD, so that the rows come from HBM once.  False: nothing to do
// (the grid is rounded up to a multiple of 8 * groups).
__device__ __forceinline__ bool group_block(int& wg, int& grp, int nwg, int groups)
{
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    grp = slot % groups;
    wg = (slot / groups) * 8 + xcd;
    return wg < nwg;
}
inline unsigned group_grid(unsigned nwg, int groups) { return (nwg + 7) / 8 * 8 * (unsigned)groups; }

// Common set-up: pivot fragments of all groups to the LDS stash, g^{k-1} to s_g.
template <typename IO, int D>
__device__ __forceinline__ void stash_all_pivots(char* zstash, const float* Z, int h, int r, int groups,
                                                 int wave, int lane)
{
    const int i = lane & 31, kg = lane >> 5;
    for (int p = wave; p < groups; p += kWaves) {
        Frag<IO, D> z0[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const int t = kGroup * p + 32 * mb + i;
            load_pivots<D>(z0[mb], Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
        }
        stash_pivots<D, 2>(zstash + (size_t)p * StashBytes<IO, D, 2>::value, z0, lane);
    }
}

// g^{k-1}_t for all t < 256 into s_g (and, by one workgroup per pair, into ghist[k-1]).
__device__ __forceinline__ void load_potentials(const LgParams& p, float* s_g, int k, int pair, int h, bool keep, int tid)
{
    const int pairs = 2 * p.G;
    for (int t = tid; t < kRmax; t += kThreads) {
        float gv = t < p.r ? 0.f : kNegBig;
        if (k > 1 && t < p.r) {
            const unsigned long long word = p.colacc[((size_t)(k - 1) * pairs + pair) * kRmax + t];
            const float cs = colsum_of(p, word);
            gv = p.ghist[((size_t)(k - 2) * pairs + pair) * kRmax + t] + p.eps * logf((float)p.n_side[pair / p.G] * p.beta[h * p.r + t] / cs);
        }
        s_g[t] = gv;
        if (keep) p.ghist[((size_t)(k - 1) * pairs + pair) * kRmax + t] = gv;
    }
}

// Where pass k keeps its rows' log-normalisers (null: not kept), and where the last pass has left them.
__device__ __forceinline__ float* lse_slot(const LgParams& p, int k)
{
    if (p.rowlse_all) return p.rowlse + (size_t)(k - 1) * 2 * p.G * p.n;
    return k == p.T ? p.rowlse : nullptr;
}
__device__ __forceinline__ const float* last_lse(const LgParams& p)
{
    return p.rowlse + (p.rowlse_all ? (size_t)(p.T - 1) * 2 * p.G * p.n : 0);
}

// acc <- W_it = exp2((C_it + g_t) c1 - L_i) for the 64 pivots of one group (zst: its stash, pot: its g).
// A row past the end carries L = +inf: weights exactly 0.
template <typename IO, int D>
__device__ __forceinline__ void weights_from_lse(f32x16 (&acc)[2], const char* zst, const float* pot,
                                                 const Frag<IO, D>& xf, float L, int lane, int kg, float c1)
{
    int skew = 0;
    asm volatile("" : "+v"(skew));
    Frag<IO, D> zf[2];
    fetch_pivots<D, 2>(zf, zst, lane, skew);
    load_pivot_vector<2>(acc, pot + skew, kg);
    similarity<D, 2>(acc, zf, xf);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[mb][j] = exp2_fast(fmaf(acc[mb][j], c1, -L));
}

// ---------------------------------------------------------------------------------------------
// pass k: column sums of W^k for both solves
// ---------------------------------------------------------------------------------------------
// The rows of a wavefront's first tile of a pass (requested before whatever the pass still waits for).
template <typename IO, int D>
__device__ __forceinline__ void first_tile_of_pass(Frag<IO, D>& xc, const LgParams& p, int pair, int chunk, int wave, int lane)
{
    const int side = pair / p.G, g = pair % p.G;
    const int n = p.n_side[side];
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.Q : p.K);
    const int tok = min((chunk * p.tiles_per_wg + wave) * kTileTokens + (lane & 31), n - 1);
    load_tokens<D>(xc, X + ((size_t)g * p.stride_side[side] + tok) * D, lane >> 5);
}

// The tiles of pass k of one workgroup, with the potentials g^{k-1} in s_g and the pivots in s_zstash (the
// workgroup has synchronised on both), xc = the rows of the wavefront's first tile: adds the workgroup's
// column sums to the pass's words.
template <typename IO, int D>
__device__ __forceinline__ void pass_tiles(const LgParams& p, int k, int pair, int chunk, const float* s_g,
                                           float (*s_cs)[kRmax], const char* s_zstash, Frag<IO, D> xc)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.G;
    const int side = pair / p.G, g = pair % p.G;
    const int n = p.n_side[side], stride = p.stride_side[side];
    const float* const mass = p.mass_side[side];     // token masses times n weight the column sums
    const float c1 = kLog2e / p.eps;
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.Q : p.K);
    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.tiles_per_wg);

    float csg[kMaxGroups] = {0.f, 0.f, 0.f, 0.f};       // this lane's pivot of each group
    float* const lse_keep = lse_slot(p, k);
    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        Frag<IO, D> xn = xc;
        if (tile + kWaves < tile_end) {
            const int tok = min((tile + kWaves) * kTileTokens + i, n - 1);
            load_tokens<D>(xn, X + ((size_t)g * stride + tok) * D, kg);
        }
        // similarities (plus potentials) of all groups stay in registers between the row reduction and the
        // exponentials: one exponential per element
        f32x16 acc[kMaxGroups][2];
        float m0 = -INFINITY, m1 = -INFINITY;
#pragma unroll
        for (int q = 0; q < kMaxGroups; ++q) {
            if (q < p.groups) {
                int skew = 0;
                asm volatile("" : "+v"(skew));
                Frag<IO, D> zf[2];
                fetch_pivots<D, 2>(zf, s_zstash + (size_t)q * StashBytes<IO, D, 2>::value, lane, skew);
                load_pivot_vector<2>(acc[q], s_g + kGroup * q + skew, kg);
                similarity<D, 2>(acc[q], zf, xc);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 2) {
                        m0 = fmaxf(m0, acc[q][mb][j]);
                        m1 = fmaxf(m1, acc[q][mb][j + 1]);
                    }
            }
        }
        const float mc = pair_max(fmaxf(m0, m1)) * c1;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int q = 0; q < kMaxGroups; ++q) {
            if (q < p.groups) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 2) {
                        const float e0 = exp2_fast(fmaf(acc[q][mb][j], c1, -mc));
                        const float e1 = exp2_fast(fmaf(acc[q][mb][j + 1], c1, -mc));
                        acc[q][mb][j] = e0; acc[q][mb][j + 1] = e1;
                        s0 += e0; s1 += e1;
                    }
            }
        }
        const bool valid = tile * kTileTokens + i < n;
        const float rowsum = pair_sum(s0 + s1);
        const float w = valid ? rcp_fast(rowsum) : 0.f;
        if (lse_keep && kg == 0 && valid) lse_keep[(size_t)pair * p.n + tile * kTileTokens + i] = mc + __builtin_amdgcn_logf(rowsum);
        const float wm = mass ? w * ((float)n * mass[(size_t)g * n + min(tile * kTileTokens + i, n - 1)]) : w;
#pragma unroll
        for (int q = 0; q < kMaxGroups; ++q) {
            if (q < p.groups) {
                float c[32];
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) c[16 * mb + j] = acc[q][mb][j] * wm;
                csg[q] += reduce_scatter_tokens<32>(c, i);
            }
        }
        xc = xn;
    }
    // lane (i, kg) holds pivot 32 (i >> 4) + 8 ((i & 15) >> 2) + 4 kg + (i & 3) of every group
    const int mine = 32 * (i >> 4) + 8 * ((i & 15) >> 2) + 4 * kg + (i & 3);
#pragma unroll
    for (int q = 0; q < kMaxGroups; ++q) s_cs[wave][kGroup * q + mine] = csg[q];
    __syncthreads();
    for (int t = tid; t < p.r; t += kThreads) {
        float tot = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) tot += s_cs[wv][t];
        const unsigned long long word = (unsigned long long)__float2ll_rn(tot * p.fx_scale) + p.count_one;
        __hip_atomic_fetch_add(p.colacc + ((size_t)k * pairs + pair) * kRmax + t, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) lg_pass(LgParams p)
{
    __shared__ float s_g[kRmax];
    __shared__ float s_cs[kWaves][kRmax];
    extern __shared__ __attribute__((aligned(16))) char s_zstash[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pair = blockIdx.x / p.chunks, chunk = blockIdx.x % p.chunks;
    const int h = (pair % p.G) % p.H;
    Frag<IO, D> xc;
    first_tile_of_pass<IO, D>(xc, p, pair, chunk, wave, lane);
    load_potentials(p, s_g, p.k, pair, h, chunk == 0, tid);
    stash_all_pivots<IO, D>(s_zstash, p.Z, h, p.r, p.groups, wave, lane);
    __syncthreads();
    pass_tiles<IO, D>(p, p.k, pair, chunk, s_g, s_cs, s_zstash, xc);
}

// ---------------------------------------------------------------------------------------------
// expand: out_i = sum_t W_it Ymat_t over the tokens of one side (potentials g^{T-1} of that side).
// Forward: side 0, Ymat = Y'', out = O.  Backward: side 1, Ymat_t = rho'_t dYraw_t, out = dV, every row times
// its token's mass times n (weight_rows).
// ---------------------------------------------------------------------------------------------
// The tiles of the expansion for one workgroup, with the side's potentials g^{T-1} in s_g and the pivots in
// s_zstash (the caller has stored both; this synchronises).  COHERENT: ymat was written by another workgroup
// of this launch and is read past the caches that might still hold an older copy.
template <typename IO, int D, bool COHERENT>
__device__ __forceinline__ void expand_tiles(const LgParams& p, int side, int g, int chunk, const void* rows, const float* ymat,
                                             void* out_rows, int weight_rows, const float* s_g, float* s_y,
                                             const char* s_zstash, bf16x8* yf)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    constexpr int kFragsPerGroup = 2 * 2 * NB * 64;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int n = p.n_side[side], stride = p.stride_side[side];
    const float c1 = kLog2e / p.eps;
    const IO* X = reinterpret_cast<const IO*>(rows);
    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.tiles_per_wg);
    const float* lse = last_lse(p) + (size_t)(side * p.G + g) * p.n;
    const float* const yg = ymat + (size_t)g * kRmax * D;
    const __amdgpu_buffer_rsrc_t yview = coherent_view(yg);
    for (int q = 0; q < p.groups; ++q) {
        for (int e = tid; e < kGroup * D; e += kThreads)
            s_y[e] = COHERENT ? ldc_f32(yview, (uint32_t)((kGroup * q * D + e) * sizeof(float))) : yg[(size_t)kGroup * q * D + e];
        __syncthreads();
        lay_out_fragments<D, 2>(s_y, yf + (size_t)(2 * q) * kFragsPerGroup, yf + (size_t)(2 * q + 1) * kFragsPerGroup, tid);
        __syncthreads();
    }

    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        const int tok = min(tile * kTileTokens + i, n - 1);
        Frag<IO, D> xc;
        load_tokens<D>(xc, X + ((size_t)g * stride + tok) * D, kg);
        const float L = tile * kTileTokens + i < n ? lse[tok] : INFINITY;
        const float mt = weight_rows && p.mass_side[side] ? (float)n * p.mass_side[side][(size_t)g * n + tok] : 1.f;
        f32x16 o[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[nb][j] = 0.f;
        for (int q = 0; q < p.groups; ++q) {
            f32x16 acc[2], part[NB];
            weights_from_lse<IO, D>(acc, s_zstash + (size_t)q * StashBytes<IO, D, 2>::value, s_g + kGroup * q, xc, L, lane, kg, c1);
            if (weight_rows) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) acc[mb][j] *= mt;
            }
            contract_pivots<D, 2, kSplit>(part, acc, yf + (size_t)(2 * q) * kFragsPerGroup,
                                          yf + (size_t)(2 * q + 1) * kFragsPerGroup, lane);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 16; ++j) o[nb][j] += part[nb][j];
        }
        IO* out = reinterpret_cast<IO*>(out_rows);
        const int row0 = tile * kTileTokens + 4 * kg;
        IO* const lane_base = out + ((size_t)g * stride + row0) * D;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (row0 + 8 * (j >> 2) + (j & 3) < n)
                store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, o[0][j], o[NB - 1][j]);
    }
}

template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) lg_expand(LgParams p, int side, const void* rows, const float* ymat, void* out_rows, int weight_rows)
{
    __shared__ float s_g[kRmax];
    __shared__ __attribute__((aligned(16))) float s_y[64 * D];
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];    // pivot stash, then Y'' fragments (hi, lo) per group
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.x / p.chunks, chunk = blockIdx.x % p.chunks, h = g % p.H;
    load_potentials(p, s_g, p.T, side * p.G + g, h, false, tid);
    stash_all_pivots<IO, D>(s_dyn, p.Z, h, p.r, p.groups, wave, lane);
    expand_tiles<IO, D, false>(p, side, g, chunk, rows, ymat, out_rows, weight_rows, s_g, s_y, s_dyn,
                               reinterpret_cast<bf16x8*>(s_dyn + (size_t)p.groups * StashBytes<IO, D, 2>::value));
}

// zeroes the column-sum words and marks the workspace as used by a launch that cannot fail on the device
// (word 1 of the status area takes a fresh nonce, which word 0, written only by a wait that gave up, cannot hold)
__global__ void lg_clear(unsigned long long* p, size_t count, unsigned long long* status, unsigned long long nonce)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < count) p[idx] = 0ull;
    if (idx == 0) status[1] = nonce;
}

}  // namespace
}  // namespace lot
