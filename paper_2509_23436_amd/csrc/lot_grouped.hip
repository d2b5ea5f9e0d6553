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
// Two forms of the same steps
//   clear | T x pass (both solves: pair = side * G + g, side 0 = queries) | reduce (keys, one workgroup
//   per group: U = sum_j W2 V) | mid (Y'' = n beta/cs1 * U/cs2) | expand (queries -> O):
//   * one launch per step, launch boundaries the only synchronisation between workgroups (any size; the form
//     of LOT_PATH_STEPWISE);
//   * lg_persistent: everything in ONE launch, for the sizes where the launches themselves
//     are what a call costs (short sequences).  A workgroup keeps its chunk of one side for the whole call, the
//     pivots and the potentials stay in its LDS, and what the launch boundaries ordered is ordered by bounded
//     waits: the words of a pass carry, in their top byte, the number of workgroups that have added their share,
//     and one wavefront per workgroup polls them (a poll per word and thread crowds out the additions
//     themselves: measured 0.5 ms per wait); the keys' workgroups count themselves off after storing their share
//     of U, form a slice of Y'' each once all have, and count themselves off again for the queries' workgroups.
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
// One group's share of U from the key tiles of one workgroup, with the keys' potentials g^{T-1} in s_g and the
// pivots in s_zstash (the workgroup has synchronised on both).  COHERENT: the result is for another workgroup
// of this launch and is written through the caches.
template <typename IO, int D, bool COHERENT>
__device__ __forceinline__ void reduce_tiles(const LgParams& p, int g, int chunk, int grp, const float* s_g, float* s_buf,
                                             uint16_t* s_tr, const char* s_zstash)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pair = p.G + g;
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
    for (int e = tid; e < kGroup * D; e += kThreads) {
        if (COHERENT) st_coherent(up + e, s_buf[e]);
        else up[e] = s_buf[e];
    }
}

template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) lg_reduce(LgParams p)
{
    __shared__ float s_g[kRmax];
    __shared__ __attribute__((aligned(16))) float s_buf[64 * D];
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[kWaves * 2 * 64 * kTrStride];
    extern __shared__ __attribute__((aligned(16))) char s_zstash[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int wg, grp;
    if (!group_block(wg, grp, p.G * p.chunks, p.groups)) return;
    const int g = wg / p.chunks, chunk = wg % p.chunks, h = g % p.H;
    load_potentials(p, s_g, p.T, p.G + g, h, false, tid);
    stash_all_pivots<IO, D>(s_zstash, p.Z, h, p.r, p.groups, wave, lane);
    __syncthreads();
    reduce_tiles<IO, D, false>(p, g, chunk, grp, s_g, s_buf, s_tr, s_zstash);
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
        const float cs1 = colsum_of(p, p.colacc[((size_t)T * pairs + g) * kRmax + t]);
        const float cs2 = colsum_of(p, p.colacc[((size_t)T * pairs + p.G + g) * kRmax + t]);
        y = ((float)p.n_side[0] * p.beta[(g % p.H) * p.r + t] / cs1) * ((u0 + u1) / cs2);
    }
    p.ypp[idx] = y;
}

// ---------------------------------------------------------------------------------------------
// The one-launch form
// ---------------------------------------------------------------------------------------------
constexpr size_t kPersistentLdsMax = 160 * 1024;

// LDS of lg_persistent: potentials, pivots of all groups, then the largest of the stages' working areas.
constexpr int kCountShiftLg = 56;     // an exchanged word: workgroups that have added their share in the top byte
// 64-bit words that hold the counters of the one-launch form: [G][2] unsigned, then one word per pair that takes
// the launch's nonce once the pair's words and counters have been zeroed
inline size_t lg_counter_words(size_t G, size_t) { return G + 2 * G; }

// The first wavefront of a workgroup polls the words of one pass of one pair until each carries `chunks`
// arrivals; lane l then holds the words of pivots l, 64 + l, ... in word[].  False, for the whole workgroup, if
// the poll budget ran out or another workgroup of the launch has given up.  Ends with a workgroup barrier.
__device__ __forceinline__ bool wait_for_words(const LgParams& p, const unsigned long long* words, unsigned long long (&word)[kMaxGroups],
                                               int* s_flag, int tid)
{
    if (tid < 64) {
        const __amdgpu_buffer_rsrc_t view = coherent_view(words);
        bool ok = false;
        for (uint32_t k = 0; k < p.spin_limit; ++k) {
            bool all = true;
#pragma unroll
            for (int q = 0; q < kMaxGroups; ++q) {
                const int t = kGroup * q + tid;
                word[q] = t < p.r ? ldc_u64(view, (uint32_t)t * 8u) : ((unsigned long long)p.chunks << kCountShiftLg);
                all = all && (int)(word[q] >> kCountShiftLg) == p.chunks;
            }
            if (__all(all)) { ok = true; break; }
            if ((k & 63u) == 63u && gave_up(p.status, p.nonce)) break;
            __builtin_amdgcn_s_sleep(1);
        }
        if (tid == 0) {
            if (!ok) give_up(p.status, p.nonce);
            s_flag[0] = ok;
        }
    }
    __syncthreads();
    return s_flag[0] != 0;
}

template <typename IO, int D>
inline size_t persistent_lds_bytes(int groups)
{
    constexpr int NB = D / 32;
    const size_t stash = (size_t)groups * StashBytes<IO, D, 2>::value;
    const size_t pass = (size_t)kWaves * kRmax * sizeof(float);
    const size_t reduce = (size_t)64 * D * sizeof(float) + (size_t)kWaves * 2 * 64 * kTrStride * sizeof(uint16_t);
    const size_t expand = (size_t)64 * D * sizeof(float) + (size_t)groups * 2 * (2 * 2 * NB * 64) * sizeof(bf16x8);
    const size_t work = pass > reduce ? (pass > expand ? pass : expand) : (reduce > expand ? reduce : expand);
    return kRmax * sizeof(float) + 64 + stash + work;
}

// Waits (thread 0 polls) until `target` workgroups have counted themselves off at *counter.  False, for the
// whole workgroup, if the poll budget ran out or another workgroup of the launch has given up.
__device__ __forceinline__ bool wait_for_count(const LgParams& p, unsigned* counter, unsigned target, int* s_flag, int tid)
{
    if (tid == 0) {
        const bool ok = spin_until(counter, target, p.status, p.nonce, p.spin_limit);
        if (!ok) give_up(p.status, p.nonce);
        s_flag[0] = ok;
    }
    __syncthreads();
    const bool ok = s_flag[0] != 0;
    __syncthreads();
    return ok;
}
// Waits (thread 0 polls) until *word holds this launch's nonce: the pair's words and counters have been zeroed.
__device__ __forceinline__ bool wait_for_nonce(const LgParams& p, const unsigned long long* word, int* s_flag, int tid)
{
    if (tid == 0) {
        bool ok = false;
        for (uint32_t k = 0; k < p.spin_limit; ++k) {
            if (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.nonce) { ok = true; break; }
            if ((k & 63u) == 63u && gave_up(p.status, p.nonce)) break;
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok) give_up(p.status, p.nonce);
        s_flag[0] = ok;
    }
    __syncthreads();
    const bool ok = s_flag[0] != 0;
    __syncthreads();
    return ok;
}
// Counts the workgroup off at *counter once everything its wavefronts have stored or added has left them.
// Returns, to every thread, how many had counted themselves off before.
__device__ __forceinline__ unsigned count_off(unsigned* counter, int* s_flag, int tid)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) s_flag[1] = (int)__hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    return (unsigned)s_flag[1];
}

template <typename IO, int D>
__device__ __forceinline__ void poison_chunk(const LgParams& p, int g, int chunk)
{
    const int n = p.n_side[0];
    const int row0 = chunk * p.tiles_per_wg * kTileTokens, row1 = min(n, row0 + p.tiles_per_wg * kTileTokens);
    if (row1 <= row0) return;
    IO* base = reinterpret_cast<IO*>(p.out) + ((size_t)g * p.stride_side[0] + row0) * D;
    for (int e = threadIdx.x; e < (row1 - row0) * D; e += kThreads) {
        if constexpr (io_is_f32<IO>::value) as_global(base)[e] = __builtin_nanf("");
        else as_global(base)[e] = (uint16_t)0x7fc0u;
    }
}

// Workgroup (pair, chunk) = blockIdx.x: T passes over its chunk of its side, then (keys) its share of U and, for
// the last key workgroup of a problem to get there, Y''; (queries) the expansion of its chunk once Y'' is there.
// Every workgroup of the grid must be resident at once (the launcher checks the occupancy); every wait is
// bounded, marks the launch in the status words when it gives up, and a query workgroup that leaves early
// fills its rows of the output with NaN.
template <typename IO, int D>
__global__ void __launch_bounds__(kThreads, 2) lg_persistent(LgParams p)
{
    extern __shared__ __attribute__((aligned(16))) char s_all[];
    float* const s_g = reinterpret_cast<float*>(s_all);
    int* const s_flag = reinterpret_cast<int*>(s_all + kRmax * sizeof(float));
    char* const s_zstash = s_all + kRmax * sizeof(float) + 64;
    char* const s_work = s_zstash + (size_t)p.groups * StashBytes<IO, D, 2>::value;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pairs = 2 * p.G, T = p.T;
    const int pair = blockIdx.x / p.chunks, chunk = blockIdx.x % p.chunks;
    const int side = pair / p.G, g = pair % p.G, h = g % p.H;
    const float nside = (float)p.n_side[side];

    Frag<IO, D> xc;
    first_tile_of_pass<IO, D>(xc, p, pair, chunk, wave, lane);
    for (int t = tid; t < kRmax; t += kThreads) s_g[t] = t < p.r ? 0.f : kNegBig;
    stash_all_pivots<IO, D>(s_zstash, p.Z, h, p.r, p.groups, wave, lane);
    // No clearing launch: the first workgroup of a pair zeroes the pair's words of every pass (the keys' also the
    // problem's two counters) and then publishes the launch's nonce; the others wait for it before they add anything.
    unsigned long long* const ready = reinterpret_cast<unsigned long long*>(p.sync + 2 * (size_t)p.G);
    if (chunk == 0) {
        for (int k = 1; k <= T; ++k)
            for (int t = tid; t < kRmax; t += kThreads)
                __hip_atomic_store(p.colacc + ((size_t)k * pairs + pair) * kRmax + t, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (side == 1 && tid < 2) __hip_atomic_store(p.sync + 2 * g + tid, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (blockIdx.x == 0 && tid == 0)   // this launch; word 0, written only by a wait that gave up, cannot hold the same nonce
            __hip_atomic_store(p.status + 1, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) __hip_atomic_store(ready + pair, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if (!wait_for_nonce(p, ready + pair, s_flag, tid)) {
        if (side == 0) poison_chunk<IO, D>(p, g, chunk);
        return;
    }
    __syncthreads();

    for (int k = 1; k <= T; ++k) {
        pass_tiles<IO, D>(p, k, pair, chunk, s_g, reinterpret_cast<float (*)[kRmax]>(s_work), s_zstash, xc);
        if (k == T) break;
        first_tile_of_pass<IO, D>(xc, p, pair, chunk, wave, lane);
        unsigned long long word[kMaxGroups];
        const bool ok = wait_for_words(p, p.colacc + ((size_t)k * pairs + pair) * kRmax, word, s_flag, tid);
        if (!ok) {
            if (side == 0) poison_chunk<IO, D>(p, g, chunk);
            return;
        }
        // g^k = g^{k-1} + eps log(n beta / column sum), the same on every workgroup of the pair
        if (tid < 64) {
#pragma unroll
            for (int q = 0; q < kMaxGroups; ++q) {
                const int t = kGroup * q + tid;
                if (t < p.r) s_g[t] += p.eps * logf(nside * p.beta[h * p.r + t] / colsum_of(p, word[q]));
            }
        }
        __syncthreads();
    }
    // s_g = g^{T-1}, the potentials of the last pass: what the contraction and the expansion rebuild the weights from
    // (the rows' log-normalisers that the last pass stored are read back below)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    if (side == 1) {
        float* const s_buf = reinterpret_cast<float*>(s_work);
        uint16_t* const s_tr = reinterpret_cast<uint16_t*>(s_work + (size_t)64 * D * sizeof(float));
        for (int grp = 0; grp < p.groups; ++grp) {
            reduce_tiles<IO, D, true>(p, g, chunk, grp, s_g, s_buf, s_tr, s_zstash);
            __syncthreads();
        }
        // Y'' once every key workgroup of the problem has stored its share of U and the last column sums of both
        // sides are complete; each key workgroup forms the slice of Y'' that falls to it, four columns per thread
        count_off(p.sync + 2 * g, s_flag, tid);
        unsigned long long word[kMaxGroups];
        if (!wait_for_count(p, p.sync + 2 * g, (unsigned)p.chunks, s_flag, tid) ||
            !wait_for_words(p, p.colacc + ((size_t)T * pairs + g) * kRmax, word, s_flag, tid) ||
            !wait_for_words(p, p.colacc + ((size_t)T * pairs + p.G + g) * kRmax, word, s_flag, tid))
            return;
        const __amdgpu_buffer_rsrc_t v1 = coherent_view(p.colacc + ((size_t)T * pairs + g) * kRmax);
        const __amdgpu_buffer_rsrc_t v2 = coherent_view(p.colacc + ((size_t)T * pairs + p.G + g) * kRmax);
        const __amdgpu_buffer_rsrc_t uv = coherent_view(p.u_part + (size_t)g * p.chunks * kRmax * D);
        float* const ypp = p.ypp + (size_t)g * kRmax * D;
        for (int e4 = chunk * kThreads + tid; e4 < kRmax * D / 4; e4 += p.chunks * kThreads) {
            const int t = (4 * e4) / D;
            f32x4 u0 = {0.f, 0.f, 0.f, 0.f}, u1 = u0;
            float scale = 0.f;
            if (t < p.r) {
                const unsigned long long c1w = ldc_u64(v1, (uint32_t)t * 8u), c2w = ldc_u64(v2, (uint32_t)t * 8u);
                int c = 0;
#pragma unroll 4
                for (; c + 1 < p.chunks; c += 2) {
                    u0 += ldc_f32x4(uv, (uint32_t)(((size_t)c * kRmax * D + 4 * (size_t)e4) * sizeof(float)));
                    u1 += ldc_f32x4(uv, (uint32_t)(((size_t)(c + 1) * kRmax * D + 4 * (size_t)e4) * sizeof(float)));
                }
                if (c < p.chunks) u0 += ldc_f32x4(uv, (uint32_t)(((size_t)c * kRmax * D + 4 * (size_t)e4) * sizeof(float)));
                scale = ((float)p.n_side[0] * p.beta[h * p.r + t] / colsum_of(p, c1w)) / colsum_of(p, c2w);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) st_coherent(ypp + 4 * (size_t)e4 + q, scale * (u0[q] + u1[q]));
        }
        count_off(p.sync + 2 * g + 1, s_flag, tid);
        return;
    }

    // queries: wait for Y'' of the problem (its counter is valid once the keys' first workgroup has zeroed it), then
    // expand this chunk
    if (!wait_for_nonce(p, ready + p.G + g, s_flag, tid) ||
        !wait_for_count(p, p.sync + 2 * g + 1, (unsigned)p.chunks, s_flag, tid)) {
        poison_chunk<IO, D>(p, g, chunk);
        return;
    }
    float* const s_y = reinterpret_cast<float*>(s_work);
    bf16x8* const yf = reinterpret_cast<bf16x8*>(s_work + (size_t)64 * D * sizeof(float));
    expand_tiles<IO, D, true>(p, 0, g, chunk, p.Q, p.ypp, p.out, 0, s_g, s_y, s_zstash, yf);
}

template <typename IO, int D>
int launch_grouped(const Args& a, LgParams p)
{
    constexpr int NB = D / 32;
    hipStream_t st = a.stream;
    const int pairs = 2 * p.G, T = a.iters;
    const size_t words = (size_t)(T + 1) * pairs * kRmax;
    p.nonce = next_nonce();

    // The one-launch form, where the launches are what the call costs: the whole grid must be resident at once,
    // and a workgroup should have few tiles (the keys' workgroups alone contract with V there, group after group).
    if (!a.stepwise) {
        const size_t lds = persistent_lds_bytes<IO, D>(p.groups);
        static thread_local int per_cu_cache[8][kMaxGroups + 1] = {};   // per device ordinal and number of groups
        int dev = 0;
        LOT_HIP_CHECK(hipGetDevice(&dev));
        int per_cu = (dev >= 0 && dev < 8) ? per_cu_cache[dev][p.groups] : 0;
        if (per_cu == 0 && lds <= kPersistentLdsMax) {
            LOT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(lg_persistent<IO, D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            LOT_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, lg_persistent<IO, D>, kThreads, lds));
            if (per_cu < 1) per_cu = -1;
            if (dev >= 0 && dev < 8) per_cu_cache[dev][p.groups] = per_cu;
        }
        // (one workgroup per compute unit: with two, the one that polls holds up the one that still works -- measured)
        const long long capacity = per_cu > 0 ? (long long)device_cus() : 0;
        const int ntiles = (a.s.n + kTileTokens - 1) / kTileTokens;
        long long c = capacity / pairs;
        if (c > p.chunks) c = p.chunks;          // (the workspace holds that many shares of U per problem)
        if (c > 255) c = 255;                    // (the arrival count of a word is a byte)
        if (c >= 1) {
            int per = (int)((ntiles + c - 1) / c);
            per = (per + kWaves - 1) / kWaves * kWaves;
            if (per <= grouped_one_launch_tiles()) {
                LgParams q = p;
                q.tiles_per_wg = per;
                q.chunks = (ntiles + per - 1) / per;
                q.count_one = 1ull << kCountShiftLg;
                q.count_mask = 0xffull << kCountShiftLg;
                const int frac = kCountShiftLg - 2 - (int)std::ceil(std::log2((double)a.s.n + 1.0));
                q.fx_scale = std::ldexp(1.0f, frac);
                q.fx_unscale = std::ldexp(1.0f, -frac);
                q.status = (unsigned long long*)a.ws;
                q.sync = reinterpret_cast<unsigned*>(p.colacc + (size_t)(T + 1) * pairs * kRmax);
                q.spin_limit = spin_limit();
                lg_persistent<IO, D><<<(unsigned)pairs * q.chunks, kThreads, lds, st>>>(q);
                LOT_HIP_CHECK(hipGetLastError());
                return LOT_OK;
            }
        }
    }
    lg_clear<<<(unsigned)((words + 255) / 256), 256, 0, st>>>(p.colacc, words, (unsigned long long*)a.ws, p.nonce);
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
    w.colacc = take(((T + 1) * pairs * kRmax + lg_counter_words(G, T)) * 8);       // the words, then the counters of the one-launch form
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
    p.count_one = 0; p.count_mask = 0; p.status = nullptr; p.sync = nullptr; p.nonce = 0; p.spin_limit = 0;
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
