// Backward pass of LOT attention, tiled path (d_k = d_v in {32, 64}, r <= 64): the same gradients
// as the plain path, computed with the tile machinery of the fused forward kernel and without ever
// materialising anything of size n x r.
//
// What makes that possible.  Write, for one solve, W^k_it = softmax_t((C_it + g^{k-1}_t)/eps) (the
// row-normalised kernel of iteration k, so that the plan after the token-side update is a W^k with
// a = 1/n), cs^k_t = sum_i W^k_it, c^k = a cs^k, and M^k = (W^k)^T W^k (r x r).  Differentiating the
// pivot-side update g^k = g^{k-1} + eps log(beta / c^k) through the softmax gives, for the
// adjoints dg^k of the potentials and dc^k = -eps dg^k / c^k of the column sums,
//       dg^{k-1} = -(a/eps) M^k dc^k                                   (k = T-1 .. 1)
// so the whole reverse recursion over the iterations is a chain of r x r matrix-vector products,
// once the Gram matrices M^k have been accumulated during the forward passes.  The last step,
// where the coupling Gamma = a W^T Diag(beta / c^T) meets its incoming gradient dGamma, starts it:
//       s_t = sum_i dGamma_it Gamma_it,   dc^T_t = -s_t / c^T_t,
//       q_i = sum_t Gamma_it dGamma_it,   N_t = sum_i W^T_it q_i,
//       dg^{T-1} = -(1/eps) (N + a M^T dc^T).
// With every dc^k known, the gradient of the similarities is local to a token,
//       dC_it = (a/eps) sum_k W^k_it (dP^k_it - e^k_i),  dP^k = dc^k (k < T),  dP^T = dGamma beta/c^T + dc^T,
//       e^k_i = sum_t dP^k_it W^k_it,
// and is assembled tile by tile in registers, all T iterations of a tile at once, then contracted
// with Z (-> dQ, dK) and with the token rows (-> dZ) by MFMA before it is dropped.
// (Paper, "Learning": the pivots, their masses and the projections are trained by backpropagating
// through both Sinkhorn problems and the glued composition.  The derivation is this file's.)
//
// Launches:
//   forward sweep (T passes: column sums and Gram matrices; then the two token contractions
//   U = sum W2 V, Wd = sum W1 dO) | mid (Y', dYraw) together with the Gram reduce | glue (s, N, dV) |
//   recursion | assemble, all iterations at once (dQ, dK, dZ partials) | assemble, iteration by iteration
//   (only workgroups the former marked; every workgroup when there are more than 16 iterations) |
//   final (dZ, dbeta).
// The forward sweep is one persistent kernel when all its workgroups can be resident at once: the
// workgroups of a pair exchange their column sums through one integer atomic per pivot that also
// counts the contributors, and wait (bounded) for the count before the next pass; the write-out of
// the pass's Gram matrix sits between posting and waiting, so the exchange is rarely waited for.
// (The first workgroup of a pair zeroes the pair's words and says so under the launch's nonce; the
// others check that before their first post.)  Otherwise the sweep is a clearing launch and T + 1
// launches of the same tile code, with launch boundaries as the only synchronisation.  Both solves share every launch (pair = side * G + g, side 0 = queries).  All
// reductions have a fixed order except the column sums, which are exchanged as integers: results
// are reproducible.

#include "lot_internal.h"
#include "lot_tile.h"
#include "lot_tile_ops.h"

namespace lot {
namespace {

inline int target_wgs() { return 2 * device_cus(); }   // two workgroups of four wavefronts per compute unit

// Tiles per workgroup: enough workgroups to fill the device once (set-up and the cross-wavefront
// reductions at the end of a workgroup are amortised over more tiles, fewer partial results go
// through memory, and the forward sweep can stay one persistent kernel), a multiple of the wavefront
// count, between one and 256 tiles per wavefront.
inline int tiles_per_wg_for(const lot_shape& s)
{
    const long long ntiles = ((long long)s.n + kTileTokens - 1) / kTileTokens;
    const long long pairs = 2LL * s.B * s.H;
    const long long target = target_wgs();
    long long per = (ntiles * pairs + target - 1) / target;
    per = (per + kWaves - 1) / kWaves * kWaves;
    if (per < kWaves) per = kWaves;
    if (per > 256 * kWaves) per = 256 * kWaves;
    return (int)per;
}

constexpr int kMaxTiledIters = 64;   // the recursion and the assembly keep per-iteration vectors of 64 pivots in LDS

struct BtParams {
    const void* Q; const void* K; const void* V; const void* dO;
    const float* Z; const float* beta;
    void* dQ; void* dK; void* dV;
    float* dZ; float* dbeta;
    unsigned long long* status;   // [0] = nonce of a launch in which a wait gave up, [1] = nonce of the last launch
    unsigned long long nonce;
    unsigned long long* colacc;   // [T+1][pairs][64] column sums of W^k (k = 1..T): contributors << 56 | fixed point
    float* ghist;                 // [T+1][pairs][64] g^k, k = 0..T-1 (padding pivots: -1e30)
    float* gram_part;             // [T][pairs][chunks][R2]
    float* gram_full;             // [T][pairs][R2]
    float* u_part;                // [pairs][chunks][64][D]   side 1: sum W2 V, side 0: sum W1 dO
    float* yp;                    // [G][64][D]  Y'
    float* dyraw;                 // [G][64][D]  dY' / beta
    float* sn_part;               // [pairs][chunks][2][64]
    float* dcs;                   // [T+1][pairs][64]  dc^k, k = 1..T
    float* rhop;                  // [pairs][64]  beta_t / cs^T_t
    float* db_pair;               // [pairs][64]
    float* db_glue;               // [G][64]
    float* dz_part;               // [pairs][chunks][64][D]
    unsigned* redo;               // [pairs][chunks]  workgroups whose tiles the assemble kernel redoes iteration by iteration
    unsigned long long* cleared;  // [pairs]  nonce of the launch whose sweep has zeroed the pair's column sums
    int G, H, B, r, chunks, tiles_per_wg, k, T;
    // per side (0 = queries, dO, dQ; 1 = keys, values, dK, dV):
    int n_side[2];                // tokens per problem
    int stride_side[2];           // tokens between consecutive problems in the caller's tensors (>= n_side)
    const float* mass_side[2];    // [G][n_side] token masses, or null: uniform 1/n_side
    float eps, fx_scale, fx_unscale;
    uint32_t spin_limit;
    float sum_lo, sum_hi;         // row sums outside [sum_lo, sum_hi] make the assemble kernel re-shift its rows
};

template <typename IO> __device__ __forceinline__ const IO* rows_of(const BtParams& p, int side)
{
    return reinterpret_cast<const IO*>(side == 0 ? p.Q : p.K);
}

// Mass of a token times the number of tokens of its side (1 for uniform masses).
__device__ __forceinline__ float token_weight(const BtParams& p, int side, int g, int tok)
{
    const float* m = p.mass_side[side];
    return m ? (float)p.n_side[side] * as_global(m)[(size_t)g * p.n_side[side] + tok] : 1.f;
}

// A column-sum word: the number of workgroups that have contributed in the top byte, their fixed-point
// sum below.
constexpr int kCountShift = 56;
constexpr unsigned long long kSumMask = (1ull << kCountShift) - 1;
__device__ __forceinline__ float colsum_of(unsigned long long word, float unscale)
{
    // a sum below the fixed-point resolution reads as half a unit, not as (almost) nothing: the potentials
    // then move by a bounded amount and the couplings of a starved pivot stay bounded
    return fmaxf((float)(long long)(word & kSumMask) * unscale, 0.5f * unscale);
}

// ---------------------------------------------------------------------------------------------
// forward sweep.  A pass k accumulates the column sums and the Gram matrix of W^k over the
// workgroup's tiles; the contraction pass (run once, with the potentials of pass T) accumulates the
// token contraction of W^T with V (keys) or dO (queries) instead -- kept apart because the two sets
// of accumulators do not fit the register file together.
// ---------------------------------------------------------------------------------------------
template <typename IO, int D, int RB> struct SweepShared {
    float g[64];                                   // g^{k-1}
    float cs[kWaves][64];
    // (sized for the 32 RB pivots in use: with r <= 32 three workgroups then fit a compute unit's local memory)
    static constexpr int kR = 32 * RB;
    __attribute__((aligned(16))) float buf[kR * kR > kR * D ? kR * kR : kR * D];    // a Gram matrix, or a [pivot][D] sum
    __attribute__((aligned(16))) uint16_t tr[kWaves * 2 * kR * kTrStride];
    __attribute__((aligned(16))) char zstash[PivotStashBytes<IO, D, RB>::value];
    static_assert(kWaves * 2 * kR * kTrStride * sizeof(uint16_t) >= kR * kR * sizeof(float),
                  "the transposition area doubles as the second buffer of the Gram reduction");
};

// Where a workgroup of the sweep works
struct SweepPlace {
    int pair, chunk, side, g, h, tile_begin, tile_end;
};
__device__ __forceinline__ SweepPlace sweep_place(const BtParams& p)
{
    SweepPlace w;
    w.pair = blockIdx.x / p.chunks; w.chunk = blockIdx.x % p.chunks;
    w.side = w.pair / p.G; w.g = w.pair % p.G; w.h = w.g % p.H;
    const int ntiles = (p.n_side[w.side] + kTileTokens - 1) / kTileTokens;
    w.tile_begin = w.chunk * p.tiles_per_wg;
    w.tile_end = min(ntiles, w.tile_begin + p.tiles_per_wg);
    return w;
}

// MASS = false: the launch has no token masses; every token weight is the constant 1.
template <typename IO, int D, bool MASS>
__device__ __forceinline__ void load_first_tile(Frag<IO, D>& xc, float& mc, const BtParams& p, const SweepPlace& w,
                                                const IO* X, int wave, int i, int kg)
{
    const int tok = min((w.tile_begin + wave) * kTileTokens + i, p.n_side[w.side] - 1);
    load_tokens<D>(xc, X + ((size_t)w.g * p.stride_side[w.side] + tok) * D, kg);
    mc = MASS ? token_weight(p, w.side, w.g, tok) : 1.f;
}

template <typename IO, int D, int RB>
__device__ __forceinline__ void stash_head_pivots(const BtParams& p, int h, char* zstash, int lane)
{
    const int i = lane & 31, kg = lane >> 5;
    Frag<IO, D> z0[RB];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb) {
        const int t = 32 * mb + i;
        load_pivots<D>(z0[mb], p.Z + ((size_t)h * p.r + min(t, p.r - 1)) * D, kg, t < p.r);
    }
    stash_similarity_pivots<IO, D, RB>(zstash, z0, lane);
}

// One pass over the wavefront's tiles with the potentials in sh.g.  xc and mc hold the first tile's
// rows and token weights on entry and, when `again`, once more on return (requested during the last
// tile, so that the next pass does not start with a round trip to memory).  The token weights (mass
// times n, 1 if uniform) multiply the column sums, the Gram matrix (as square roots on both factors)
// and the key side's contraction with V; the query side's contraction with dO is unweighted.
template <typename IO, int D, int RB, bool WITH_U, bool MASS>
__device__ __forceinline__ void sweep_tiles(const BtParams& p, const SweepPlace& w, const IO* X, const IO* vals,
                                            SweepShared<IO, D, RB>& sh, Frag<IO, D>& xc, float& mc, bool again,
                                            int wave, int lane, float c1,
                                            f32x16 (&cs)[RB], f32x16 (&Gm)[RB][RB], f32x16 (&U)[RB][D / 32])
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    const int i = lane & 31, kg = lane >> 5, n = p.n_side[w.side], stride = p.stride_side[w.side];
    uint16_t* tr_hi = sh.tr + (wave * 2 + 0) * 32 * RB * kTrStride;
    uint16_t* tr_lo = sh.tr + (wave * 2 + 1) * 32 * RB * kTrStride;
    for (int tile = w.tile_begin + wave; tile < w.tile_end; tile += kWaves) {
        Frag<IO, D> xn = xc;
        float mn = mc;
        if (tile + kWaves < w.tile_end) {
            const int tok = min((tile + kWaves) * kTileTokens + i, n - 1);
            load_tokens<D>(xn, X + ((size_t)w.g * stride + tok) * D, kg);
            if (MASS) mn = token_weight(p, w.side, w.g, tok);
        } else if (again) {
            load_first_tile<IO, D, MASS>(xn, mn, p, w, X, wave, i, kg);
        }
        bf16x8 vh[2][NB], vl[2][NB];
        if (WITH_U) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
                const int left = max(1, min(8, n - t0));
                load_values<D>(vh[s], vl[s], vals, (size_t)w.g * stride + min(t0, n - 1), left, i);
            }
        }
        f32x16 acc[RB];
        float wt;
        tile_weights<IO, D, RB>(acc, wt, sh.zstash, xc, sh.g, lane, c1, tile * kTileTokens + i < n);
        // what goes through the transposition: W sqrt(m) for the Gram matrix, W m for the keys'
        // contraction with V, W for the queries' contraction with dO
        const float wcs = MASS ? wt * mc : wt;
        const float wtr = !MASS ? wt : WITH_U ? (w.side == 1 ? wcs : wt) : wt * __builtin_amdgcn_sqrtf(mc);
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (!WITH_U) cs[mb][j] = fmaf(acc[mb][j], wcs, cs[mb][j]);
                acc[mb][j] *= wtr;
            }
        // bf16 I/O: the Gram matrix takes its weights as fp16 (the recursion through the iterations divides
        // by the column sums, so pivots of small mass feel the rounding of their few weights)
        constexpr bool kHalfGram = !WITH_U && !kSplit;
        transpose_tile<RB, kSplit, kHalfGram>(acc, tr_hi, tr_lo, i, kg);
        if (WITH_U) contract_tokens<D, RB, kSplit>(U, tr_hi, tr_lo, vh, vl, i, kg);
        else contract_gram<RB, kSplit, kHalfGram>(Gm, tr_hi, tr_lo, i, kg);
        transpose_done();
        xc = xn;
        mc = mn;
    }
}

// The same pass for a workgroup none of whose wavefronts has more than KEEP tiles: the similarities C_it of the
// wavefront's tiles stay in registers from the first pass on (ck, and the token weights in mk), so the later
// passes and the contraction pass read no token rows and run no similarity product -- which with fp32 I/O is
// most of a pass (six bf16 products over the pieces of every row, and cutting the rows into them).  `first`:
// compute them (the rows of all KEEP tiles are requested together).  The weights are formed as (C + g), where the
// pass above lets the product accumulate onto g: the two differ by rounding (1e-7), which is why a shape runs all
// its passes in one of the two forms.
template <typename IO, int D, int RB, bool WITH_U, bool MASS, int KEEP>
__device__ __forceinline__ void sweep_kept_tiles(const BtParams& p, const SweepPlace& w, const IO* X, const IO* vals,
                                                 SweepShared<IO, D, RB>& sh, bool first, int wave, int lane, float c1,
                                                 f32x16 (&ck)[KEEP][RB], float (&mk)[KEEP],
                                                 f32x16 (&cs)[RB], f32x16 (&Gm)[RB][RB], f32x16 (&U)[RB][D / 32])
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    const int i = lane & 31, kg = lane >> 5, n = p.n_side[w.side], stride = p.stride_side[w.side];
    uint16_t* tr_hi = sh.tr + (wave * 2 + 0) * 32 * RB * kTrStride;
    uint16_t* tr_lo = sh.tr + (wave * 2 + 1) * 32 * RB * kTrStride;
    if (first) {
        Frag<IO, D> xs[KEEP];
#pragma unroll
        for (int slot = 0; slot < KEEP; ++slot) {
            const int tile = w.tile_begin + wave + slot * kWaves;
            const int tok = min(tile * kTileTokens + i, n - 1);
            if (tile < w.tile_end) {
                load_tokens<D>(xs[slot], X + ((size_t)w.g * stride + tok) * D, kg);
                mk[slot] = MASS ? token_weight(p, w.side, w.g, tok) : 1.f;
            }
        }
#pragma unroll
        for (int slot = 0; slot < KEEP; ++slot) {
            const int tile = w.tile_begin + wave + slot * kWaves;
            if (tile < w.tile_end) {
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) ck[slot][mb][j] = 0.f;
                int skew = 0;
                asm volatile("" : "+v"(skew));
                similarity_stashed<IO, D, RB>(ck[slot], sh.zstash, xs[slot], lane, skew);
            }
        }
    }
#pragma unroll
    for (int slot = 0; slot < KEEP; ++slot) {
        const int tile = w.tile_begin + wave + slot * kWaves;
        if (tile < w.tile_end) {
            bf16x8 vh[2][NB], vl[2][NB];
            if (WITH_U) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
                    const int left = max(1, min(8, n - t0));
                    load_values<D>(vh[s], vl[s], vals, (size_t)w.g * stride + min(t0, n - 1), left, i);
                }
            }
            f32x16 acc[RB];
            float wt;
            tile_weights_from_similarities<RB>(acc, wt, ck[slot], sh.g, lane, c1, tile * kTileTokens + i < n);
            const float mc = mk[slot];
            const float wcs = MASS ? wt * mc : wt;
            const float wtr = !MASS ? wt : WITH_U ? (w.side == 1 ? wcs : wt) : wt * __builtin_amdgcn_sqrtf(mc);
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    if (!WITH_U) cs[mb][j] = fmaf(acc[mb][j], wcs, cs[mb][j]);
                    acc[mb][j] *= wtr;
                }
            constexpr bool kHalfGram = !WITH_U && !kSplit;
            transpose_tile<RB, kSplit, kHalfGram>(acc, tr_hi, tr_lo, i, kg);
            if (WITH_U) contract_tokens<D, RB, kSplit>(U, tr_hi, tr_lo, vh, vl, i, kg);
            else contract_gram<RB, kSplit, kHalfGram>(Gm, tr_hi, tr_lo, i, kg);
            transpose_done();
        }
    }
}

// End of pass k: the workgroup's column sums go to one integer atomic per pivot (which also counts
// the workgroup), its Gram matrix to this chunk's slot of gram_part.  Contains barriers.
// Only the blocks on and above the diagonal of the (symmetric) Gram matrix are accumulated and
// written; the reduction over the chunks mirrors them.
template <typename IO, int D, int RB>
__device__ __forceinline__ void finish_pass(const BtParams& p, const SweepPlace& w, SweepShared<IO, D, RB>& sh, int k,
                                            int tid, int wave, int lane, const f32x16 (&cs)[RB], const f32x16 (&Gm)[RB][RB])
{
    constexpr int R = 32 * RB;
    const int i = lane & 31, kg = lane >> 5, pairs = 2 * p.G;
    // column sums: one pivot per lane, then across the wavefronts
    {
        float c[16 * RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) c[16 * mb + j] = cs[mb][j];
        const float total = reduce_scatter_tokens<16 * RB>(c, i);
        const int q = RB == 2 ? i : i >> 1;
        sh.cs[wave][32 * (q >> 4) + 8 * ((q & 15) >> 2) + 4 * kg + (q & 3)] = total;
        if (RB == 1) sh.cs[wave][32 + lane % 32] = 0.f;
    }
    __syncthreads();      // every wavefront has also left its tile loop: sh.tr is free
    if (tid < 64) {
        float tot = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) tot += sh.cs[wv][tid];
        const unsigned long long word = (1ull << kCountShift) + (unsigned long long)__float2ll_rn(tot * p.fx_scale);
        __hip_atomic_fetch_add(p.colacc + ((size_t)k * pairs + w.pair) * 64 + tid, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // Gram matrix, block (mb, mb2): rows t = pivot_of(mb, j, kg), columns t' = 32 mb2 + i.  Wavefronts
    // 0 and 1 lay theirs down in two buffers, 2 and 3 add to them, the write-out adds the buffers.
    float* const bufs[2] = {sh.buf, reinterpret_cast<float*>(sh.tr)};
    for (int turn = 0; turn < 2; ++turn) {
        if ((wave >> 1) == turn) {
            float* const b = bufs[wave & 1];
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int mb2 = mb; mb2 < RB; ++mb2)
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        float* dst = &b[pivot_of(mb, j, kg) * R + 32 * mb2 + i];
                        *dst = turn == 0 ? Gm[mb][mb2][j] : *dst + Gm[mb][mb2][j];
                    }
        }
        __syncthreads();
    }
    if (p.chunks == 1) {
        // the only workgroup of its pair: its matrix is the pair's, written whole (blocks above the diagonal
        // also to their mirror image) where the recursion reads it; no reduction launch follows
        float* gf = p.gram_full + ((size_t)(k - 1) * pairs + w.pair) * R * R;
        for (int e = tid; e < R * R; e += kThreads) {
            const int row = e / R, col = e % R;
            if (col / 32 < row / 32) continue;
            const float v = bufs[0][e] + bufs[1][e];
            gf[e] = v;
            if (col / 32 > row / 32) gf[col * R + row] = v;
        }
        return;
    }
    float* gp = p.gram_part + (((size_t)(k - 1) * pairs + w.pair) * p.chunks + w.chunk) * R * R;
    for (int e = tid; e < R * R; e += kThreads)
        if (e % R / 32 >= e / R / 32) gp[e] = bufs[0][e] + bufs[1][e];
}

template <typename IO, int D, int RB>
__device__ __forceinline__ void finish_contraction(const BtParams& p, const SweepPlace& w, SweepShared<IO, D, RB>& sh,
                                                   int tid, int wave, int lane, const f32x16 (&U)[RB][D / 32])
{
    sum_over_waves<D, RB>(U, sh.buf, wave, lane & 31, lane >> 5);
    float* up = p.u_part + ((size_t)w.pair * p.chunks + w.chunk) * 64 * D;
    for (int e = tid; e < 32 * RB * D; e += kThreads) up[e] = sh.buf[e];
}

template <int RB, int NB>
__device__ __forceinline__ void zero_pass(f32x16 (&cs)[RB], f32x16 (&Gm)[RB][RB])
{
#pragma unroll
    for (int mb = 0; mb < RB; ++mb) {
#pragma unroll
        for (int j = 0; j < 16; ++j) cs[mb][j] = 0.f;
#pragma unroll
        for (int mb2 = 0; mb2 < RB; ++mb2)
#pragma unroll
            for (int j = 0; j < 16; ++j) Gm[mb][mb2][j] = 0.f;
    }
}

// g^k from g^{k-1} and the complete column sums of pass k
__device__ __forceinline__ float next_potential(const BtParams& p, int side, float g_prev, unsigned long long word, int h, int t)
{
    return g_prev + p.eps * logf((float)p.n_side[side] * p.beta[h * p.r + t] / colsum_of(word, p.fx_unscale));
}

// One pass per launch (WITH_U = false: pass p.k; true: the contraction pass), for grids that cannot
// be resident at once.
template <typename IO, int D, int RB, bool WITH_U, bool MASS>
__global__ void __launch_bounds__(kThreads, 2) bt_forward(BtParams p)
{
    constexpr int NB = D / 32;
    __shared__ SweepShared<IO, D, RB> sh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const SweepPlace w = sweep_place(p);
    const int pairs = 2 * p.G, r = p.r, k = p.k;
    const IO* X = rows_of<IO>(p, w.side);

    // the first tile is requested before anything else: its latency overlaps the set-up
    Frag<IO, D> xc;
    float mc;
    load_first_tile<IO, D, MASS>(xc, mc, p, w, X, wave, lane & 31, lane >> 5);

    // g^{k-1} from the column sums of the previous launch
    if (tid < 64) {
        float gv = tid < r ? 0.f : kNegBig;
        if (k > 1 && tid < r)
            gv = next_potential(p, w.side, p.ghist[((size_t)(k - 2) * pairs + w.pair) * 64 + tid],
                                p.colacc[((size_t)(k - 1) * pairs + w.pair) * 64 + tid], w.h, tid);
        sh.g[tid] = gv;
        if (!WITH_U && w.chunk == 0) p.ghist[((size_t)(k - 1) * pairs + w.pair) * 64 + tid] = gv;
    }
    if (wave == 0) stash_head_pivots<IO, D, RB>(p, w.h, sh.zstash, lane);
    __syncthreads();

    f32x16 cs[RB], Gm[RB][RB], U[RB][NB];
    zero_pass<RB, NB>(cs, Gm);
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 16; ++j) U[mb][nb][j] = 0.f;
    const IO* vals = reinterpret_cast<const IO*>(w.side == 0 ? p.dO : p.V);
    const float c1 = kLog2e / p.eps;
    sweep_tiles<IO, D, RB, WITH_U, MASS>(p, w, X, vals, sh, xc, mc, false, wave, lane, c1, cs, Gm, U);
    if (WITH_U) finish_contraction<IO, D, RB>(p, w, sh, tid, wave, lane, U);
    else finish_pass<IO, D, RB>(p, w, sh, k, tid, wave, lane, cs, Gm);
}

// All T passes and the contraction pass in one launch.  Requires every workgroup of a pair to be
// resident together (the host checks the grid against the device's capacity); the waits are bounded
// all the same, and a wait that runs out marks the status word and ends the workgroup.
template <typename IO, int D, int RB, bool MASS, int KEEP = 0>
__global__ void __launch_bounds__(kThreads, 2) bt_sweep(BtParams p)
{
    constexpr int NB = D / 32;
    __shared__ SweepShared<IO, D, RB> sh;
    __shared__ int s_ok;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const SweepPlace w = sweep_place(p);
    const int pairs = 2 * p.G, r = p.r, T = p.T;
    const IO* X = rows_of<IO>(p, w.side);
    const float c1 = kLog2e / p.eps;

    Frag<IO, D> xc;
    float mc = 1.f;
    if constexpr (KEEP == 0) load_first_tile<IO, D, MASS>(xc, mc, p, w, X, wave, lane & 31, lane >> 5);
    f32x16 ck[KEEP > 0 ? KEEP : 1][RB];      // KEEP > 0: the similarities of this wavefront's tiles, from the first pass on
    float mk[KEEP > 0 ? KEEP : 1];
    if (wave == 0) stash_head_pivots<IO, D, RB>(p, w.h, sh.zstash, lane);
    if (tid == 0) s_ok = 1;
    float gv = tid < r ? 0.f : kNegBig;     // g^{k-1}_t, carried by thread t < 64
    if (blockIdx.x == 0 && tid == 0)
        __hip_atomic_store(p.status + 1, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // this launch
    if (w.chunk == 0) {
        // The first workgroup of a pair zeroes the pair's column sums of every pass and announces it
        // under this launch's nonce; the others wait for that before their first post, a whole pass
        // later.  (No separate clearing launch.)
        for (int e = tid; e < (T + 1) * 64; e += kThreads)
            __hip_atomic_store(p.colacc + ((size_t)(e >> 6) * pairs + w.pair) * 64 + (e & 63), 0ull, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        publish_barrier();   // the zeroes have been acknowledged
        if (tid == 0) __hip_atomic_store(p.cleared + w.pair, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    for (int k = 1; k <= T; ++k) {
        if (tid < 64) {
            if (k > 1) {
                // the column sums of pass k-1 are complete once every chunk has been counted
                const unsigned long long* src = p.colacc + ((size_t)(k - 1) * pairs + w.pair) * 64 + tid;
                unsigned long long word = 0;
                bool done = false;
                for (uint32_t it = 0; it < p.spin_limit; ++it) {
                    word = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    done = (int)(word >> kCountShift) == p.chunks;
                    if (__all(done)) break;
                    if ((it & 63u) == 63u && __hip_atomic_load(p.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.nonce) break;
                    __builtin_amdgcn_s_sleep(1);
                }
                if (!__all(done)) {
                    if (tid == 0) {
                        __hip_atomic_store(p.status, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        s_ok = 0;
                    }
                } else if (tid < r) {
                    gv = next_potential(p, w.side, gv, word, w.h, tid);
                }
            }
            sh.g[tid] = gv;
            if (w.chunk == 0) p.ghist[((size_t)(k - 1) * pairs + w.pair) * 64 + tid] = gv;
        }
        __syncthreads();      // also: the previous pass's write-out has finished with sh.buf and sh.tr
        if (!s_ok) return;
        f32x16 cs[RB], Gm[RB][RB], U[RB][NB];
        zero_pass<RB, NB>(cs, Gm);
        if constexpr (KEEP > 0) sweep_kept_tiles<IO, D, RB, false, MASS, KEEP>(p, w, X, nullptr, sh, k == 1, wave, lane, c1, ck, mk, cs, Gm, U);
        else sweep_tiles<IO, D, RB, false, MASS>(p, w, X, nullptr, sh, xc, mc, true, wave, lane, c1, cs, Gm, U);
        if (k == 1 && w.chunk != 0) {
            // first post of this launch: the pair's column sums must have been zeroed
            if (tid == 0) {
                bool ok = false;
                for (uint32_t it = 0; it < p.spin_limit; ++it) {
                    if (__hip_atomic_load(p.cleared + w.pair, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.nonce) { ok = true; break; }
                    if ((it & 63u) == 63u && __hip_atomic_load(p.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.nonce) break;
                    __builtin_amdgcn_s_sleep(1);
                }
                if (!ok) {
                    __hip_atomic_store(p.status, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_ok = 0;
                }
            }
            __syncthreads();
            if (!s_ok) return;
        }
        finish_pass<IO, D, RB>(p, w, sh, k, tid, wave, lane, cs, Gm);
    }
    __syncthreads();
    {
        f32x16 cs[RB], Gm[RB][RB], U[RB][NB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 16; ++j) U[mb][nb][j] = 0.f;
        const IO* vals = reinterpret_cast<const IO*>(w.side == 0 ? p.dO : p.V);
        if constexpr (KEEP > 0) sweep_kept_tiles<IO, D, RB, true, MASS, KEEP>(p, w, X, vals, sh, false, wave, lane, c1, ck, mk, cs, Gm, U);
        else sweep_tiles<IO, D, RB, true, MASS>(p, w, X, vals, sh, xc, mc, false, wave, lane, c1, cs, Gm, U);
        __syncthreads();
        finish_contraction<IO, D, RB>(p, w, sh, tid, wave, lane, U);
    }
}

// ---------------------------------------------------------------------------------------------
// mid: Y'_t = U_t / cs2_t, dYraw_t = n Wd_t / cs1_t, db_glue_t = -<dYraw_t, Y'_t>, rho'_t = beta_t / cs_t
// ---------------------------------------------------------------------------------------------
// One thread per (g, t, four columns): sums the per-chunk contractions in chunk order; the D / 4 threads of a
// (g, t) row are adjacent lanes of one wavefront, so the row's dot product <dYraw_t, Y'_t> is a
// butterfly sum over them and lane 0 of the row writes the per-pivot numbers.
template <int D>
__device__ __forceinline__ void mid_body(const BtParams& p, int block)
{
    const int idx = block * blockDim.x + threadIdx.x;      // the blocks cover G * 64 * D / 4 exactly: whole wavefronts
    const int g = idx / (16 * D), e = (idx % (16 * D)) * 4, t = e / D;
    const int pairs = 2 * p.G, T = p.T;
    f32x4 y = {0.f, 0.f, 0.f, 0.f}, dy = y;
    float r1 = 0.f, r2 = 0.f;
    if (t < p.r) {
        f32x4 u0 = y, u1 = y, w0 = y, w1 = y;     // two interleaved chains each: the loads overlap
        const f32x4* wp = reinterpret_cast<const f32x4*>(p.u_part + ((size_t)(0 * p.G + g) * p.chunks) * 64 * D + e);
        const f32x4* up = reinterpret_cast<const f32x4*>(p.u_part + ((size_t)(1 * p.G + g) * p.chunks) * 64 * D + e);
        constexpr int kStep = 16 * D;             // f32x4 words between consecutive chunks
        int c = 0;
        for (; c + 1 < p.chunks; c += 2) {
            w0 += wp[(size_t)c * kStep]; w1 += wp[(size_t)(c + 1) * kStep];
            u0 += up[(size_t)c * kStep]; u1 += up[(size_t)(c + 1) * kStep];
        }
        if (c < p.chunks) { w0 += wp[(size_t)c * kStep]; u0 += up[(size_t)c * kStep]; }
        const float cs1 = colsum_of(p.colacc[((size_t)T * pairs + g) * 64 + t], p.fx_unscale);
        const float cs2 = colsum_of(p.colacc[((size_t)T * pairs + p.G + g) * 64 + t], p.fx_unscale);
        const float ns = (float)p.n_side[0];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            y[q] = (u0[q] + u1[q]) / cs2;
            dy[q] = ns * (w0[q] + w1[q]) / cs1;
        }
        const float b = p.beta[(g % p.H) * p.r + t];
        r1 = b / cs1;
        r2 = b / cs2;
    }
    reinterpret_cast<f32x4*>(p.yp)[idx] = y;
    reinterpret_cast<f32x4*>(p.dyraw)[idx] = dy;
    float dot = (dy[0] * y[0] + dy[1] * y[1]) + (dy[2] * y[2] + dy[3] * y[3]);
#pragma unroll
    for (int o = D / 8; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
    if (e % D == 0) {
        p.db_glue[g * 64 + t] = -dot;
        p.rhop[(size_t)g * 64 + t] = r1;
        p.rhop[(size_t)(p.G + g) * 64 + t] = r2;
    }
}

// ---------------------------------------------------------------------------------------------
// glue: per tile the incoming gradient of the coupling, dGamma1_it = n <dO_i, Y'_t> (queries) or
// dGamma2_jt = <V_j, dYraw_t> (keys), and from it s_t, q_i, N_t; the key side also writes
// dV_j = sum_t Gamma2_jt dYraw_t.
// ---------------------------------------------------------------------------------------------
template <typename IO, int D, int RB>
__global__ void __launch_bounds__(kThreads, 2) bt_glue(BtParams p)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    __shared__ float s_g[64], s_rho[64];
    __shared__ float s_part[kWaves][2][64];
    __shared__ __attribute__((aligned(16))) float s_y[64 * D];
    __shared__ __attribute__((aligned(16))) bf16x8 s_yf[2][2 * RB * NB * 64];
    __shared__ __attribute__((aligned(16))) char s_zstash[PivotStashBytes<IO, D, RB>::value];
    constexpr bool kYPieces = true;   // the matrix operand of the dGamma product as bf16 pieces (fp32 I/O)
    __shared__ __attribute__((aligned(16))) char s_ystash[PivotStashBytes<IO, D, RB, kYPieces>::value];
    // bf16 I/O: what the bf16 rounding of that operand leaves out (see the incoming-gradient tile below)
    __shared__ __attribute__((aligned(16))) char s_ystash_lo[kSplit ? 16 : StashBytes<IO, D, RB>::value];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.G;
    const int pair = blockIdx.x / p.chunks, chunk = blockIdx.x % p.chunks;
    const int side = pair / p.G, g = pair % p.G, h = g % p.H;
    const int n = p.n_side[side], stride = p.stride_side[side], r = p.r, T = p.T;
    const bool weighted = side == 1 && p.mass_side[1] != nullptr;    // dGamma2 and dV carry the keys' masses
    const float c1 = kLog2e / p.eps;
    const IO* X = rows_of<IO>(p, side);
    const IO* vals = reinterpret_cast<const IO*>(side == 0 ? p.dO : p.V);
    // the matrix whose rows meet the value rows: n Y' for the queries, dYraw for the keys
    const float* ymat = (side == 0 ? p.yp : p.dyraw) + (size_t)g * 64 * D;
    const float yscale = side == 0 ? (float)n : 1.f;

    // (requested with the rest of the set-up's loads, kept in registers until the staging area is free)
    constexpr int kMatPer = 64 * D / kThreads;
    float yreg[kMatPer];
#pragma unroll
    for (int q = 0; q < kMatPer; ++q) yreg[q] = ymat[tid + q * kThreads] * yscale;
    if (tid < 64) {
        s_g[tid] = p.ghist[((size_t)(T - 1) * pairs + pair) * 64 + tid];
        s_rho[tid] = p.rhop[(size_t)pair * 64 + tid];
    }
    if (wave == 0) {
        Frag<IO, D> z0[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            const int t = 32 * mb + i;
            load_pivots<D>(z0[mb], p.Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
        }
        stash_similarity_pivots<IO, D, RB>(s_zstash, z0, lane);
    }
    // keys: the expansion to dV needs rho'_t dYraw_t as B fragments
    if (side == 1) {
        for (int e = tid; e < 64 * D; e += kThreads) s_y[e] = p.dyraw[(size_t)g * 64 * D + e] * p.rhop[(size_t)pair * 64 + e / D];
    } else {
        for (int e = tid; e < 64 * D; e += kThreads) s_y[e] = 0.f;
    }
    __syncthreads();
    lay_out_fragments<D, RB>(s_y, s_yf[0], s_yf[1], tid);
    __syncthreads();
    // rows of ymat as the "pivot" operand of the similarity MFMA (scaled), via LDS staging
#pragma unroll
    for (int q = 0; q < kMatPer; ++q) s_y[tid + q * kThreads] = yreg[q];
    __syncthreads();
    if (wave == 0) {
        Frag<IO, D> y0[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) load_pivots_lds<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
        stash_similarity_pivots<IO, D, RB, kYPieces>(s_ystash, y0, lane);
        if (!kSplit) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb) load_pivots_lds_lo<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
            stash_pivots<D, RB>(s_ystash_lo, y0, lane);
        }
    }
    __syncthreads();

    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.tiles_per_wg);
    f32x16 sacc[RB], nacc[RB];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) { sacc[mb][j] = 0.f; nacc[mb][j] = 0.f; }

    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        const int tok = min(tile * kTileTokens + i, n - 1);
        Frag<IO, D> xc, vc;
        load_tokens<D>(xc, X + ((size_t)g * stride + tok) * D, kg);
        load_tokens<D>(vc, vals + ((size_t)g * stride + tok) * D, kg);
        const float m = weighted ? token_weight(p, 1, g, tok) : 1.f;
        f32x16 acc[RB], dgam[RB], rho[RB];
        float w;
        int skew = 0;
        asm volatile("" : "+v"(skew));
        {
            tile_weights<IO, D, RB>(acc, w, s_zstash, xc, s_g, lane, c1, tile * kTileTokens + i < n);
        }
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) { acc[mb][j] *= w; dgam[mb][j] = 0.f; }
        {
            // The incoming gradient of the coupling.  s, q and N below meet in differences (N - P s) that
            // are an order of magnitude smaller than their terms, so with bf16 I/O the matrix operand is
            // taken as bf16 hi + lo (two products): its rounding would otherwise show in dbeta.
            similarity_stashed<IO, D, RB, kYPieces>(dgam, s_ystash, vc, lane, skew);
            if (!kSplit) similarity_stashed<IO, D, RB, kYPieces>(dgam, s_ystash_lo, vc, lane, skew);
        }
        if (weighted) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) dgam[mb][j] *= m;
        }
        load_pivot_vector<RB>(rho, s_rho + skew, kg);
        // q_i = sum_t Gamma_it dGamma_it with Gamma_it = W_it rho'_t
        float q0 = 0.f, q1 = 0.f;
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; j += 2) {
                const float a0 = acc[mb][j] * dgam[mb][j], a1 = acc[mb][j + 1] * dgam[mb][j + 1];
                sacc[mb][j] += a0; sacc[mb][j + 1] += a1;          // s_t / rho'_t, scaled at the end
                q0 = fmaf(a0, rho[mb][j], q0);
                q1 = fmaf(a1, rho[mb][j + 1], q1);
            }
        const float q = pair_sum(q0 + q1);
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) nacc[mb][j] = fmaf(acc[mb][j], q, nacc[mb][j]);
        if (side == 1) {
            f32x16 o[NB];
            if (weighted) {
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) acc[mb][j] *= m;
            }
            contract_pivots<D, RB, kSplit>(o, acc, s_yf[0], s_yf[1], lane);
            IO* out = reinterpret_cast<IO*>(p.dV);
            const int row0 = tile * kTileTokens + 4 * kg;
            IO* const lane_base = out + ((size_t)g * stride + row0) * D;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (row0 + 8 * (j >> 2) + (j & 3) < n)
                    store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, o[0][j], o[NB - 1][j]);
        }
    }
    // per-workgroup partials of s (scaled by rho') and N
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        float c[16 * RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) c[16 * mb + j] = which == 0 ? sacc[mb][j] : nacc[mb][j];
        const float total = reduce_scatter_tokens<16 * RB>(c, i);
        const int q = RB == 2 ? i : i >> 1;
        s_part[wave][which][32 * (q >> 4) + 8 * ((q & 15) >> 2) + 4 * kg + (q & 3)] = total;
        if (RB == 1) s_part[wave][which][32 + lane % 32] = 0.f;
    }
    __syncthreads();
    if (tid < 128) {
        const int which = tid >> 6, t = tid & 63;
        float tot = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) tot += s_part[wv][which][t];
        if (which == 0) tot *= s_rho[t];
        p.sn_part[(((size_t)pair * p.chunks + chunk) * 2 + which) * 64 + t] = tot;
    }
}

// ---------------------------------------------------------------------------------------------
// Gram reduce: gram_full[k][pair] = sum over chunks (index order).  The partial results hold the
// 32 x 32 blocks on and above the diagonal; a sum above the diagonal blocks is also written to its
// mirror image.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void gram_reduce_body(const BtParams& p, int R, size_t total, size_t block)
{
    const size_t idx = block * blockDim.x + threadIdx.x;    // (kp, e)
    if (idx >= total) return;
    const int R2 = R * R;
    const size_t kp = idx / R2;
    const int e = (int)(idx % R2);
    const int row = e / R, col = e % R;
    if (col / 32 < row / 32) return;
    const float* src = p.gram_part + kp * p.chunks * R2 + e;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int c = 0;
    for (; c + 3 < p.chunks; c += 4) {
        a0 += src[(size_t)c * R2]; a1 += src[(size_t)(c + 1) * R2];
        a2 += src[(size_t)(c + 2) * R2]; a3 += src[(size_t)(c + 3) * R2];
    }
    for (; c < p.chunks; ++c) a0 += src[(size_t)c * R2];
    const float sum = (a0 + a1) + (a2 + a3);
    p.gram_full[idx] = sum;
    if (col / 32 > row / 32) p.gram_full[kp * R2 + (size_t)col * R + row] = sum;
}

// mid and Gram reduce share a launch: neither depends on the other, both are short, and the glue kernel
// that follows needs only the first (blocks [0, mid_blocks) are mid's, the rest the reduction's; total == 0:
// no reduction, the pairs' only workgroups have written their matrices in place).
template <int D>
__global__ void bt_mid_gram(BtParams p, int R, size_t total, int mid_blocks)
{
    if ((int)blockIdx.x < mid_blocks) mid_body<D>(p, (int)blockIdx.x);
    else gram_reduce_body(p, R, total, (size_t)blockIdx.x - mid_blocks);
}

// ---------------------------------------------------------------------------------------------
// recursion over the iterations: one workgroup per pair
// ---------------------------------------------------------------------------------------------
// Sum over the 64 lanes of a wavefront, the same bits in every lane: the two halves and the two rows of 16 of
// a half through lane swaps, then rotations within the rows of 16 (every lane adds the same pairs, in the
// same tree).  No LDS: about sixty cycles, where six shuffles through the LDS crossbar take several hundred.
__device__ __forceinline__ float wave_sum(float x)
{
    float lo, hi;
    both_halves(x, lo, hi);
    x = lo + hi;
    x = swap16_add(x, x);
    x += dpp_move<0x128>(x);   // row_ror:8
    x += dpp_move<0x124>(x);   // row_ror:4
    x += dpp_move<0x122>(x);   // row_ror:2
    x += dpp_move<0x121>(x);   // row_ror:1
    return x;
}

// Four wavefronts: thread (q, t) = (tid / 64, tid % 64) sums the products of R / 4 rows of M^k (R x R, R = 32 or 64)
// with column t.
// All four carry the recursion, with the same operations in the same order (hence the same bits), so what a
// step needs of the pivot vector's other lanes a wavefront reads from its own lanes, and the only exchange of a
// step is the one between the four partial sums and their addition (one workgroup barrier).  The chain of T
// steps is all latency -- a step is a few hundred cycles of work, a load from memory 1.5 us -- so nothing in it
// may wait for memory or divide.  KEPT > 0 (T <= KEPT): the shares of all T Gram matrices are requested before
// the chain starts and sit in registers (a wavefront has a SIMD's 512 to itself); KEPT == 0: any T, the matrix
// of the next step is requested before this one's is used, which hides one step's worth of the latency.
template <int KEPT, int R>
__global__ void __launch_bounds__(256) bt_recursion(BtParams p)
{
    constexpr int kPer = R / 4, per = kPer;   // rows of M^k per thread
    constexpr int kHeld = KEPT > 0 ? KEPT : 2;
    __shared__ float s_c[kMaxTiledIters][64]; // c^k_t, k = 1 .. T
    __shared__ float s_q[2][4][64];           // the partial sums (two parities: one barrier per step)
    const int pair = blockIdx.x, t = threadIdx.x & 63, pairs = 2 * p.G, T = p.T;
    const int q = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = (pair % p.G) % p.H;
    const bool live = t < p.r;
    const float a = 1.f / (float)p.n_side[pair / p.G];
    const float b = live ? p.beta[h * p.r + t] : 1.f;
    float gm[kHeld][kPer];
    auto fetch = [&](float (&dst)[kPer], int k) {
        // M^k is symmetric: thread t walks column t, so that a wavefront reads whole rows
        const float* col = p.gram_full + ((size_t)(k - 1) * pairs + pair) * R * R + min(t, R - 1);
#pragma unroll
        for (int j = 0; j < kPer; ++j) dst[j] = j < per ? col[(size_t)(q * per + j) * R] : 0.f;
    };
    if constexpr (KEPT > 0) {
#pragma unroll
        for (int kk = KEPT - 1; kk >= 0; --kk)
            if (kk < T) fetch(gm[kk], kk + 1);
    } else {
        fetch(gm[0], T);
    }
    for (int e = threadIdx.x; e < T * 64; e += 256) {
        const int k = e / 64 + 1, u = e % 64;
        s_c[k - 1][u] = colsum_of(p.colacc[((size_t)k * pairs + pair) * 64 + u], p.fx_unscale) * a;   // c^k_u
    }
    // s and N of the pair: the chunks' shares, every fourth one per wavefront (eight loads in flight), then the
    // four partial sums in a fixed order
    {
        float ps = 0.f, pn = 0.f;
        for (int c0 = q; c0 < p.chunks; c0 += 16) {
            float vs[4], vn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = c0 + 4 * j;
                vs[j] = c < p.chunks ? p.sn_part[(((size_t)pair * p.chunks + c) * 2 + 0) * 64 + t] : 0.f;
                vn[j] = c < p.chunks ? p.sn_part[(((size_t)pair * p.chunks + c) * 2 + 1) * 64 + t] : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) { ps += vs[j]; pn += vn[j]; }
        }
        s_q[0][q][t] = ps;
        s_q[1][q][t] = pn;
    }
    __syncthreads();
    const float s = (s_q[0][0][t] + s_q[0][1][t]) + (s_q[0][2][t] + s_q[0][3][t]);
    const float nn = (s_q[1][0][t] + s_q[1][1][t]) + (s_q[1][2][t] + s_q[1][3][t]);
    __syncthreads();
    int parity = 0;
    auto gram_times = [&](const float (&m)[kPer], float v) {             // (M^k v)_t with this thread's rows of M^k in m
        const int vbits = __builtin_bit_cast(int, live ? v : 0.f);
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (j < per) acc = fmaf(m[j], __builtin_bit_cast(float, __builtin_amdgcn_readlane(vbits, q * per + j)), acc);
        s_q[parity][q][t] = live && t < R ? acc : 0.f;
        lds_barrier();     // (orders LDS only: a full barrier would wait for the stores of dc^k and for the matrices still on their way)
        const float sum = (s_q[parity][0][t] + s_q[parity][1][t]) + (s_q[parity][2][t] + s_q[parity][3][t]);
        parity ^= 1;
        return sum;
    };
    // The potentials are defined up to a common constant, so every dg^k sums to zero over the pivots, and
    // the step dg^k -> dg^{k-1} leaves the direction c^k unchanged (its eigenvector of eigenvalue 1, which
    // changes no similarity gradient): whatever rounding puts into that sum would stay for all remaining
    // iterations and end up, T times over, in the gradient of the masses.  It is taken out along c^k
    // (sum_t c^k_t = 1) before dg^k is used.
    const float eps_over_b = live ? p.eps / b : 0.f;
    float db = live ? s / b : 0.f;
    float dc = live ? -s / s_c[T - 1][t] : 0.f;
    float dg = 0.f;
    if (q == 0) p.dcs[((size_t)T * pairs + pair) * 64 + t] = dc;
    auto step = [&](int k, const float (&m)[kPer], float ck, float eps_over_ck) {       // dg^k -> dg^{k-1}, k < T
        dg -= ck * wave_sum(live ? dg : 0.f);
        dc = live ? -dg * eps_over_ck : 0.f;
        db += dg * eps_over_b;
        if (q == 0) p.dcs[((size_t)k * pairs + pair) * 64 + t] = dc;
        dg = -(a / p.eps) * gram_times(m, dc);
    };
    // (the column sums and their reciprocals of the next step are read and formed while this one runs)
    float ck = T > 1 ? s_c[T - 2][t] : 1.f, eck = live ? p.eps / ck : 0.f;
    if constexpr (KEPT > 0) {
#pragma unroll
        for (int kk = KEPT - 1; kk >= 0; --kk) {
            const int k = kk + 1;
            if (k > T) continue;
            if (k == T) {
                dg = -(nn + a * gram_times(gm[kk], dc)) / p.eps;     // dg^{T-1}
            } else {
                const float ck_now = ck, eck_now = eck;
                if (k > 1) { ck = s_c[k - 2][t]; eck = live ? p.eps / ck : 0.f; }
                step(k, gm[kk], ck_now, eck_now);
            }
        }
    } else {
        if (T > 1) fetch(gm[1], T - 1);
        dg = -(nn + a * gram_times(gm[0], dc)) / p.eps;      // dg^{T-1}
        for (int k = T - 1; k >= 1; --k) {
#pragma unroll
            for (int j = 0; j < kPer; ++j) gm[0][j] = gm[1][j];
            if (k > 1) fetch(gm[1], k - 1);
            const float ck_now = ck, eck_now = eck;
            if (k > 1) { ck = s_c[k - 2][t]; eck = live ? p.eps / ck : 0.f; }
            step(k, gm[0], ck_now, eck_now);
        }
    }
    if (q == 0) p.db_pair[(size_t)pair * 64 + t] = live ? db : 0.f;
}

// ---------------------------------------------------------------------------------------------
// assemble: dC tile over all iterations, then dQ / dK rows and the workgroup's share of dZ
// ---------------------------------------------------------------------------------------------
template <typename IO, int D, int RB>
__global__ void __launch_bounds__(kThreads, 2) bt_assemble(BtParams p, int Tcap, const unsigned* redo)
{
    // after the all-at-once kernel: only the workgroups that it marked
    if (redo && redo[blockIdx.x] == 0) return;
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];   // [Tcap][2][64] floats: g^{k-1} c1, dc^k
    __shared__ float s_rho[64];
    __shared__ __attribute__((aligned(16))) float s_y[64 * D];
    constexpr int kParts = kSplit ? 2 : 1;     // bf16 hi only, or hi and lo
    __shared__ __attribute__((aligned(16))) bf16x8 s_zf[2][2 * RB * NB * 64];
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[kWaves * kParts * 32 * RB * kTrStride];
    __shared__ __attribute__((aligned(16))) char s_zstash[PivotStashBytes<IO, D, RB>::value];
    constexpr bool kYPieces = !(D == 32 && RB == 2);   // the matrix operand of the dGamma product as bf16 pieces (fp32 I/O)
    __shared__ __attribute__((aligned(16))) char s_ystash[PivotStashBytes<IO, D, RB, kYPieces>::value];
    static_assert(kSplit || sizeof(s_zf[1]) >= (size_t)StashBytes<IO, D, RB>::value, "the lo stash takes the place of s_zf[1]");
    char* const s_ystash_lo = reinterpret_cast<char*>(s_zf[1]);   // bf16 I/O only (s_zf[1] is then unused)
    float* s_hist = reinterpret_cast<float*>(s_dyn);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.G;
    const int pair = blockIdx.x / p.chunks, chunk = blockIdx.x % p.chunks;
    const int side = pair / p.G, g = pair % p.G, h = g % p.H;
    const int n = p.n_side[side], stride = p.stride_side[side], r = p.r, T = p.T;
    const float c1 = kLog2e / p.eps;
    const IO* X = rows_of<IO>(p, side);
    const IO* vals = reinterpret_cast<const IO*>(side == 0 ? p.dO : p.V);
    const float* ymat = (side == 0 ? p.yp : p.dyraw) + (size_t)g * 64 * D;
    const float yscale = side == 0 ? (float)n : 1.f;
    uint16_t* tr_hi = s_tr + (wave * kParts + 0) * 32 * RB * kTrStride;
    uint16_t* tr_lo = s_tr + (wave * kParts + kParts - 1) * 32 * RB * kTrStride;

    for (int e = tid; e < T * 64; e += kThreads) {
        const int k = e / 64 + 1, t = e % 64;
        s_hist[((k - 1) * 2 + 0) * 64 + t] = p.ghist[((size_t)(k - 1) * pairs + pair) * 64 + t] * c1;   // padding: -1e30 c1
        s_hist[((k - 1) * 2 + 1) * 64 + t] = p.dcs[((size_t)k * pairs + pair) * 64 + t];
    }
    if (tid < 64) s_rho[tid] = p.rhop[(size_t)pair * 64 + tid];
    if (wave == 0) {
        Frag<IO, D> z0[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            const int t = 32 * mb + i;
            load_pivots<D>(z0[mb], p.Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
        }
        stash_similarity_pivots<IO, D, RB>(s_zstash, z0, lane);
    }
    // Z rows as B fragments (the values the forward pass multiplied with: rounded to bf16 for bf16 I/O)
    for (int e = tid; e < 64 * D; e += kThreads) {
        const int t = e / D;
        float z = t < r ? p.Z[((size_t)h * r + t) * D + e % D] : 0.f;
        if (!kSplit) z = (float)(__bf16)z;
        s_y[e] = z;
    }
    __syncthreads();
    lay_out_fragments<D, RB>(s_y, s_zf[0], s_zf[1], tid);
    __syncthreads();
    for (int e = tid; e < 64 * D; e += kThreads) s_y[e] = ymat[e] * yscale;
    __syncthreads();
    if (wave == 0) {
        Frag<IO, D> y0[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) load_pivots_lds<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
        stash_similarity_pivots<IO, D, RB, kYPieces>(s_ystash, y0, lane);
        if (!kSplit) {
            // bf16 I/O: the lo part of the same operand (see the glue kernel); it takes the place of the
            // lo half of the Z fragments, which only fp32 I/O uses
#pragma unroll
            for (int mb = 0; mb < RB; ++mb) load_pivots_lds_lo<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
            stash_pivots<D, RB>(s_ystash_lo, y0, lane);
        }
    }
    __syncthreads();   // s_y is reused below for the dZ partial

    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.tiles_per_wg);
    f32x16 dZacc[RB][NB];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 16; ++j) dZacc[mb][nb][j] = 0.f;
    const float scale_out = 1.f / ((float)n * p.eps);   // a / eps

    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        const int tok = min(tile * kTileTokens + i, n - 1);
        const bool valid = tile * kTileTokens + i < n;
        Frag<IO, D> xc, vc;
        load_tokens<D>(xc, X + ((size_t)g * stride + tok) * D, kg);
        load_tokens<D>(vc, vals + ((size_t)g * stride + tok) * D, kg);
        // mass times n of this lane's token: multiplies the column-sum adjoints dc^k on their way into the
        // row (dW^k_it = a_i dc^k_t) and, for the keys, the incoming gradient of the coupling
        const float m = token_weight(p, side, g, tok);
        const float mdc = side == 0 ? m : 1.f;       // the keys' factor is applied to the whole of dW^T instead
        int skew = 0;
        asm volatile("" : "+v"(skew));
        // similarities scaled to base-2 exponents, once
        f32x16 sc[RB], dacc[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) { sc[mb][j] = 0.f; dacc[mb][j] = 0.f; }
        {
            similarity_stashed<IO, D, RB>(sc, s_zstash, xc, lane, skew);
        }
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) sc[mb][j] *= c1;

        // One iteration's share: dacc += W^k (dP - e_i), with W^k rebuilt from the scaled similarities
        // and that iteration's potentials (pot, LDS, already times c1).  W^k = e / sum(e) with
        // e = exp2(x - shift) for ANY row shift that keeps the row sum well inside the fp32 range, so
        // the shift is not recomputed per iteration: it is the row maximum of the first iteration
        // processed (folded into sc), and the maxima of the others differ from it by the change of
        // the potentials, a few binary orders.  The row sums are checked; if one leaves the safe range
        // the rows are re-shifted by this iteration's maxima and the iteration is redone (its sums
        // then lie in [1, 64]).
        // (dp holds dW^k up to the row factor ms: dW^k_it = ms dp_it)
        auto add_iteration = [&](const float* pot, const f32x16 (&dp)[RB], float ms, bool fold) {
            f32x16 e[RB];
            float ssum, sdot;
            for (;;) {
                load_pivot_vector<RB>(e, pot + skew, kg);
                if (fold) {
                    float m0 = -INFINITY, m1 = -INFINITY;
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int j = 0; j < 16; j += 2) {
                            m0 = fmaxf(m0, e[mb][j] + sc[mb][j]);
                            m1 = fmaxf(m1, e[mb][j + 1] + sc[mb][j + 1]);
                        }
                    const float m = pair_max(fmaxf(m0, m1));
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int j = 0; j < 16; ++j) sc[mb][j] -= m;
                }
                float s0 = 0.f, s1 = 0.f, d0 = 0.f, d1 = 0.f;
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 2) {
                        const float e0 = exp2_fast(e[mb][j] + sc[mb][j]), e1 = exp2_fast(e[mb][j + 1] + sc[mb][j + 1]);
                        e[mb][j] = e0; e[mb][j + 1] = e1;
                        s0 += e0; s1 += e1;
                        d0 = fmaf(dp[mb][j], e0, d0);
                        d1 = fmaf(dp[mb][j + 1], e1, d1);
                    }
                float lo, hi;
                both_halves(s0 + s1, lo, hi); ssum = lo + hi;
                both_halves(d0 + d1, lo, hi); sdot = lo + hi;
                const bool safe = ssum >= p.sum_lo && ssum <= p.sum_hi;      // false for NaN too
                if (fold || __all(safe)) break;
                fold = true;
            }
            const float w = valid ? rcp_fast(ssum) : 0.f;
            const float wm = w * ms;
            const float nwe = -(sdot * wm) * w;           // -w e^k_i,  e^k_i = sum_t dW_it W_it
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) dacc[mb][j] = fmaf(e[mb][j], fmaf(dp[mb][j], wm, nwe), dacc[mb][j]);
        };
        {
            // last iteration: dP^T = dGamma rho + dc^T with rho_t = beta_t / c^T_t = n rho'_t
            f32x16 dp[RB];
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) dp[mb][j] = 0.f;
            {
                similarity_stashed<IO, D, RB, kYPieces>(dp, s_ystash, vc, lane, skew);                 // dGamma tile
                if (!kSplit) similarity_stashed<IO, D, RB, kYPieces>(dp, s_ystash_lo, vc, lane, skew);
            }
            {
                f32x16 rho[RB], dc[RB];
                load_pivot_vector<RB>(rho, s_rho + skew, kg);
                load_pivot_vector<RB>(dc, s_hist + ((T - 1) * 2 + 1) * 64 + skew, kg);
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) dp[mb][j] = fmaf(dp[mb][j] * (float)n, rho[mb][j], dc[mb][j] * mdc);
            }
            add_iteration(s_hist + ((T - 1) * 2 + 0) * 64, dp, side == 0 ? 1.f : m, true);
        }
        for (int k = T - 1; k >= 1; --k) {
            f32x16 dp[RB];
            load_pivot_vector<RB>(dp, s_hist + ((k - 1) * 2 + 1) * 64 + skew, kg);
            add_iteration(s_hist + ((k - 1) * 2 + 0) * 64, dp, m, false);
        }
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) dacc[mb][j] *= scale_out;      // dC tile

        // dQ (or dK) rows = dC Z
        {
            f32x16 o[NB];
            contract_pivots<D, RB, kSplit>(o, dacc, s_zf[0], s_zf[1], lane);
            IO* out = reinterpret_cast<IO*>(side == 0 ? p.dQ : p.dK);
            const int row0 = tile * kTileTokens + 4 * kg;
            IO* const lane_base = out + ((size_t)g * stride + row0) * D;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (row0 + 8 * (j >> 2) + (j & 3) < n)
                    store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, o[0][j], o[NB - 1][j]);
        }
        // dZ += dC^T X
        bf16x8 vh[2][NB], vl[2][NB];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
            const int left = max(1, min(8, n - t0));
            load_values<D>(vh[s], vl[s], X, (size_t)g * stride + min(t0, n - 1), left, i);
        }
        transpose_tile<RB, kSplit>(dacc, tr_hi, tr_lo, i, kg);
        contract_tokens<D, RB, kSplit>(dZacc, tr_hi, tr_lo, vh, vl, i, kg);
        transpose_done();
    }
    __syncthreads();
    sum_over_waves<D, RB>(dZacc, s_y, wave, i, kg);
    float* zp = p.dz_part + ((size_t)pair * p.chunks + chunk) * 64 * D;
    for (int e = tid; e < 32 * RB * D; e += kThreads) zp[e] = s_y[e];
}

// ---------------------------------------------------------------------------------------------
// assemble, all iterations of a tile at once (T <= 16): the per-iteration work of the kernel above as
// two small matrix products.  With the rows shifted once, by the row maxima of the last iteration,
//   e^k_it = E_it P^k_t,   E_it = exp2((C_it + g^{T-1}_t) c1 - max_i),   P^k_t = exp2((g^{k-1}_t - g^{T-1}_t) c1 - h_k)
// (h_k = the largest such difference, so P <= 1; P^T = 1), the row sums and the row products with dP^k are
//   ssum^k_i = sum_t Tab[P^k][t] E_it,   sdot^k_i = sum_t Tab[P^k dc^k][t] E_it          (first product: Tab E)
// and, with w^k_i = 1 / ssum^k_i and the row factors R^k_i = ms w^k_i, S^k_i = R^k_i w^k_i sdot^k_i,
//   dC_it = (a/eps) E_it [ sum_k R^k_i Tab[P^k dc^k][t] - S^k_i Tab[P^k][t]  +  R^T_i n rho_t dGamma_it ]
// (second product: Tab^T applied to the row factors).  Both products run on the fp32 matrix cores
// (32 x 32 x 2 per instruction): one exponential per element instead of one per iteration, and the
// vector ALU is left with a handful of operations per element.  The row sums are checked against the
// same range as above; a workgroup that finds one outside marks itself in `redo`, and the kernel above
// then redoes that workgroup's tiles iteration by iteration.
// Table rows: 2 (k - 1) = P^k dc^k, 2 (k - 1) + 1 = P^k  (k < T);  2 (T - 1) = dc^T, 2 (T - 1) + 1 = 1.
// ---------------------------------------------------------------------------------------------
constexpr int kAllAtOnceIters = 16;
constexpr int kTabStride = 65;     // floats per table row (64 pivots + 1: rows fall into different banks)

template <typename IO, int D, int RB>
__global__ void __launch_bounds__(kThreads, 2) bt_assemble_mf(BtParams p, unsigned* redo)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    __shared__ float s_brho[64], s_pot[64], s_h[kAllAtOnceIters];
    __shared__ int s_redo;
    __shared__ __attribute__((aligned(16))) float s_tab[32 * kTabStride];
    __shared__ __attribute__((aligned(16))) float s_y[32 * RB * D];     // staging of the 32 RB pivot rows in use, then the dZ partial
    constexpr int kParts = kSplit ? 2 : 1;     // bf16 hi only, or hi and lo
    __shared__ __attribute__((aligned(16))) bf16x8 s_zf[2][2 * RB * NB * 64];
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[kWaves * kParts * 32 * RB * kTrStride];
    __shared__ __attribute__((aligned(16))) char s_zstash[PivotStashBytes<IO, D, RB>::value];
    constexpr bool kYPieces = true;   // the matrix operand of the dGamma product as bf16 pieces (fp32 I/O)
    __shared__ __attribute__((aligned(16))) char s_ystash[PivotStashBytes<IO, D, RB, kYPieces>::value];
    static_assert(kSplit || sizeof(s_zf[1]) >= (size_t)StashBytes<IO, D, RB>::value, "the lo stash takes the place of s_zf[1]");
    char* const s_ystash_lo = reinterpret_cast<char*>(s_zf[1]);   // bf16 I/O only (s_zf[1] is then unused)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 31, kg = lane >> 5;
    const int pairs = 2 * p.G;
    const int pair = blockIdx.x / p.chunks, chunk = blockIdx.x % p.chunks;
    const int side = pair / p.G, g = pair % p.G, h = g % p.H;
    const int n = p.n_side[side], stride = p.stride_side[side], r = p.r, T = p.T;
    const float c1 = kLog2e / p.eps;
    const IO* X = rows_of<IO>(p, side);
    const IO* vals = reinterpret_cast<const IO*>(side == 0 ? p.dO : p.V);
    const float* ymat = (side == 0 ? p.yp : p.dyraw) + (size_t)g * 64 * D;
    const float yscale = side == 0 ? (float)n : 1.f;
    uint16_t* tr_hi = s_tr + (wave * kParts + 0) * 32 * RB * kTrStride;
    uint16_t* tr_lo = s_tr + (wave * kParts + kParts - 1) * 32 * RB * kTrStride;
    const float* g_last = p.ghist + ((size_t)(T - 1) * pairs + pair) * 64;

    if (tid == 0) s_redo = 0;
    // Every global load of the set-up is requested here, together (the table's inputs and the matrix rows are
    // kept in registers until the LDS areas they go to are free): one round trip to memory, not three.
    constexpr int kTabPer = 32 * 64 / kThreads, kMatPer = 32 * RB * D / kThreads;
    float tdc[kTabPer], tg[kTabPer], yreg[kMatPer];
#pragma unroll
    for (int q = 0; q < kTabPer; ++q) {
        const int e = tid + q * kThreads, t = e % 64, k = e / 64 / 2 + 1;
        const bool live = k <= T && t < r;
        tdc[q] = live ? p.dcs[((size_t)k * pairs + pair) * 64 + t] : 0.f;
        tg[q] = live && k < T ? p.ghist[((size_t)(k - 1) * pairs + pair) * 64 + t] : 0.f;
    }
#pragma unroll
    for (int q = 0; q < kMatPer; ++q) yreg[q] = ymat[tid + q * kThreads] * yscale;
    if (tid < 64) {
        s_brho[tid] = (float)n * p.rhop[(size_t)pair * 64 + tid];
        s_pot[tid] = g_last[tid] * c1;                       // padding: -1e30 c1
    }
    // h_k: one wavefront per iteration k < T
    for (int k = 1 + wave; k < T; k += kWaves) {
        float dmax = lane < r ? (p.ghist[((size_t)(k - 1) * pairs + pair) * 64 + lane] - g_last[lane]) * c1 : -INFINITY;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dmax = fmaxf(dmax, __shfl_xor(dmax, o, 64));
        if (lane == 0) s_h[k - 1] = dmax;
    }
    if (wave == 0) {
        Frag<IO, D> z0[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            const int t = 32 * mb + i;
            load_pivots<D>(z0[mb], p.Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
        }
        stash_similarity_pivots<IO, D, RB>(s_zstash, z0, lane);
    }
    // Z rows as B fragments (the values the forward pass multiplied with: rounded to bf16 for bf16 I/O)
    for (int e = tid; e < 32 * RB * D; e += kThreads) {
        const int t = e / D;
        float z = t < r ? p.Z[((size_t)h * r + t) * D + e % D] : 0.f;
        if (!kSplit) z = (float)(__bf16)z;
        s_y[e] = z;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kTabPer; ++q) {
        const int e = tid + q * kThreads, row = e / 64, t = e % 64, k = row / 2 + 1;
        float v = 0.f;
        if (k <= T && t < r) {
            if (k == T) {
                v = (row & 1) ? 1.f : tdc[q];
            } else {
                const float P = exp2_fast(fmaf(tg[q], c1, -s_pot[t]) - s_h[k - 1]);
                v = (row & 1) ? P : P * tdc[q];
            }
        }
        s_tab[row * kTabStride + t] = v;
    }
    lay_out_fragments<D, RB>(s_y, s_zf[0], s_zf[1], tid);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kMatPer; ++q) s_y[tid + q * kThreads] = yreg[q];
    __syncthreads();
    if (wave == 0) {
        Frag<IO, D> y0[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) load_pivots_lds<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
        stash_similarity_pivots<IO, D, RB, kYPieces>(s_ystash, y0, lane);
        if (!kSplit) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb) load_pivots_lds_lo<D>(y0[mb], s_y + (32 * mb + i) * D, kg);
            stash_pivots<D, RB>(s_ystash_lo, y0, lane);
        }
    }
    __syncthreads();   // s_y is reused below for the dZ partial

    const int ntiles = (n + kTileTokens - 1) / kTileTokens;
    const int tile_begin = chunk * p.tiles_per_wg, tile_end = min(ntiles, tile_begin + p.tiles_per_wg);
    f32x16 dZacc[RB][NB];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 16; ++j) dZacc[mb][nb][j] = 0.f;
    const float scale_out = 1.f / ((float)n * p.eps);   // a / eps
    bool all_safe = true;

    for (int tile = tile_begin + wave; tile < tile_end; tile += kWaves) {
        const int tok = min(tile * kTileTokens + i, n - 1);
        const bool valid = tile * kTileTokens + i < n;
        Frag<IO, D> xc, vc;
        load_tokens<D>(xc, X + ((size_t)g * stride + tok) * D, kg);
        load_tokens<D>(vc, vals + ((size_t)g * stride + tok) * D, kg);
        const float m = token_weight(p, side, g, tok);
        const float mdc = side == 0 ? m : 1.f, ms_last = side == 0 ? 1.f : m;
        int skew = 0;
        asm volatile("" : "+v"(skew));
        // E: the last iteration's exponentials, rows shifted by their maxima
        f32x16 E[RB];
        load_pivot_vector<RB>(E, s_pot + skew, kg);
        {
            f32x16 sc[RB];
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) sc[mb][j] = 0.f;
            similarity_stashed<IO, D, RB>(sc, s_zstash, xc, lane, skew);
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) E[mb][j] = fmaf(sc[mb][j], c1, E[mb][j]);
        }
        {
            float m0 = -INFINITY, m1 = -INFINITY;
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; j += 2) {
                    m0 = fmaxf(m0, E[mb][j]);
                    m1 = fmaxf(m1, E[mb][j + 1]);
                }
            const float mx = pair_max(fmaxf(m0, m1));
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) E[mb][j] = exp2_fast(E[mb][j] - mx);
        }
        // the incoming gradient of the coupling times n rho_t, and its row product with E
        f32x16 dgam[RB];
        float qd;
        {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) dgam[mb][j] = 0.f;
            similarity_stashed<IO, D, RB, kYPieces>(dgam, s_ystash, vc, lane, skew);
            if (!kSplit) similarity_stashed<IO, D, RB, kYPieces>(dgam, s_ystash_lo, vc, lane, skew);
            f32x16 br[RB];
            load_pivot_vector<RB>(br, s_brho + skew, kg);
            float q0 = 0.f, q1 = 0.f;
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; j += 2) {
                    dgam[mb][j] *= br[mb][j];
                    dgam[mb][j + 1] *= br[mb][j + 1];
                    q0 = fmaf(E[mb][j], dgam[mb][j], q0);
                    q1 = fmaf(E[mb][j + 1], dgam[mb][j + 1], q1);
                }
            qd = pair_sum(q0 + q1);
        }
        // first product: rows of the table against E (32 x 32 x 2 per instruction: this lane's pivot of the step)
        f32x16 rows;
#pragma unroll
        for (int j = 0; j < 16; ++j) rows[j] = 0.f;
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float a = s_tab[i * kTabStride + pivot_of(mb, j, kg) + skew];
                rows = __builtin_amdgcn_mfma_f32_32x32x2f32(a, E[mb][j], rows, 0, 0, 0);
            }
        // row factors, then the second product: the table transposed against them
        f32x16 br2[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) br2[mb][j] = 0.f;
        float r_last = 0.f;
        bool safe = true;
#pragma unroll
        for (int s = 0; s < kAllAtOnceIters; ++s) {
            if (s < T) {
                // rows 2 s (sdot) and 2 s + 1 (ssum) sit in registers jr, jr + 1 of the lanes with kg == (s / 2) % 2
                const int jr = 4 * (s / 4) + 2 * (s % 2);
                float lo, hi;
                both_halves(rows[jr], lo, hi);
                float sdot = (s / 2) % 2 == 0 ? lo : hi;
                both_halves(rows[jr + 1], lo, hi);
                const float ssum = (s / 2) % 2 == 0 ? lo : hi;
                safe = safe && ssum >= p.sum_lo && ssum <= p.sum_hi;      // false for NaN too
                const float w = valid ? rcp_fast(ssum) : 0.f;
                float R, ms;
                if (s == T - 1) {
                    sdot = fmaf(sdot, mdc, qd);
                    ms = ms_last;
                    r_last = w * ms;
                    R = r_last * mdc;
                } else {
                    ms = m;
                    R = w * ms;
                }
                const float S = (sdot * (w * ms)) * w;
                const float b = kg ? -S : R;
#pragma unroll
                for (int mb = 0; mb < RB; ++mb) {
                    const float a = s_tab[(2 * s + kg) * kTabStride + 32 * mb + i + skew];
                    br2[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, br2[mb], 0, 0, 0);
                }
            }
        }
        all_safe = all_safe && __all(safe);
        f32x16 dacc[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) dacc[mb][j] = E[mb][j] * scale_out * fmaf(r_last, dgam[mb][j], br2[mb][j]);

        // dQ (or dK) rows = dC Z
        {
            f32x16 o[NB];
            contract_pivots<D, RB, kSplit>(o, dacc, s_zf[0], s_zf[1], lane);
            IO* out = reinterpret_cast<IO*>(side == 0 ? p.dQ : p.dK);
            const int row0 = tile * kTileTokens + 4 * kg;
            IO* const lane_base = out + ((size_t)g * stride + row0) * D;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (row0 + 8 * (j >> 2) + (j & 3) < n)
                    store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, o[0][j], o[NB - 1][j]);
        }
        // dZ += dC^T X
        bf16x8 vh[2][NB], vl[2][NB];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
            const int left = max(1, min(8, n - t0));
            load_values<D>(vh[s], vl[s], X, (size_t)g * stride + min(t0, n - 1), left, i);
        }
        transpose_tile<RB, kSplit>(dacc, tr_hi, tr_lo, i, kg);
        contract_tokens<D, RB, kSplit>(dZacc, tr_hi, tr_lo, vh, vl, i, kg);
        transpose_done();
    }
    if (!all_safe) s_redo = 1;         // (every writer writes the same value)
    __syncthreads();
    sum_over_waves<D, RB>(dZacc, s_y, wave, i, kg);
    float* zp = p.dz_part + ((size_t)pair * p.chunks + chunk) * 64 * D;
    for (int e = tid; e < 32 * RB * D; e += kThreads) zp[e] = s_y[e];
    if (tid == 0) redo[blockIdx.x] = (unsigned)s_redo;
}

// ---------------------------------------------------------------------------------------------
// final: dZ[h][t][c] and dbeta[h][t], summed over chunks, sides and the batch.  32 outputs per workgroup,
// each summed by 8 to 32 threads (`slices`) that take every slices-th of the (problem of the batch, side, chunk) shares, four loads
// in flight each, and are then added in order: a fixed order, and one round of loads whether the shares are many
// problems with one chunk each or few problems with many chunks.
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
__global__ void __launch_bounds__(kFinalSlices * kFinalOutputs) bt_final(BtParams p, int D, int step_q, int step_ch)   // (slices / chunks, slices % chunks)
{
    __shared__ float s_part[kFinalSlices][kFinalOutputs];
    const int o = threadIdx.x % kFinalOutputs, slice = threadIdx.x / kFinalOutputs, slices = blockDim.x / kFinalOutputs;
    const int idx = blockIdx.x * kFinalOutputs + o;     // (h, t, c), c == D meaning beta
    const int per = p.r * (D + 1);
    const bool live = idx < p.H * per;
    const int h = live ? idx / per : 0, t = live ? (idx % per) / (D + 1) : 0, c = live ? idx % (D + 1) : 0;
    float acc = 0.f;
    if (live && c < D) {
        // the shares of every (problem of the batch, side, chunk), numbered (side B + b) chunks + chunk: every
        // slices-th one, four loads in flight; the walk carries (row, chunk) along instead of dividing each time
        const int rows = 2 * p.B;
        int q = slice / p.chunks, ch = slice % p.chunks;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        auto next_share = [&]() {
            float v = 0.f;
            if (q < rows) {
                const int side = q >= p.B ? 1 : 0, g = (q - side * p.B) * p.H + h;
                v = p.dz_part[(((size_t)(side * p.G + g) * p.chunks) + ch) * 64 * D + t * D + c];
            }
            q += step_q; ch += step_ch;
            if (ch >= p.chunks) { ch -= p.chunks; ++q; }
            return v;
        };
        while (q < rows) {
            const float v0 = next_share(), v1 = next_share(), v2 = next_share(), v3 = next_share();
            a0 += v0; a1 += v1; a2 += v2; a3 += v3;
        }
        acc = (a0 + a1) + (a2 + a3);
    } else if (live) {
        for (int b = slice; b < p.B; b += slices) {
            const int g = b * p.H + h;
            acc += p.db_glue[g * 64 + t];
            acc += p.db_pair[(size_t)g * 64 + t];
            acc += p.db_pair[(size_t)(p.G + g) * 64 + t];
        }
    }
    s_part[slice][o] = acc;
    __syncthreads();
    if (slice == 0 && live) {
        float tot = 0.f;
        for (int sl = 0; sl < slices; ++sl) tot += s_part[sl][o];
        // a sweep whose wait between workgroups gave up has marked this launch: the gradients of the
        // pivots and their masses are made NaN, so that the failure cannot pass for a result
        if (p.status[0] == p.nonce) tot = __builtin_nanf("");
        if (c < D) p.dZ[((size_t)h * p.r + t) * D + c] = tot;
        else p.dbeta[h * p.r + t] = tot;
    }
}

// zeroes the column-sum words and records the launch in the status area (only where the sweep is a
// launch per pass: the persistent sweep clears for itself)
__global__ void bt_clear(unsigned long long* p, size_t count, unsigned long long* status, unsigned long long nonce)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < count) p[idx] = 0ull;
    if (idx == 0) status[1] = nonce;
}

template <typename IO, int D, int RB>
int launch_all(const BwdArgs& a, BtParams p)
{
    const lot_shape& s = a.s;
    const int pairs = 2 * p.G, T = a.iters, R = 32 * RB;
    hipStream_t st = a.stream;
    const unsigned grid = (unsigned)pairs * p.chunks;
    // The persistent sweep needs the workgroups of a pair resident together: the whole grid fits the
    // device, or a pair is a single workgroup (which then waits for nobody but itself).
    // (the capacity is taken from the variant with token masses: the same code plus a few registers)
    // which form of the sweep kernel this shape takes: with token masses; at most two tiles per wavefront, whose
    // similarities then stay in registers between the passes (measured: DeiT shape, fp32, backward 170 -> 135 us;
    // B H = 192, n = 256, r = 64: fp32 336 -> 258, bf16 186 -> 177; four kept tiles with bf16 I/O and 32 pivots, the
    // BERT shape, gained nothing and are not compiled); or the plain one
    const bool mass = p.mass_side[0] != nullptr || p.mass_side[1] != nullptr;
    const int per_wave = (p.tiles_per_wg + kWaves - 1) / kWaves;
    const int form = mass ? 0 : (per_wave <= 2 && sweep_keeps_similarities()) ? 1 : 2;
    void (*const sweep)(BtParams) = form == 0 ? bt_sweep<IO, D, RB, true, 0> : form == 1 ? bt_sweep<IO, D, RB, false, 2>
                                                                                            : bt_sweep<IO, D, RB, false, 0>;
    bool persistent = p.chunks == 1;
    if (!persistent && p.chunks <= 255) {
        static thread_local int capacity_cache[8][3] = {};   // per device ordinal and form of the kernel
        int dev = 0;
        LOT_HIP_CHECK(hipGetDevice(&dev));
        int capacity = (dev >= 0 && dev < 8) ? capacity_cache[dev][form] : 0;
        if (capacity == 0) {
            int per_cu = 0, cus = 0;
            LOT_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sweep, kThreads, 0));
            LOT_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
            capacity = per_cu * cus;
            if (dev >= 0 && dev < 8) capacity_cache[dev][form] = capacity;
        }
        persistent = (int)grid <= capacity;
    }
    // testing aid: run the sweep as one launch per pass although it would fit (the fallback of devices
    // that cannot hold the grid), so that this form stays exercised
    if (sweep_by_launches() || a.stepwise) persistent = false;
    if (persistent) {
        sweep<<<grid, kThreads, 0, st>>>(p);
    } else {
        const size_t words = (size_t)(T + 1) * pairs * 64;
        bt_clear<<<(unsigned)((words + 255) / 256), 256, 0, st>>>(p.colacc, words, p.status, p.nonce);
        for (int k = 1; k <= T; ++k) {
            p.k = k;
            if (mass) bt_forward<IO, D, RB, false, true><<<grid, kThreads, 0, st>>>(p);
            else bt_forward<IO, D, RB, false, false><<<grid, kThreads, 0, st>>>(p);
        }
        p.k = T;       // the contractions, with g^{T-1}
        if (mass) bt_forward<IO, D, RB, true, true><<<grid, kThreads, 0, st>>>(p);
        else bt_forward<IO, D, RB, true, false><<<grid, kThreads, 0, st>>>(p);
    }
    {
        const int mid_blocks = (int)((size_t)p.G * 64 * D / 1024);     // four columns per thread
        // (a pair with a single workgroup has written its Gram matrices in place: nothing to reduce)
        const size_t total = p.chunks > 1 ? (size_t)T * pairs * R * R : 0;
        bt_mid_gram<D><<<(unsigned)(mid_blocks + (total + 255) / 256), 256, 0, st>>>(p, R, total, mid_blocks);
    }
    bt_glue<IO, D, RB><<<grid, kThreads, 0, st>>>(p);
    if (R == 32) {
        if (T <= 16) bt_recursion<16, 32><<<pairs, 256, 0, st>>>(p);
        else bt_recursion<0, 32><<<pairs, 256, 0, st>>>(p);
    } else {
        if (T <= 16) bt_recursion<16, 64><<<pairs, 256, 0, st>>>(p);
        else bt_recursion<0, 64><<<pairs, 256, 0, st>>>(p);
    }
    const size_t dyn = (size_t)T * 2 * 64 * sizeof(float);
    if (T <= kAllAtOnceIters && !assemble_by_iteration()) {
        bt_assemble_mf<IO, D, RB><<<grid, kThreads, 0, st>>>(p, p.redo);
        bt_assemble<IO, D, RB><<<grid, kThreads, dyn, st>>>(p, T, p.redo);
    } else {
        bt_assemble<IO, D, RB><<<grid, kThreads, dyn, st>>>(p, T, nullptr);
    }
    {
        const int slices = final_slices(s.H * s.r * (D + 1));
        bt_final<<<(unsigned)((s.H * s.r * (D + 1) + kFinalOutputs - 1) / kFinalOutputs), slices * kFinalOutputs, 0, st>>>(p, D, slices / p.chunks, slices % p.chunks);
    }
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

}  // namespace

bool bwd_tiled_supports(const lot_shape& s, int iters)
{
    // the assemble kernel keeps the potentials and column-sum adjoints of all iterations in LDS: 512 bytes
    // per iteration beside up to 107 KB of operands
    return fused_supports(s) && iters <= kMaxTiledIters;
}

BwdTiledWorkspace carve_bwd_tiled(const lot_shape& s, int iters)
{
    BwdTiledWorkspace w{};
    size_t off = 256;      // the status words come first, as in the other workspaces
    auto take = [&](size_t bytes) { size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
    const size_t G = (size_t)s.B * s.H, pairs = 2 * G, T = iters, D = s.d_k;
    const size_t ntiles = ((size_t)s.n + kTileTokens - 1) / kTileTokens;
    const size_t per_wg = (size_t)tiles_per_wg_for(s);
    const size_t chunks = (ntiles + per_wg - 1) / per_wg;
    const size_t R = s.r <= 32 ? 32 : 64;
    w.chunks = (int)chunks;
    w.colacc = take((T + 1) * pairs * 64 * 8);
    w.ghist = take((T + 1) * pairs * 64 * 4);
    w.gram_part = take(T * pairs * chunks * R * R * 4);
    w.gram_full = take(T * pairs * R * R * 4);
    w.u_part = take(pairs * chunks * 64 * D * 4);
    w.yp = take(G * 64 * D * 4);
    w.dyraw = take(G * 64 * D * 4);
    w.sn_part = take(pairs * chunks * 2 * 64 * 4);
    w.dcs = take((T + 1) * pairs * 64 * 4);
    w.rhop = take(pairs * 64 * 4);
    w.db_pair = take(pairs * 64 * 4);
    w.db_glue = take(G * 64 * 4);
    w.dz_part = take(pairs * chunks * 64 * D * 4);
    w.redo = take(pairs * chunks * 4);
    w.cleared = take(pairs * 8);
    w.total = off;
    return w;
}

int run_backward_tiled(const BwdArgs& a)
{
    const lot_shape& s = a.s;
    if (!bwd_tiled_supports(s, a.iters)) return LOT_ERR_PATH;
    const BwdTiledWorkspace L = carve_bwd_tiled(s, a.iters);
    BtParams p{};
    p.Q = a.Q; p.K = a.K; p.V = a.V; p.dO = a.dO; p.Z = a.Z; p.beta = a.beta;
    p.dQ = a.dQ; p.dK = a.dK; p.dV = a.dV; p.dZ = a.dZ; p.dbeta = a.dbeta;
    p.status = (unsigned long long*)a.ws;
    p.nonce = next_nonce();
    p.spin_limit = spin_limit();
    p.sum_hi = reshift_limit();
    p.sum_lo = 1.0f / p.sum_hi;
    p.colacc = (unsigned long long*)(a.ws + L.colacc);
    p.ghist = (float*)(a.ws + L.ghist);
    p.gram_part = (float*)(a.ws + L.gram_part);
    p.gram_full = (float*)(a.ws + L.gram_full);
    p.u_part = (float*)(a.ws + L.u_part);
    p.yp = (float*)(a.ws + L.yp);
    p.dyraw = (float*)(a.ws + L.dyraw);
    p.sn_part = (float*)(a.ws + L.sn_part);
    p.dcs = (float*)(a.ws + L.dcs);
    p.rhop = (float*)(a.ws + L.rhop);
    p.db_pair = (float*)(a.ws + L.db_pair);
    p.db_glue = (float*)(a.ws + L.db_glue);
    p.dz_part = (float*)(a.ws + L.dz_part);
    p.redo = (unsigned*)(a.ws + L.redo);
    p.cleared = (unsigned long long*)(a.ws + L.cleared);
    p.G = s.B * s.H; p.H = s.H; p.B = s.B; p.r = s.r; p.chunks = L.chunks; p.tiles_per_wg = tiles_per_wg_for(s); p.T = a.iters;
    // s.n is the longer side (cross attention); a side with fewer tiles leaves its last workgroups idle
    p.n_side[0] = a.n_q > 0 ? a.n_q : s.n;
    p.n_side[1] = a.n_k > 0 ? a.n_k : s.n;
    for (int sd = 0; sd < 2; ++sd) p.stride_side[sd] = a.n_stride > 0 ? a.n_stride : p.n_side[sd];
    p.mass_side[0] = a.mass_q; p.mass_side[1] = a.mass_k;
    p.eps = a.eps;
    {
        // column sums of a row-normalised kernel are at most n: with 2^(55 - ceil(log2(n + 1))) units per
        // one the sum stays below 2^55, clear of the contributor count in the top byte
        int frac = 55 - (int)std::ceil(std::log2((double)s.n + 1.0));
        p.fx_scale = std::ldexp(1.0f, frac);
        p.fx_unscale = std::ldexp(1.0f, -frac);
    }
    const bool bf16 = s.io_dtype == LOT_BF16;
    const int D = s.d_k, RB = s.r <= 32 ? 1 : 2;
    if (bf16) {
        if (D == 64) return RB == 2 ? launch_all<uint16_t, 64, 2>(a, p) : launch_all<uint16_t, 64, 1>(a, p);
        return RB == 2 ? launch_all<uint16_t, 32, 2>(a, p) : launch_all<uint16_t, 32, 1>(a, p);
    }
    if (D == 64) return RB == 2 ? launch_all<float, 64, 2>(a, p) : launch_all<float, 64, 1>(a, p);
    return RB == 2 ? launch_all<float, 32, 2>(a, p) : launch_all<float, 32, 1>(a, p);
}

}  // namespace lot
